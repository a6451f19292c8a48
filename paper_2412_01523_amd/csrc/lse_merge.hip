// Merge of two partial attentions of the same queries over disjoint key sets (context parallelism,
// paper Sec. 2.1.3: attention is computed chunk by chunk while key/value chunks travel round the
// ring).  With the parts' log-sum-exps la, lb the softmax over the union of the keys is
//     LSE = log(exp(la) + exp(lb)),   O = exp(la - LSE) O_a + exp(lb - LSE) O_b,
// a part with LSE = -inf (it saw no key) counting nothing.  Element-wise, bound by HBM bandwidth:
// one thread per 16-byte piece of an output row, rows of one head walked in token order so that the
// log-sum-exp reads ([H, T]) are contiguous too.
#include "attn_common.h"

namespace flexsp {
namespace {

__global__ __launch_bounds__(256) void lse_merge_kernel(const uint16_t *oa, const float *la, const uint16_t *ob,
                                                        const float *lb, uint16_t *oo, float *lo, int T, int H, int CH,
                                                        int32_t oa_st, int32_t oa_sh, int32_t ob_st, int32_t ob_sh,
                                                        int32_t oo_st, int32_t oo_sh, uint32_t total)
{
    const uint32_t idx = blockIdx.x * 256u + threadIdx.x;
    if (idx >= total) return;
    const int c = (int)(idx % (uint32_t)CH);
    const uint32_t row = idx / (uint32_t)CH;  // = h * T + t
    const int t = (int)(row % (uint32_t)T), h = (int)(row / (uint32_t)T);
    const float a = la[row], b = lb[row];
    const float m = fmaxf(a, b);
    float wa = 0.f, wb = 0.f, lse = -INFINITY;
    if (m > -INFINITY) {
        const float ea = __expf(a - m), eb = __expf(b - m);  // exp(-inf) = 0 for the part without keys
        const float inv = 1.0f / (ea + eb);
        wa = ea * inv;
        wb = eb * inv;
        lse = m + __logf(ea + eb);
    }
    const u32x4 xa = *(const u32x4 *)(oa + (int64_t)t * oa_st + (int64_t)h * oa_sh + c * 8);
    const u32x4 xb = *(const u32x4 *)(ob + (int64_t)t * ob_st + (int64_t)h * ob_sh + c * 8);
    u32x4 y;
#pragma unroll
    for (int i = 0; i < 4; i++) {
        const uint32_t ua = xa[i], ub = xb[i];
        // a weight of exactly 0 must silence its part even if that part holds non-finite rubbish
        const float lo_ = (wa > 0.f ? wa * bf16_lo(ua) : 0.f) + (wb > 0.f ? wb * bf16_lo(ub) : 0.f);
        const float hi_ = (wa > 0.f ? wa * bf16_hi(ua) : 0.f) + (wb > 0.f ? wb * bf16_hi(ub) : 0.f);
        y[i] = pack_bf16x2(lo_, hi_);
    }
    *(u32x4 *)(oo + (int64_t)t * oo_st + (int64_t)h * oo_sh + c * 8) = y;
    if (c == 0) lo[row] = lse;
}

// The same with the running result kept in fp32 (folding many parts into a bf16 result rounds it once
// per fold): acc <- merge(acc, b) in place, and, if `ob16` is given, the merged rows rounded to bf16.
__global__ __launch_bounds__(256) void lse_merge_acc_kernel(float *oacc, float *lacc, const uint16_t *ob, const float *lb,
                                                            uint16_t *ob16, int T, int H, int CH, int32_t oa_st,
                                                            int32_t oa_sh, int32_t ob_st, int32_t ob_sh, int32_t o16_st,
                                                            int32_t o16_sh, uint32_t total)
{
    const uint32_t idx = blockIdx.x * 256u + threadIdx.x;
    if (idx >= total) return;
    const int c = (int)(idx % (uint32_t)CH);
    const uint32_t row = idx / (uint32_t)CH;  // = h * T + t
    const int t = (int)(row % (uint32_t)T), h = (int)(row / (uint32_t)T);
    const float a = lacc[row], b = lb[row];
    const float m = fmaxf(a, b);
    float wa = 0.f, wb = 0.f, lse = -INFINITY;
    if (m > -INFINITY) {
        const float ea = __expf(a - m), eb = __expf(b - m);
        const float inv = 1.0f / (ea + eb);
        wa = ea * inv;
        wb = eb * inv;
        lse = m + __logf(ea + eb);
    }
    float *pa = oacc + (int64_t)t * oa_st + (int64_t)h * oa_sh + c * 8;
    const f32x4 a0 = *(const f32x4 *)pa, a1 = *(const f32x4 *)(pa + 4);
    const u32x4 xb = *(const u32x4 *)(ob + (int64_t)t * ob_st + (int64_t)h * ob_sh + c * 8);
    f32x4 y0, y1;
#pragma unroll
    for (int i = 0; i < 4; i++) {
        const uint32_t ub = xb[i];
        const float alo = i < 2 ? a0[2 * i] : a1[2 * i - 4], ahi = i < 2 ? a0[2 * i + 1] : a1[2 * i - 3];
        // a weight of exactly 0 must silence its part even if that part holds non-finite rubbish
        const float lo_ = (wa > 0.f ? wa * alo : 0.f) + (wb > 0.f ? wb * bf16_lo(ub) : 0.f);
        const float hi_ = (wa > 0.f ? wa * ahi : 0.f) + (wb > 0.f ? wb * bf16_hi(ub) : 0.f);
        if (i < 2) {
            y0[2 * i] = lo_;
            y0[2 * i + 1] = hi_;
        } else {
            y1[2 * i - 4] = lo_;
            y1[2 * i - 3] = hi_;
        }
    }
    *(f32x4 *)pa = y0;
    *(f32x4 *)(pa + 4) = y1;
    if (ob16) {
        u32x4 z;
        z[0] = pack_bf16x2(y0[0], y0[1]);
        z[1] = pack_bf16x2(y0[2], y0[3]);
        z[2] = pack_bf16x2(y1[0], y1[1]);
        z[3] = pack_bf16x2(y1[2], y1[3]);
        *(u32x4 *)(ob16 + (int64_t)t * o16_st + (int64_t)h * o16_sh + c * 8) = z;
    }
    if (c == 0) lacc[row] = lse;
}

}  // namespace

hipError_t launch_lse_merge_acc(float *oacc, float *lacc, const uint16_t *ob, const float *lb, uint16_t *ob16, int64_t T,
                                int H, int D, int32_t oa_st, int32_t oa_sh, int32_t ob_st, int32_t ob_sh, int32_t o16_st,
                                int32_t o16_sh, hipStream_t s)
{
    const int CH = D / 8;
    const uint32_t total = (uint32_t)(T * H * CH);
    hipLaunchKernelGGL(lse_merge_acc_kernel, dim3((total + 255) / 256), dim3(256), 0, s, oacc, lacc, ob, lb, ob16, (int)T, H,
                       CH, oa_st, oa_sh, ob_st, ob_sh, o16_st, o16_sh, total);
    return hipGetLastError();
}

hipError_t launch_lse_merge(const uint16_t *oa, const float *la, const uint16_t *ob, const float *lb, uint16_t *oo,
                            float *lo, int64_t T, int H, int D, int32_t oa_st, int32_t oa_sh, int32_t ob_st,
                            int32_t ob_sh, int32_t oo_st, int32_t oo_sh, hipStream_t s)
{
    const int CH = D / 8;
    const uint32_t total = (uint32_t)(T * H * CH);
    hipLaunchKernelGGL(lse_merge_kernel, dim3((total + 255) / 256), dim3(256), 0, s, oa, la, ob, lb, oo, lo, (int)T, H, CH,
                       oa_st, oa_sh, ob_st, ob_sh, oo_st, oo_sh, total);
    return hipGetLastError();
}

}  // namespace flexsp
