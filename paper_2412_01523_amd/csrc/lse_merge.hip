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

}  // namespace

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
