// Forward of packed causal attention (paper Sec. 2.1.2, Eq. 3, evaluated per sequence of
// the packed stream, Sec. 2.2.2) for gfx950.
//
// One work item = 128 query rows of one (sequence, head).  A workgroup of 4 wavefronts
// takes items from the longest-first queues until they are empty.  Each wavefront owns 32
// query rows and keeps their Q in registers.  Key/value tiles of 64 rows are staged in LDS.
// The score block is computed TRANSPOSED, S^T = K Q^T, so that in the 32x32 accumulator a
// lane holds one query (its column) and 16 keys: the row-wise softmax is a reduction over a
// lane's own registers plus one exchange with the lane 32 away, and the exponentiated block,
// rounded to bf16, is directly the B operand of O^T += V^T P^T.  V^T fragments come from
// the row-major V tile through the LDS transpose read.
#include "attn_common.h"

namespace flexsp {
namespace {

template <int D>
struct FwdCfg {
    static constexpr int KS = D / 16;         // k steps of the score product
    static constexpr int DB = D / 32;         // 32-wide blocks of the head dim
    static constexpr int KSTRIDE = D + 8;     // K tile row stride (elements): natural reads
    static constexpr int VSTRIDE = D + 32;    // V tile row stride: transpose reads
    static constexpr int CH = D / 8;          // 16-byte chunks per row
    static constexpr int NLD = kFwdBk * CH / kThreads;  // chunks per thread per tile
};

template <int D>
__global__ __launch_bounds__(kThreads, 2) void attn_fwd_kernel(const AttnArgs a)
{
    typedef FwdCfg<D> C;
    __shared__ __attribute__((aligned(16))) uint16_t sK[kFwdBk * C::KSTRIDE];
    __shared__ __attribute__((aligned(16))) uint16_t sV[kFwdBk * C::VSTRIDE];
    __shared__ int s_item;

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int r = lane & 31, hl = lane >> 5;
    int cursor = 0;

    for (;;) {
        if (tid == 0) s_item = queue_fetch(a.pq, cursor);
        __syncthreads();
        const int item = s_item;
        if (item < 0) break;
        const flexsp_item it = a.pq.items[item];
        const int s = it.seq_len, h = it.head, g = h / a.G;
        const int q0 = it.tile * kFwdBq;
        const int64_t tok0 = it.seq_start;
        const int kv_end = a.causal ? min(s, q0 + kFwdBq) : s;  // keys this item needs
        const int ntiles = (kv_end + kFwdBk - 1) / kFwdBk;

        // ---- Q fragments (B operand: column = query row, k = head dim), kept in registers
        const int qrow = q0 + wave * 32 + r;  // row inside the sequence
        bf16x8 qf[C::KS];
        {
            const bool ok = qrow < s;
            const uint16_t *qp = a.q + (tok0 + (ok ? qrow : 0)) * a.q_st + (int64_t)h * a.q_sh + 8 * hl;
#pragma unroll
            for (int ks = 0; ks < C::KS; ks++) {
                Frag8 f;
                f.u = ok ? *(const u32x4 *)(qp + 16 * ks) : u32x4{0, 0, 0, 0};
                qf[ks] = f.v;
            }
        }

        f32x16 oacc[C::DB];
#pragma unroll
        for (int db = 0; db < C::DB; db++)
#pragma unroll
            for (int i = 0; i < 16; i++) oacc[db][i] = 0.f;
        float m_run = -INFINITY, l_run = 0.f;

        const uint16_t *kbase = a.k + tok0 * a.k_st + (int64_t)g * a.k_sh;
        const uint16_t *vbase = a.v + tok0 * a.v_st + (int64_t)g * a.v_sh;

        // register staging of the next K/V tile
        u32x4 kreg[C::NLD], vreg[C::NLD];
        auto gload = [&](int kv0) {
#pragma unroll
            for (int n = 0; n < C::NLD; n++) {
                int c = n * kThreads + tid;
                int row = c / C::CH, col = (c % C::CH) * 8;
                bool ok = kv0 + row < s;
                kreg[n] = ok ? *(const u32x4 *)(kbase + (int64_t)(kv0 + row) * a.k_st + col) : u32x4{0, 0, 0, 0};
                vreg[n] = ok ? *(const u32x4 *)(vbase + (int64_t)(kv0 + row) * a.v_st + col) : u32x4{0, 0, 0, 0};
            }
        };
        auto lstore = [&]() {
#pragma unroll
            for (int n = 0; n < C::NLD; n++) {
                int c = n * kThreads + tid;
                int row = c / C::CH, col = (c % C::CH) * 8;
                *(u32x4 *)(sK + row * C::KSTRIDE + col) = kreg[n];
                *(u32x4 *)(sV + row * C::VSTRIDE + col) = vreg[n];
            }
        };

        gload(0);
        const int wq_lo = q0 + wave * 32;  // smallest query row of this wavefront
        for (int t = 0; t < ntiles; t++) {
            const int kv0 = t * kFwdBk;
            __syncthreads();  // everyone is done reading the previous tile
            lstore();
            __syncthreads();
            if (t + 1 < ntiles) gload(kv0 + kFwdBk);

            // wavefronts whose rows all lie above this tile (causal) have nothing to do
            if (a.causal && kv0 > wq_lo + 31) continue;

            // ---- S^T = K Q^T : two 32-key blocks
            f32x16 sacc[2];
#pragma unroll
            for (int kb = 0; kb < 2; kb++)
#pragma unroll
                for (int i = 0; i < 16; i++) sacc[kb][i] = 0.f;
#pragma unroll
            for (int ks = 0; ks < C::KS; ks++) {
#pragma unroll
                for (int kb = 0; kb < 2; kb++) {
                    bf16x8 kf = lds_frag(sK, C::KSTRIDE, kb * 32, ks * 16, lane);
                    sacc[kb] = mfma32(kf, qf[ks], sacc[kb]);
                }
            }
            // ---- mask (only tiles that touch the diagonal or the end of the sequence)
            const bool need_mask = a.causal ? (kv0 + kFwdBk - 1 > wq_lo) : (kv0 + kFwdBk > s);
            if (need_mask) {
                const int lim = a.causal ? qrow : s - 1;  // largest visible key
#pragma unroll
                for (int kb = 0; kb < 2; kb++)
#pragma unroll
                    for (int i = 0; i < 16; i++) {
                        int kv = kv0 + kb * 32 + 8 * (i >> 2) + 4 * hl + (i & 3);
                        if (kv > lim) sacc[kb][i] = -INFINITY;
                    }
            }
            // ---- online softmax (one query per lane, 32 of its keys here, 32 in lane^32)
            float mx = sacc[0][0];
#pragma unroll
            for (int kb = 0; kb < 2; kb++)
#pragma unroll
                for (int i = 0; i < 16; i++) mx = fmaxf(mx, sacc[kb][i]);
            mx = fmaxf(mx, __shfl_xor(mx, 32));
            const float m_new = fmaxf(m_run, mx);
            const float m_use = (m_new == -INFINITY) ? 0.f : m_new;
            const float alpha = __builtin_amdgcn_exp2f((m_run - m_use) * a.scale_l2);
            const float moff = m_use * a.scale_l2;
            float psum = 0.f;
            uint32_t pk[2][8];
#pragma unroll
            for (int kb = 0; kb < 2; kb++)
#pragma unroll
                for (int i = 0; i < 16; i += 2) {
                    float p0 = __builtin_amdgcn_exp2f(__builtin_fmaf(sacc[kb][i], a.scale_l2, -moff));
                    float p1 = __builtin_amdgcn_exp2f(__builtin_fmaf(sacc[kb][i + 1], a.scale_l2, -moff));
                    psum += p0 + p1;
                    pk[kb][i >> 1] = pack_bf16x2(p0, p1);
                }
            l_run = l_run * alpha + psum;
            m_run = m_new;
#pragma unroll
            for (int db = 0; db < C::DB; db++)
#pragma unroll
                for (int i = 0; i < 16; i++) oacc[db][i] *= alpha;
            // ---- O^T += V^T P^T
#pragma unroll
            for (int kb = 0; kb < 2; kb++)
#pragma unroll
                for (int hf = 0; hf < 2; hf++) {
                    Frag8 pf;
                    pf.u = u32x4{pk[kb][4 * hf], pk[kb][4 * hf + 1], pk[kb][4 * hf + 2], pk[kb][4 * hf + 3]};
#pragma unroll
                    for (int db = 0; db < C::DB; db++) {
                        bf16x8 vf = lds_frag_tr(sV, C::VSTRIDE, kb * 32 + hf * 16, db * 32, lane);
                        oacc[db] = mfma32(vf, pf.v, oacc[db]);
                    }
                }
        }

        // ---- epilogue: normalise, write O (bf16) and LSE (natural log)
        const float l_tot = l_run + __shfl_xor(l_run, 32);
        if (qrow < s) {
            const float inv = 1.0f / l_tot;
            uint16_t *op = a.out_o + (tok0 + qrow) * a.o_st + (int64_t)h * a.o_sh;
#pragma unroll
            for (int db = 0; db < C::DB; db++)
#pragma unroll
                for (int i4 = 0; i4 < 4; i4++) {
                    u32x2 w;
                    w[0] = pack_bf16x2(oacc[db][4 * i4] * inv, oacc[db][4 * i4 + 1] * inv);
                    w[1] = pack_bf16x2(oacc[db][4 * i4 + 2] * inv, oacc[db][4 * i4 + 3] * inv);
                    *(u32x2 *)(op + db * 32 + 8 * i4 + 4 * hl) = w;
                }
            if (hl == 0) a.lse_out[(int64_t)h * a.T + tok0 + qrow] = m_run * a.scale + __logf(l_tot);
        }
        __syncthreads();  // s_item and the LDS tiles are reused by the next item
    }
    if (tid == 0) queue_retire(a.pq);
}

}  // namespace

hipError_t launch_attn_fwd(const AttnArgs &a, int D, int grid, hipStream_t s)
{
    if (D == 128)
        hipLaunchKernelGGL(attn_fwd_kernel<128>, dim3(grid), dim3(kThreads), 0, s, a);
    else
        hipLaunchKernelGGL(attn_fwd_kernel<64>, dim3(grid), dim3(kThreads), 0, s, a);
    return hipGetLastError();
}

}  // namespace flexsp
