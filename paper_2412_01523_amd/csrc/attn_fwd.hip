// Forward of packed causal attention (paper Sec. 2.1.2, Eq. 3, evaluated per sequence of
// the packed stream, Sec. 2.2.2) for gfx950.
//
// One work item = 128 query rows of one (sequence, head).  A workgroup of 4 wavefronts
// takes items from the longest-first queues until they are empty.  Each wavefront owns 32
// query rows and keeps their Q in registers.  Key/value tiles of 64 rows go straight from
// global memory into swizzled LDS tiles (no staging registers), double-buffered: the next
// tile is in flight while this one is consumed, one barrier per tile.
// The score block is computed TRANSPOSED, S^T = K Q^T, so that in the 32x32 accumulator a
// lane holds one query (its column) and 16 keys: the row-wise softmax is a reduction over a
// lane's own registers plus one exchange with the lane 32 away, and the exponentiated block,
// rounded to bf16, is directly the B operand of O^T += V^T P^T.  V^T fragments come from
// the row-major V tile through the LDS transpose read.  The running output is rescaled only
// when some row's maximum actually grew.
#include <type_traits>

#include "attn_common.h"

namespace flexsp {
namespace {

template <int D>
__global__ __launch_bounds__(kThreads, 2) void attn_fwd_kernel(const AttnArgs a)
{
    typedef LdsTile<D> L;
    constexpr int KS = D / 16;                  // k steps of the score product
    constexpr int DB = D / 32;                  // 32-wide blocks of the head dim
    constexpr int TILE = kFwdBk * L::ROWB;      // bytes of one 64-row tile
    // [buffer][K | V]
    __shared__ __attribute__((aligned(1024))) char smem[4 * TILE];

    const int tid = threadIdx.x;
    const int lane0 = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    LaneOffsets<D> lo;
    lo.init(lane0);
    ItemDealer deal;
    deal.init(a.pq);

    for (int item = deal.next(); item >= 0; item = deal.next()) {
        const flexsp_item it = load_item(a.pq.items, item);
        // opaque per-item copy of the lane id: per-lane address arithmetic of an item stays inside
        // the item instead of being hoisted out of this loop into long-lived registers
        int lane = lane0;
        asm volatile("" : "+v"(lane));
        const int r = lane & 31, hl = lane >> 5;
        const int s = it.seq_len, h = it.head, g = h / a.G;
        const int q0 = it.tile * kFwdBq;
        const int64_t tok0 = it.seq_start;
        const int kv_end = a.causal ? min(s, q0 + kFwdBq) : s;  // keys this item needs
        const int ntiles = (kv_end + kFwdBk - 1) / kFwdBk;
        const uint16_t *kbase = a.k + tok0 * a.k_st + (int64_t)g * a.k_sh;
        const uint16_t *vbase = a.v + tok0 * a.v_st + (int64_t)g * a.v_sh;

        const uint32_t goffk = tile_goff<D>(a.k_st, wave, lane), goffv = tile_goff<D>(a.v_st, wave, lane);
        auto prefetch = [&](int t, int buf) {
            char *dk = smem + buf * 2 * TILE, *dv = dk + TILE;
            if ((t + 1) * kFwdBk <= s) {  // whole tile inside the sequence
                load_tile_async_fast<D, kFwdBk>(dk, kbase + (int64_t)t * kFwdBk * a.k_st, a.k_st, goffk, wave);
                load_tile_async_fast<D, kFwdBk>(dv, vbase + (int64_t)t * kFwdBk * a.v_st, a.v_st, goffv, wave);
            } else {
                load_tile_async<D, kFwdBk>(dk, kbase, a.k_st, t * kFwdBk, s - 1, wave, lane);
                load_tile_async<D, kFwdBk>(dv, vbase, a.v_st, t * kFwdBk, s - 1, wave, lane);
            }
        };
        prefetch(0, 0);

        // ---- Q fragments (B operand: column = query row, k = head dim), kept in registers
        const int qrow = q0 + wave * 32 + r;  // row inside the sequence
        const int wq_lo = q0 + wave * 32;     // smallest query row of this wavefront
        bf16x8 qf[KS];
        {
            const bool ok = qrow < s;
            const uint16_t *qp = a.q + (tok0 + (ok ? qrow : 0)) * a.q_st + (int64_t)h * a.q_sh + 8 * hl;
#pragma unroll
            for (int ks = 0; ks < KS; ks++) {
                Frag8 f;
                f.u = ok ? *(const u32x4 *)(qp + 16 * ks) : u32x4{0, 0, 0, 0};
                qf[ks] = f.v;
            }
        }

        f32x16 oacc[DB];
#pragma unroll
        for (int db = 0; db < DB; db++)
#pragma unroll
            for (int i = 0; i < 16; i++) oacc[db][i] = 0.f;
        float m_run = -INFINITY, l_run = 0.f, moff = 0.f;

        auto step = [&](auto bufc, int t) {
            constexpr int BUF = decltype(bufc)::value;
            const char *sK = smem + BUF * 2 * TILE;
            const char *sV = sK + TILE;
            const int kv0 = t * kFwdBk;
            lo.pin();
            wait_vmem();      // this wavefront's share of tile t has landed
            __syncthreads();  // everybody's has, and everybody is done with tile t-1
            if (t + 1 < ntiles) prefetch(t + 1, BUF ^ 1);
            // wavefronts whose rows all lie above this tile (causal) have nothing to do
            if (a.causal && kv0 > wq_lo + 31) return;

            // ---- S^T = K Q^T : two 32-key blocks
            f32x16 sacc[2];
#pragma unroll
            for (int kb = 0; kb < 2; kb++)
#pragma unroll
                for (int i = 0; i < 16; i++) sacc[kb][i] = 0.f;
#pragma unroll
            for (int ks = 0; ks < KS; ks++)
#pragma unroll
                for (int kb = 0; kb < 2; kb++)
                    sacc[kb] = mfma32(lds_nat(sK, kb * 32 * L::ROWB + lo.nat[ks]), qf[ks], sacc[kb]);
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
            float mx = fmaxf(sacc[0][0], sacc[1][0]);
#pragma unroll
            for (int i = 1; i < 16; i++) mx = fmaxf(mx, fmaxf(sacc[0][i], sacc[1][i]));
            mx = halves_max(mx);
            if (__builtin_amdgcn_ballot_w64(mx > m_run) != 0) {  // some row's maximum grew
                const float m_new = fmaxf(m_run, mx);
                const float alpha = __builtin_amdgcn_exp2f((m_run - m_new) * a.scale_l2);
                m_run = m_new;
                moff = m_new * a.scale_l2;
                l_run *= alpha;
#pragma unroll
                for (int db = 0; db < DB; db++)
#pragma unroll
                    for (int i = 0; i < 16; i++) oacc[db][i] *= alpha;
            }
            float psum = 0.f;
            uint32_t pk[2][8];
#pragma unroll
            for (int kb = 0; kb < 2; kb++)
#pragma unroll
                for (int i = 0; i < 16; i += 2) {
                    float p0 = __builtin_amdgcn_exp2f(__builtin_fmaf(sacc[kb][i], a.scale_l2, -moff));
                    float p1 = __builtin_amdgcn_exp2f(__builtin_fmaf(sacc[kb][i + 1], a.scale_l2, -moff));
                    psum += p0 + p1;  // fp32: the log-sum-exp feeds the backward recomputation
                    pk[kb][i >> 1] = pack_bf16x2(p0, p1);
                }
            l_run += psum;
            // ---- O^T += V^T P^T
#pragma unroll
            for (int kb = 0; kb < 2; kb++)
#pragma unroll
                for (int hf = 0; hf < 2; hf++) {
                    Frag8 pf;
                    pf.u = u32x4{pk[kb][4 * hf], pk[kb][4 * hf + 1], pk[kb][4 * hf + 2], pk[kb][4 * hf + 3]};
                    const int rowoff = (kb * 32 + hf * 16) * L::ROWB;
#pragma unroll
                    for (int db = 0; db < DB; db++)
                        oacc[db] = mfma32(lds_tr(sV, rowoff + lo.tr[db][0], rowoff + lo.tr[db][1]), pf.v, oacc[db]);
                }
        };

        for (int t = 0; t < ntiles; t += 2) {
            step(std::integral_constant<int, 0>{}, t);
            if (t + 1 < ntiles) step(std::integral_constant<int, 1>{}, t + 1);
        }

        // ---- epilogue: normalise, write O (bf16) and LSE (natural log)
        const float l_tot = halves_sum(l_run);
        if (qrow < s && hl == 0) a.lse_out[(int64_t)h * a.T + tok0 + qrow] = m_run * a.scale + __logf(l_tot);
        // O goes out through the tile buffer the last step did not use (every wavefront is past the
        // barrier of the last step, so nobody reads that buffer any more)
        if (wq_lo < s)
            store_rowT_bf16_lds<DB>(smem + (ntiles & 1) * 2 * TILE + wave * (32 * L::ROWB),
                                    a.out_o + (tok0 + wq_lo) * a.o_st + (int64_t)h * a.o_sh, a.o_st,
                                    min(32, s - wq_lo), oacc, 1.0f / l_tot, lane);
        barrier_lds_only();  // the LDS buffers are reused by the next item
    }
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
