// Forward of packed causal attention (paper Sec. 2.1.2, Eq. 3, evaluated per sequence of
// the packed stream, Sec. 2.2.2) for gfx950.
//
// One work item = 128 query rows of one (sequence, head).  A workgroup of 4 wavefronts
// takes items from the longest-first queues until they are empty.  Each wavefront owns 32
// query rows and keeps their Q in registers.  Key/value tiles of 64 rows go straight from
// global memory into swizzled LDS tiles (no staging registers), double-buffered, one barrier
// per tile.
//
// The score block is computed TRANSPOSED, S^T = K Q^T, so that in the 32x32 accumulator a
// lane holds one query (its column) and 16 keys: the row-wise softmax is a reduction over a
// lane's own registers plus one exchange with the lane 32 away, and the exponentiated block,
// rounded to bf16, is directly the B operand of O^T += V^T P^T.  V^T fragments come from
// the row-major V tile through the LDS transpose read.  The running output is rescaled only
// when some row's maximum actually grew.
//
// A wavefront walks the keys in blocks of 32 (two per tile) as a software pipeline: iteration
// c issues the matrix instructions of S(c+1) and of O += P(c-1) V(c-1) and, between them, the
// softmax arithmetic of block c, so that the matrix pipe and the vector pipe of the SIMD work
// at the same time inside one wavefront (the file is compiled with the compiler's
// pre-allocation schedulers off: the order written here is the order executed).  The K tiles
// therefore run one tile ahead of the V tiles: between the barriers of tile t and t+1 the
// wavefronts read K tile t+1 and V tile t while K tile t+2 and V tile t+1 are in flight.
#include <type_traits>

#include "attn_common.h"

namespace flexsp {
namespace {

template <int V>
using ic = std::integral_constant<int, V>;

// SHARD = true is the variant for one shard of the keys (context parallelism): a work item then
// names separate query and key ranges and an offset `shift` between their positions, key j is
// visible to query row i iff j <= i + shift (when causal), rows may see no key at all (O = 0,
// LSE = -inf), and up to three 32-key blocks of a wavefront need masking (the diagonal crosses two
// when shift is not a multiple of 32, plus the ragged end of the shard).
template <int D, bool SHARD>
__global__ __launch_bounds__(kThreads, 2) void attn_fwd_kernel(const AttnArgs a)
{
    typedef LdsTile<D> L;
    constexpr int KS = D / 16;                  // k steps of the score product
    constexpr int DB = D / 32;                  // 32-wide blocks of the head dim
    constexpr int TILE = kFwdBk * L::ROWB;      // bytes of one 64-row tile
    constexpr int NCP = 2 * kFwdBk * L::CH / kThreads;  // copy instructions per wavefront for a K and a V tile
    constexpr int NSLOT = KS + 2 * DB;          // matrix instructions of one pipeline iteration
    static_assert(NSLOT == 2 * NCP, "one copy instruction per two matrix instructions");
    // [K buffer 0 | K buffer 1 | V buffer 0 | V buffer 1]
    __shared__ __attribute__((aligned(1024))) char smem[4 * TILE];

    const int tid = threadIdx.x;
    const int lane0 = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    LaneOffsets<D> lo;
    lo.init(lane0);
    __shared__ int deal_word, split_word;
    ItemDealer deal;

    int item = deal.first(a.pq, &deal_word, wave, lane0);
    for (; item >= 0; item = deal.advance()) {
        // s: query rows of the sequence; sk: its keys; tok0 / ktok0: their first rows in q / k, v
        int s, sk, shift, h, q0;
        int64_t tok0, ktok0;
        int part = 0, nparts = 1, slot = -1, t_lo = 0, t_hi = 0;  // (see flexsp_item): the item walks key tiles t_lo .. t_hi-1
        if constexpr (SHARD) {
            const flexsp_shard_item it = load_shard_item((const flexsp_shard_item *)a.pq.items, item);
            s = it.q_len; sk = it.k_len; shift = it.shift; h = it.head_parts & 0xffff; q0 = it.tile * kFwdBq;
            tok0 = it.q_start; ktok0 = it.k_start;
            // (a part of a cut tile comes with its own key range and shift: nothing else differs)
            part = (it.head_parts >> 16) & 0xff; nparts = it.head_parts >> 24; slot = it.slot;
        } else {
            const flexsp_item it = load_item(a.pq.items, item);
            s = it.seq_len; sk = s; shift = 0; h = it.head; q0 = it.tile * kFwdBq;
            tok0 = it.seq_start; ktok0 = tok0;
            part = it.parts >> 16; nparts = it.parts & 0xffff; slot = it.slot;
            t_lo = it.step_begin; t_hi = it.step_end;
        }
        // opaque per-item copy of the lane id: per-lane address arithmetic of an item stays inside
        // the item instead of being hoisted out of this loop into long-lived registers
        int lane = lane0;
        asm volatile("" : "+v"(lane));
        const int r = lane & 31, hl = lane >> 5;
        const int g = h / a.G;
        // keys this item needs
        int kv_end = SHARD ? (a.causal ? max(0, min(sk, q0 + kFwdBq + shift)) : sk)
                           : (a.causal ? min(s, q0 + kFwdBq) : s);
        // The item walks key tiles t_lo .. t_hi-1 (all of them unless the tile was cut).  From here on keys are counted
        // from the part's first one (koff keys are skipped: a multiple of the tile size, so blocks
        // stay aligned and still at most one block per wavefront needs masking); a wavefront whose
        // rows see none of the part's keys (the part after the diagonal of the tile's upper rows) ends
        // with maximum -inf and sum 0, which the merge below weighs with zero.
        int koff = 0;
        if constexpr (!SHARD) {
            koff = t_lo * kFwdBk;
            kv_end = min(kv_end, t_hi * kFwdBk) - koff;
            sk = s - koff;
            ktok0 += koff;
        }
        if constexpr (SHARD) {
            if (kv_end <= 0) {
                // no row of this item sees a key of the shard: O = 0, LSE = -inf (the neutral element
                // of the merge); deal.advance() holds the barrier every item ends with
                if (a.dq) {
                    // folding into a running result: it stays as it is; only its bf16 copy, if asked for, is written
                    if (a.out_o) {
                        for (int idx = tid; idx < kFwdBq * L::CH; idx += kThreads) {
                            const int row = q0 + idx / L::CH;
                            if (row >= s) continue;
                            const bool live = a.delta_out[(int64_t)h * a.T + tok0 + row] > -INFINITY;
                            const float *src = (const float *)a.dq + (tok0 + row) * a.dq_st + (int64_t)h * a.dq_sh + (idx % L::CH) * 8;
                            const f32x4 x0 = *(const f32x4 *)src, x1 = *(const f32x4 *)(src + 4);
                            u32x4 y = {pack_bf16x2(x0[0], x0[1]), pack_bf16x2(x0[2], x0[3]), pack_bf16x2(x1[0], x1[1]),
                                       pack_bf16x2(x1[2], x1[3])};
                            if (!live) y = u32x4{0, 0, 0, 0};
                            *(u32x4 *)(a.out_o + (tok0 + row) * a.o_st + (int64_t)h * a.o_sh + (idx % L::CH) * 8) = y;
                        }
                    }
                    deal.prefetch();
                    continue;
                }
                for (int idx = tid; idx < kFwdBq * L::CH; idx += kThreads) {
                    const int row = q0 + idx / L::CH;
                    if (row < s)
                        *(u32x4 *)(a.out_o + (tok0 + row) * a.o_st + (int64_t)h * a.o_sh + (idx % L::CH) * 8) =
                            u32x4{0, 0, 0, 0};
                }
                if (tid < kFwdBq && q0 + tid < s) a.lse_out[(int64_t)h * a.T + tok0 + q0 + tid] = -INFINITY;
                deal.prefetch();
                continue;
            }
        }
        const int ntiles = (kv_end + kFwdBk - 1) / kFwdBk;
        const uint16_t *kbase = a.k + ktok0 * a.k_st + (int64_t)g * a.k_sh;
        const uint16_t *vbase = a.v + ktok0 * a.v_st + (int64_t)g * a.v_sh;

        const uint32_t goffk = tile_goff<D>(a.k_st, wave, lane), goffv = tile_goff<D>(a.v_st, wave, lane);
        // whole-tile copies (all of this wavefront's copy instructions back to back)
        auto prefetch_k = [&](int t, int buf) {
            char *dst = smem + buf * TILE;
            if ((t + 1) * kFwdBk <= sk)  // whole tile inside the sequence
                load_tile_async_fast<D, kFwdBk>(dst, kbase + (int64_t)t * kFwdBk * a.k_st, a.k_st, goffk, wave);
            else
                load_tile_async<D, kFwdBk>(dst, kbase, a.k_st, t * kFwdBk, sk - 1, wave, lane);
        };
        auto prefetch_v = [&](int t, int buf) {
            char *dst = smem + (2 + buf) * TILE;
            if ((t + 1) * kFwdBk <= sk)
                load_tile_async_fast<D, kFwdBk>(dst, vbase + (int64_t)t * kFwdBk * a.v_st, a.v_st, goffv, wave);
            else
                load_tile_async<D, kFwdBk>(dst, vbase, a.v_st, t * kFwdBk, sk - 1, wave, lane);
        };
        prefetch_k(0, 0);

        // ---- Q fragments (B operand: column = query row, k = head dim), kept in registers: the rows
        // are requested here and become fragments just before the barrier below
        const int qrow = q0 + wave * 32 + r;  // row inside the sequence
        const int wq_lo = q0 + wave * 32;     // smallest query row of this wavefront
        RowBlock<D> qrows;
        qrows.load(a.q + tok0 * a.q_st + (int64_t)h * a.q_sh, a.q_st, wq_lo, s - 1, lane);
        bf16x8 qf[KS];
        // last 32-key block this wavefront has to look at (-1: none, its rows lie past the sequence)
        int cmax, cmask, lim;
        if constexpr (SHARD) {
            // (>> of a negative number rounds down: a diagonal left of the shard gives a negative block)
            cmax = wq_lo >= s ? -1 : max(-1, a.causal ? min((kv_end - 1) >> 5, (wq_lo + 31 + shift) >> 5) : (kv_end - 1) >> 5);
            cmask = a.causal ? min((wq_lo + shift) >> 5, (sk - 1) >> 5) : ((sk - 1) >> 5);  // FIRST block that needs masking
            lim = a.causal ? min(qrow + shift, sk - 1) : sk - 1;
        } else {
            // (wq_lo - koff is negative for rows that lie before the part's keys: >> rounds down, no block)
            cmax = wq_lo >= s ? -1 : (a.causal ? min((kv_end - 1) >> 5, (wq_lo - koff) >> 5) : (kv_end - 1) >> 5);
            cmask = a.causal ? ((wq_lo - koff) >> 5) : ((sk - 1) >> 5);  // the block that needs masking
            lim = a.causal ? qrow - koff : sk - 1;                        // largest visible key of this lane's row
        }

        f32x16 oacc[DB];
#pragma unroll
        for (int db = 0; db < DB; db++)
#pragma unroll
            for (int i = 0; i < 16; i++) oacc[db][i] = 0.f;
        // (SHARD: a finite floor instead of -inf, because a row may have every key of a block masked:
        // its scores are -inf, and -inf minus a reference of -inf would not be a number)
        float m_run = SHARD ? -1e30f : -INFINITY, l_run = 0.f;
        float psum_max = 0.f;  // largest row sum of a block taken without its maximum (see iter_fast)
        f32x16 sacc[2];     // S of block c in sacc[c & 1]
        uint32_t pk[2][8];  // P of block c (bf16 pairs) in pk[c & 1]

        // ---------------- the three stages of a block, one after the other (pipeline ends) -----
        // S(c) = K(c) Q^T; `sK` points at the block's first row inside its K tile
        auto scores = [&](f32x16 &sa, const char *sK) {
            constexpr int AH = 4;
            bf16x8 kf[KS];
#pragma unroll
            for (int i = 0; i < 16; i++) sa[i] = 0.f;
#pragma unroll
            for (int j = 0; j < AH && j < KS; j++) kf[j] = lds_nat(sK, lo.nat[j]);
#pragma unroll
            for (int j = 0; j < KS; j++) {
                if (j + AH < KS) kf[j + AH] = lds_nat(sK, lo.nat[j + AH]);
                sa = mfma32(kf[j], qf[j], sa);
            }
        };
        // O^T += V(c)^T P(c)^T
        auto pv = [&](const uint32_t (&p)[8], const char *sV) {
            constexpr int AH = 4, N = 2 * DB;
            bf16x8 vf[N];
            auto vread = [&](int j) {
                const int rowoff = (j / DB) * 16 * L::ROWB;
                return lds_tr(sV, rowoff + lo.tr[j % DB][0], rowoff + lo.tr[j % DB][1]);
            };
#pragma unroll
            for (int j = 0; j < AH && j < N; j++) vf[j] = vread(j);
#pragma unroll
            for (int j = 0; j < N; j++) {
                if (j + AH < N) vf[j + AH] = vread(j + AH);
                const int st = j / DB;
                Frag8 pf;
                pf.u = u32x4{p[4 * st], p[4 * st + 1], p[4 * st + 2], p[4 * st + 3]};
                oacc[j % DB] = mfma32(vf[j], pf.v, oacc[j % DB]);
            }
        };
        // Online-softmax bookkeeping shared by both forms of an iteration.
        //   row maximum of a block: own 16 keys, then the other half-wave's
        auto block_max = [&](const f32x16 &sa) {
            float mx = fmaxf(sa[0], sa[1]);
#pragma unroll
            for (int i = 2; i < 16; i += 2) mx = fmaxf(mx, fmaxf(sa[i], sa[i + 1]));
            return halves_max(mx);
        };
        //   the reference value subtracted from a block's scores: the running one, which only moves
        //   when some row's maximum exceeds it by more than 8 in the exponent's units (P then stays
        //   below 2^8: exact in bf16 and fp32 alike, and the final O / l and LSE do not depend on
        //   the reference).  Without the slack the first blocks of every item, where the maxima still
        //   grow a little with each block, would rescale O (64 multiplications) almost every time.
        const float slack = 8.0f / a.scale_l2;
        auto reference = [&](float mx) {
            const bool move = __builtin_amdgcn_ballot_w64(mx > m_run + slack) != 0;
            return move ? fmaxf(m_run, mx) : m_run;
        };
        //   after the iteration's O += P V: rescale if the reference moved, fold in the row sums
        auto finish_block = [&](float m_new, float psum) {
            if (__builtin_amdgcn_ballot_w64(m_new > m_run) != 0) {
                const float alpha = __builtin_amdgcn_exp2f((m_run - m_new) * a.scale_l2);
                l_run *= alpha;
#pragma unroll
                for (int db = 0; db < DB; db++)
#pragma unroll
                    for (int i = 0; i < 16; i++) oacc[db][i] *= alpha;
                m_run = m_new;
            }
            l_run += psum;  // fp32: the log-sum-exp feeds the backward recomputation
        };

        // ---------------- iteration c, general form: any subset of the three stages ------------
        // S(c+1), softmax(c), O += P(c-1) V(c-1), done one after the other.  Used where the pipeline
        // fills and drains and for the masked block.  sK / sV: first row of block c+1 / c-1.
        auto iter_slow = [&](auto cpc, int c, const char *sK, const char *sV) {
            constexpr int CP = decltype(cpc)::value;  // c & 1
            if (c + 1 <= cmax) scores(sacc[CP ^ 1], sK);
            float m_new = m_run, psum = 0.f;
            if (c <= cmax) {
                f32x16 &sa = sacc[CP];
                if (SHARD ? c >= cmask : c == cmask) {
#pragma unroll
                    for (int i = 0; i < 16; i++) {
                        const int kv = c * 32 + 8 * (i >> 2) + 4 * hl + (i & 3);
                        if (kv > lim) sa[i] = -INFINITY;
                    }
                }
                m_new = reference(block_max(sa));
                const float moff = m_new * a.scale_l2;
#pragma unroll
                for (int i = 0; i < 16; i += 2) {
                    const float p0 = __builtin_amdgcn_exp2f(__builtin_fmaf(sa[i], a.scale_l2, -moff));
                    const float p1 = __builtin_amdgcn_exp2f(__builtin_fmaf(sa[i + 1], a.scale_l2, -moff));
                    psum += p0 + p1;
                    pk[CP][i >> 1] = pack_bf16x2(p0, p1);
                }
            }
            if (c >= 1 && c - 1 <= cmax) pv(pk[CP ^ 1], sV);
            if (c <= cmax) finish_block(m_new, psum);
        };

        // ---------------- iteration c, pipelined form: all three stages, interleaved -----------
        // Slot j issues matrix instruction j (first the KS of S(c+1), then the 2*DB of O += P V),
        // the LDS read of the operand AH slots ahead, every second slot one copy instruction of the
        // tiles in flight (PF; K tile t+2 and V tile t+1), and a share of the softmax arithmetic of
        // block c: the row maximum in slots 0 and 1, the 16 exponentials over the remaining slots.
        // One basic block on purpose: a branch inside it would let the optimiser sink the softmax
        // arithmetic below the matrix instructions.
        auto iter_fast = [&](auto cpc, auto kbc, auto vbc, auto pfc, int t) {
            constexpr int CP = decltype(cpc)::value;  // c & 1; blocks c+1 and c-1 start at row 0 (CP = 1) or 32 of their tile
            constexpr int KB = decltype(kbc)::value, VB = decltype(vbc)::value;
            constexpr bool PF = decltype(pfc)::value != 0;
            constexpr int AH = 4;
            const char *sK = smem + KB * TILE + (CP ? 0 : 32 * L::ROWB);
            const char *sV = smem + (2 + VB) * TILE + (CP ? 0 : 32 * L::ROWB);
            f32x16 &sn = sacc[CP ^ 1];
            const f32x16 &sc = sacc[CP];
            const uint32_t(&pp)[8] = pk[CP ^ 1];
            bf16x8 fr[NSLOT];
            auto rd = [&](int j) {
                if (j < KS) return lds_nat(sK, lo.nat[j < KS ? j : 0]);
                const int rowoff = ((j - KS) / DB) * 16 * L::ROWB;
                return lds_tr(sV, rowoff + lo.tr[(j - KS) % DB][0], rowoff + lo.tr[(j - KS) % DB][1]);
            };
#pragma unroll
            for (int j = 0; j < AH; j++) fr[j] = rd(j);
#pragma unroll
            for (int i = 0; i < 16; i++) sn[i] = 0.f;
            // The block's scores are taken against the running reference as it stands, without looking
            // at their maximum first: bf16 and fp32 share their exponent range, so P may grow far
            // beyond 1 before anything is lost (O and the row sums are accumulated in fp32 and divided
            // at the end).  The largest row sum seen is kept instead (one instruction); if it shows,
            // when the item's steps are done, that some scores outgrew the reference by 2^64 or
            // overflowed, the wavefront recomputes its rows the careful way (see below).  The maximum,
            // its exchange between the half-waves and the comparison were a sixth of this loop's
            // vector instructions, and those are what bounds it.
            float psum = 0.f, pprev = 0.f;
            const float moff = m_run * a.scale_l2;
#pragma unroll
            for (int j = 0; j < NSLOT; j++) {
                if (j + AH < NSLOT) fr[j + AH] = rd(j + AH);
                if (j < KS) {
                    sn = mfma32(fr[j], qf[j < KS ? j : 0], sn);
                } else {
                    const int st = (j - KS) / DB;
                    Frag8 pf;
                    pf.u = u32x4{pp[4 * st], pp[4 * st + 1], pp[4 * st + 2], pp[4 * st + 3]};
                    oacc[(j - KS) % DB] = mfma32(fr[j], pf.v, oacc[(j - KS) % DB]);
                }
                if (PF && (j & 1)) {
                    const int n = j >> 1;
                    if (n < NCP / 2)
                        load_tile_async_fast_one<D>(smem + (KB ^ 1) * TILE, kbase + (int64_t)(t + 2) * kFwdBk * a.k_st,
                                                    a.k_st, goffk, wave, n);
                    else
                        load_tile_async_fast_one<D>(smem + (2 + (VB ^ 1)) * TILE, vbase + (int64_t)(t + 1) * kFwdBk * a.v_st,
                                                    a.v_st, goffv, wave, n - NCP / 2);
                }
                {
                    constexpr int NE = NSLOT;  // every slot carries its share of the 16 exponentials
#pragma unroll
                    for (int e = (j * 16) / NE; e < ((j + 1) * 16) / NE; e++) {
                        const float p = __builtin_amdgcn_exp2f(__builtin_fmaf(sc[e], a.scale_l2, -moff));
                        psum += p;
                        if (e & 1) {
                            pk[CP][e >> 1] = pack_bf16x2(pprev, p);
                            // keeps the arithmetic of this pair here: the optimiser would otherwise sink
                            // it to the pair's first use, below the matrix instructions it is to overlap
                            asm volatile("" : "+v"(pk[CP][e >> 1]));
                        } else {
                            pprev = p;
                        }
                    }
                }
            }
            asm volatile("" : "+v"(psum));  // the row-sum additions stay above, among the matrix instructions
            l_run += psum;
            psum_max = fmaxf(psum_max, psum);
        };

        // ---------------- pipeline fill: K tile 0 -> S(0), then iteration 0 --------------------
        // (the Q rows pass through this wavefront's quarter of the V buffers, which are idle until the
        // barrier: V tile 0 is requested after it)
        qrows.fragments(smem + 2 * TILE + wave * (32 * L::ROWB), 0, lo, qf, lane);
        wait_vmem();
        __builtin_amdgcn_s_waitcnt(0xC07F);  // lgkmcnt(0): the fragments are in registers
        __syncthreads();
        // (short items draw their ticket here, long ones near their end: see window())
        const int draw_t = ntiles >= kLateTicketSteps ? ntiles - 2 : -1;
        if (draw_t < 0) deal.prefetch();
        if (ntiles > 1) prefetch_k(1, 1);
        prefetch_v(0, 0);
        if (cmax >= 0) scores(sacc[0], smem);
        iter_slow(ic<0>{}, 0, smem + 32 * L::ROWB, smem);

        // ---------------- window t: iterations 2t+1 and 2t+2 ------------------------------------
        // Steady state: both iterations pipelined, and the copies of K tile t+2 and V tile t+1 (both
        // wholly inside the sequence) ride along with iteration 2t+1.  No branch but the rare rescale.
        auto window_steady = [&](auto vbc, int t) {
            constexpr int VB = decltype(vbc)::value, KB = VB ^ 1;  // V tile t in VB, K tile t+1 in KB
            lo.pin();
            wait_vmem();      // this wavefront's share of K tile t+1 and V tile t has landed
            __syncthreads();  // everybody's has, and everybody is done with K tile t and V tile t-1
            iter_fast(ic<1>{}, ic<KB>{}, ic<VB>{}, ic<1>{}, t);
            iter_fast(ic<0>{}, ic<KB>{}, ic<VB>{}, ic<0>{}, t);
        };
        // General form (pipeline fill and drain, masked block, ragged last tile): the copies go out in
        // one go after the barrier and the stages of an iteration run one after the other.  One copy
        // of the code for both buffer parities: the tile addresses are run-time values here.
        auto window = [&](int t) {
            const int vb = t & 1, kb = vb ^ 1;  // V tile t in vb, K tile t+1 in kb
            lo.pin();
            wait_vmem();      // this wavefront's share of K tile t+1 and V tile t has landed
            __syncthreads();  // everybody's has, and everybody is done with K tile t and V tile t-1
            if (t + 2 < ntiles) prefetch_k(t + 2, kb ^ 1);
            if (t + 1 < ntiles) prefetch_v(t + 1, vb ^ 1);
            // The ticket of the item after a LONG one is drawn in the item's last window but one: late enough
            // that the workgroup commits itself to another item only a few microseconds before it is
            // free for it (a ticket drawn when the item starts reserves the then-largest item for the
            // whole length of this one, and at the end of a pass every workgroup still owes an item
            // while others idle), early enough that the counter's round trip is over when the epilogue
            // is.  An item of a few steps gains nothing from that and pays the wait for the answer at its
            // end, so it draws right after its first barrier (behind its first loads, not in front of
            // them: answers come back in request order).
            if (t == draw_t) deal.prefetch();
            const char *sK = smem + kb * TILE, *sV = smem + (2 + vb) * TILE;
            iter_slow(ic<1>{}, 2 * t + 1, sK, sV);
            iter_slow(ic<0>{}, 2 * t + 2, sK + 32 * L::ROWB, sV + 32 * L::ROWB);
        };
        // windows [0, tsteady) are steady ones: t + 3 <= ntiles, (t + 3) * kFwdBk <= s, 2t + 3 <= cmax
        // (SHARD: and the blocks of a steady window lie before the first masked one)
        const int tsteady = max(0, min(min(ntiles, sk / kFwdBk) - 2, ((SHARD ? min(cmax, cmask) : cmax) - 1) >> 1));
        int t = 0;
        for (; t + 1 < tsteady; t += 2) {
            window_steady(ic<0>{}, t);
            window_steady(ic<1>{}, t + 1);
        }
        for (; t < ntiles; t++) window(t);

        // ---------------- (rare) the careful way, per wavefront ----------------------------------
        // Some row sum of a fast iteration was 2^64 or more, infinite or not a number: scores that
        // outgrew the reference such an iteration does not update.  The wavefront then computes its
        // 32 rows again, every block against its own maximum, on its own: K and V blocks of 32 keys
        // come straight from global memory through this wavefront's quarter of the K buffers (no
        // wavefront reads a K tile after the last window's barrier, and this one is past it).
        if (__builtin_expect(__builtin_amdgcn_ballot_w64(!(psum_max < 0x1p64f)) != 0, 0)) {
            char *mine = smem + wave * (32 * L::ROWB);
#pragma unroll
            for (int db = 0; db < DB; db++)
#pragma unroll
                for (int i = 0; i < 16; i++) oacc[db][i] = 0.f;
            m_run = SHARD ? -1e30f : -INFINITY;
            l_run = 0.f;
            for (int c = 0; c <= cmax; c++) {
                RowBlock<D> blk;
                blk.load(kbase, a.k_st, c * 32, sk - 1, lane);
                blk.stage(mine, 0, lane);
                f32x16 &sa = sacc[0];
                scores(sa, mine);
                if (SHARD ? c >= cmask : c == cmask) {
#pragma unroll
                    for (int i = 0; i < 16; i++) {
                        const int kv = c * 32 + 8 * (i >> 2) + 4 * hl + (i & 3);
                        if (kv > lim) sa[i] = -INFINITY;
                    }
                }
                const float m_new = reference(block_max(sa));
                const float mo = m_new * a.scale_l2;
                float ps = 0.f;
#pragma unroll
                for (int i = 0; i < 16; i += 2) {
                    const float p0 = __builtin_amdgcn_exp2f(__builtin_fmaf(sa[i], a.scale_l2, -mo));
                    const float p1 = __builtin_amdgcn_exp2f(__builtin_fmaf(sa[i + 1], a.scale_l2, -mo));
                    ps += p0 + p1;
                    pk[0][i >> 1] = pack_bf16x2(p0, p1);
                }
                blk.load(vbase, a.v_st, c * 32, sk - 1, lane);
                blk.stage(mine, 0, lane);  // (after the reads of the K block: one wavefront's LDS instructions execute in order)
                finish_block(m_new, ps);   // O and the row sum move to the block's reference first
                pv(pk[0], mine);
            }
        }

        // ---- epilogue: normalise, write O (bf16) and LSE (natural log)
        float l_tot = halves_sum(l_run);
        {
            if (nparts > 1) {
                // hand over (O unnormalised, row maximum, row sum); the part that arrives last merges
                // all parts in part order: O = sum_p 2^((m_p - M) scale_l2) O_p, likewise the row sums
                const int tid_ = wave * 64 + lane;  // (recomputed: keeping threadIdx alive through the tile loop costs a register)
                char *rec = a.pq.split_scratch + (int64_t)(slot + part) * kPartialBytes;
                split_store<DB>(rec, oacc, tid_);
                split_put((float *)(rec + 64 * kThreads * 4) + 2 * tid_, m_run);
                split_put((float *)(rec + 64 * kThreads * 4) + 2 * tid_ + 1, l_tot);
                if (!split_arrive(a.pq.split_flags + slot, nparts, &split_word, tid_)) continue;
                // all parts' row statistics first (one trip to memory for the lot), then the records in turn
                float mp[kMaxParts], lp[kMaxParts];
#pragma unroll
                for (int p = 0; p < kMaxParts; p++) {
                    const float *st = (const float *)(a.pq.split_scratch + (int64_t)(slot + min(p, nparts - 1)) * kPartialBytes +
                                                      64 * kThreads * 4) + 2 * tid_;
                    mp[p] = split_get(st);
                    lp[p] = split_get(st + 1);
                }
                float M = -INFINITY;
#pragma unroll
                for (int p = 0; p < kMaxParts; p++) M = p < nparts ? fmaxf(M, mp[p]) : M;
#pragma unroll
                for (int db = 0; db < DB; db++)
#pragma unroll
                    for (int i = 0; i < 16; i++) oacc[db][i] = 0.f;
                l_tot = 0.f;
#pragma unroll
                for (int p = 0; p < kMaxParts; p++) {
                    if (p < nparts) {
                        const float w = mp[p] == -INFINITY ? 0.f : __builtin_amdgcn_exp2f((mp[p] - M) * a.scale_l2);
                        split_sum<DB>(a.pq.split_scratch + (int64_t)(slot + p) * kPartialBytes, oacc, w, tid_);
                        l_tot += w * lp[p];
                    }
                }
                m_run = M;
            }
        }
        if constexpr (SHARD) {
            if (a.dq) {
                // Fold into the fp32 running result of a ring instead of writing this shard's own O and LSE:
                // (o_acc, lse_acc) <- merge((o_acc, lse_acc), (O, LSE)), the row's two half-wave lanes each
                // taking their head-dim elements of the row; a part that counts nothing is silenced even
                // if it holds rubbish (a running result is started with lse_acc = -inf over anything).
                if (qrow < s) {
                    const int64_t li = (int64_t)h * a.T + tok0 + qrow;
                    const float la = a.delta_out[li];
                    const float lb = l_tot > 0.f ? m_run * a.scale + __logf(l_tot) : -INFINITY;
                    const float m = fmaxf(la, lb);
                    float wa = 0.f, wb = 0.f, lse = -INFINITY;
                    if (m > -INFINITY) {
                        const float ea = __expf(la - m), eb = __expf(lb - m);
                        const float inv = 1.0f / (ea + eb);
                        wa = ea * inv;
                        wb = l_tot > 0.f ? eb * inv / l_tot : 0.f;  // (with the row's normalisation)
                        lse = m + __logf(ea + eb);
                    }
                    float *row = (float *)a.dq + (tok0 + qrow) * a.dq_st + (int64_t)h * a.dq_sh;
#pragma unroll
                    for (int db = 0; db < DB; db++)
#pragma unroll
                        for (int i4 = 0; i4 < 4; i4++) {
                            f32x4 *p = (f32x4 *)(row + db * 32 + 8 * i4 + 4 * hl);
                            f32x4 w = *p;
#pragma unroll
                            for (int e = 0; e < 4; e++) {
                                w[e] = (wa > 0.f ? wa * w[e] : 0.f) + wb * oacc[db][4 * i4 + e];
                                oacc[db][4 * i4 + e] = w[e];
                            }
                            *p = w;
                        }
                    if (hl == 0) a.delta_out[li] = lse;  // (after both lanes of the row have read it: one wavefront)
                }
                if (a.out_o && wq_lo < s)  // the merged rows rounded to bf16, if asked for
                    store_rowT_bf16_lds<DB>(smem + wave * (32 * L::ROWB), a.out_o + (tok0 + wq_lo) * a.o_st + (int64_t)h * a.o_sh,
                                            a.o_st, min(32, s - wq_lo), oacc, 1.0f, lane);
                continue;
            }
        }
        if (qrow < s && hl == 0) a.lse_out[(int64_t)h * a.T + tok0 + qrow] = m_run * a.scale + __logf(l_tot);
        // O is staged through the K buffers without a barrier: no wavefront reads a K tile after the
        // barrier of the last window (the scores of the last blocks were issued in the window before),
        // and this wavefront is past that barrier, so every wavefront has reached it
        if (wq_lo < s)
            store_rowT_bf16_lds<DB>(smem + wave * (32 * L::ROWB), a.out_o + (tok0 + wq_lo) * a.o_st + (int64_t)h * a.o_sh,
                                    a.o_st, min(32, s - wq_lo), oacc,
                                    (SHARD && !(l_tot > 0.f)) ? 0.f : 1.0f / l_tot, lane);
        // deal.advance() holds the barrier after which the LDS buffers are reused by the next item
    }
    deal.finish();
}

}  // namespace

hipError_t launch_attn_fwd(const AttnArgs &a, int D, int grid, hipStream_t s)
{
    if (D == 128)
        hipLaunchKernelGGL((attn_fwd_kernel<128, false>), dim3(grid), dim3(kThreads), 0, s, a);
    else
        hipLaunchKernelGGL((attn_fwd_kernel<64, false>), dim3(grid), dim3(kThreads), 0, s, a);
    return hipGetLastError();
}

hipError_t launch_attn_fwd_kvshard(const AttnArgs &a, int D, int grid, hipStream_t s)
{
    if (D == 128)
        hipLaunchKernelGGL((attn_fwd_kernel<128, true>), dim3(grid), dim3(kThreads), 0, s, a);
    else
        hipLaunchKernelGGL((attn_fwd_kernel<64, true>), dim3(grid), dim3(kThreads), 0, s, a);
    return hipGetLastError();
}

}  // namespace flexsp
