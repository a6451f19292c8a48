// Backward of packed causal attention (gradient of paper Sec. 2.1.2, Eq. 3, per sequence
// of the packed stream) for gfx950.  With P = softmax(scale Q K^T) recomputed from the saved
// log-sum-exp, and delta_i = dO_i . O_i:
//     dV = P^T dO,   dP = dO V^T,   dS = P o (dP - delta),
//     dQ = scale dS K,   dK = scale dS^T Q.
// Two kernels, no floating-point atomics (results are deterministic):
//   dQ      runs first; one work item = 128 query rows of one (sequence, head); loops over key
//           tiles; its prologue also computes delta and the base-2 log-sum-exp of its rows and
//           leaves them in the plan's scratch for the second kernel;
//   dK/dV   one work item = 64 keys of one (sequence, kv head); loops over the query heads of
//           the group and over the query rows that see those keys; dK^T, dV^T stay in
//           registers, so grouped-query heads are summed without a reduction pass.
// The 32x32 accumulator keeps one COLUMN per lane, and only its ROW index can be contracted
// in a following MFMA.  Hence dK/dV computes S = Q K^T (rows = queries) and dQ computes
// S^T = K Q^T (rows = keys).  Operands whose contraction index runs along the rows of a
// row-major LDS tile are fetched with the LDS transpose read.
#include <type_traits>

#include "attn_common.h"

namespace flexsp {
namespace {

// LDS fragments are read this many matrix instructions ahead of the one that uses them (the file is
// compiled in source order, like the forward kernel: the schedulers would sink the reads back)
constexpr int kReadAhead = 4;


// ------------------------------------------------------------------------------ dK / dV
// One work item = 64 keys of one (sequence, kv head).  The accumulators of 32 keys x D for both
// dK and dV, next to the K and V fragments, would take more than half of the register file and
// leave one wavefront per SIMD with nothing to hide its LDS latencies behind.  So TWO wavefronts
// share each block of 32 keys: per step of 64 query rows, wavefront j of the pair computes
// S = Q K^T, dP = dO V^T, P and dS for query block j only; then wavefront 0 accumulates
// dV^T += dO^T P and wavefront 1 accumulates dK^T += Q^T dS, each over BOTH query blocks.  For
// the other block each needs one bf16 fragment set from its partner (P one way, dS the other),
// swapped through LDS: a fragment is written and read back by the same lane numbers, so the swap
// is a plain linear copy.  No matrix work is duplicated, every wavefront fits in 256 registers,
// and two workgroups share a CU.
//
// SHARD = true is the variant for one shard of the keys (context parallelism; see the forward kernel):
// an item names 64 keys of the shard and the query rows of its sequence on this device, key j is
// visible to query row i iff j <= i + shift, the rows' log-sum-exp and delta are those of the COMPLETE
// attention, and the gradients may be added to what dK / dV hold.  Tiles are not cut into parts.
template <int D, bool SHARD>
__global__ __launch_bounds__(kThreads, 2) void attn_bwd_dkv_kernel(const AttnArgs a)
{
    typedef LdsTile<D> L;
    constexpr int KS = D / 16;
    constexpr int DB = D / 32;
    constexpr int BQ = kDkvBq;                  // query rows per step: two 32-row blocks
    constexpr int QTILE = BQ * L::ROWB;
    constexpr int STEP = 2 * QTILE + 512;       // Q | dO | lse2[64] delta[64]
    constexpr int XSLOT = 2048;                 // one 32 x 32 bf16 block (P or dS)
    __shared__ __attribute__((aligned(1024))) char smem[2 * STEP + 4 * XSLOT];
    char *const exch = smem + 2 * STEP;

    const int tid = threadIdx.x;
    const int lane0 = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int kb = wave >> 1, j = wave & 1;     // key block; role: 0 accumulates dV, 1 accumulates dK
    LaneOffsets<D> lo;
    lo.init(lane0);
    // What depends on the wavefront's role is folded into the per-lane offsets once: phase 1 reads the
    // rows of query block j, phase 2 reads the dO tile (role 0) or the Q tile (role 1).  Every LDS
    // read of a step is then "offset register + compile-time constant", with no address arithmetic.
#pragma unroll
    for (int ks = 0; ks < KS; ks++) lo.nat[ks] += j * 32 * L::ROWB;
#pragma unroll
    for (int db = 0; db < DB; db++) {
        lo.tr[db][0] += j ? 0 : QTILE;
        lo.tr[db][1] += j ? 0 : QTILE;
    }
    __shared__ int deal_word, split_word;
    ItemDealer deal;

    for (int item = deal.first(a.pq, &deal_word, wave, lane0); item >= 0; item = deal.advance()) {
        // s: query rows of the sequence; sk: its keys; sh: position of the first query minus position of
        // the first key (0 unless SHARD); tok0 / ktok0: their first rows in q, dO / k, v
        int s, sk, sh, g, kv0, first, total, nparts, part, slot, qfirst, nsteps;
        int64_t tok0, ktok0;
        if constexpr (SHARD) {
            const flexsp_shard_item it = load_shard_item((const flexsp_shard_item *)a.pq.items, item);
            s = it.q_len; sk = it.k_len; sh = it.shift; g = it.head_parts & 0xffff; kv0 = it.tile * kDkvBk;
            tok0 = it.q_start; ktok0 = it.k_start;
            // the first query row that sees the tile's first key, rounded down to a step boundary; no
            // steps at all when no row of the device sees these keys
            qfirst = a.causal ? (max(0, kv0 - sh) & ~(BQ - 1)) : 0;
            nsteps = max(0, (s - qfirst + BQ - 1) / BQ);
            first = 0; total = nsteps * a.G; nparts = 1; part = 0; slot = -1;
        } else {
            const flexsp_item it = load_item(a.pq.items, item);
            s = it.seq_len; sk = s; sh = 0; g = it.head; kv0 = it.tile * kDkvBk;
            tok0 = it.seq_start; ktok0 = tok0;
            qfirst = a.causal ? kv0 : 0;  // kv0 is a multiple of BQ
            nsteps = (s - qfirst + BQ - 1) / BQ;
            // the item walks steps `first` .. `total`-1 of the tile's nsteps * G (all of them unless the tile was cut)
            first = it.step_begin; total = it.step_end;
            nparts = it.parts & 0xffff; part = it.parts >> 16; slot = it.slot;
        }
        // opaque per-item copy of the lane id: per-lane address arithmetic of an item stays inside
        // the item instead of being hoisted out of this loop into long-lived registers
        int lane = lane0;
        asm volatile("" : "+v"(lane));
        const int r = lane & 31, hl = lane >> 5;
        const int wk_lo = kv0 + kb * 32;
        const int kvrow = wk_lo + r;  // this lane's key (column of S)

        const uint32_t goffq = tile_goff<D>(a.q_st, wave, lane), goffg = tile_goff<D>(a.do_st, wave, lane);
        // Steps are counted from the item's first one (n of them); which head and which query rows a step
        // covers is carried along instead of being divided out of a step number: (h_cur, q_cur) for the
        // step being computed, (h_nxt, q_nxt) for the one whose tiles are fetched meanwhile.
        const int n = total - first;
        // The ticket of the item after this one: a short item draws it now, a long one when its steps are
        // done (see the forward kernel; here not inside the steps: any branch there costs this kernel
        // 1-2 %, and behind a long item the wait for the answer, what the epilogue does not cover of
        // it, does not show).
        if (n < kLateTicketSteps) deal.prefetch();
        const int q_end = qfirst + nsteps * BQ;
        int h_cur = g * a.G + (SHARD ? 0 : first / nsteps), q_cur = qfirst + (SHARD ? 0 : (first % nsteps) * BQ);
        int h_nxt = h_cur, q_nxt = q_cur;
        auto advance_nxt = [&]() {
            q_nxt += BQ;
            if (q_nxt >= q_end) {
                q_nxt = qfirst;
                h_nxt++;
            }
        };
        auto prefetch = [&](int h, int qs, int buf) {
            char *base = smem + buf * STEP;
            const uint16_t *qb = a.q + tok0 * a.q_st + (int64_t)h * a.q_sh;
            const uint16_t *gb = a.dO + tok0 * a.do_st + (int64_t)h * a.do_sh;
            if (__builtin_expect(qs + BQ <= s, 1)) {  // whole tile inside the sequence
                load_tile_async_fast<D, BQ>(base, qb + (int64_t)qs * a.q_st, a.q_st, goffq, wave);
                load_tile_async_fast<D, BQ>(base + QTILE, gb + (int64_t)qs * a.do_st, a.do_st, goffg, wave);
            } else {
                load_tile_async<D, BQ>(base, qb, a.q_st, qs, s - 1, wave, lane);
                load_tile_async<D, BQ>(base + QTILE, gb, a.do_st, qs, s - 1, wave, lane);
            }
            if (wave < 2) {  // wavefront 0: lse2 of the 64 rows, wavefront 1: delta
                const float *src = (wave ? a.delta_in : a.lse_in) + (int64_t)h * a.T + tok0 + min(qs + lane, s - 1);
                global_to_lds4(src, base + 2 * QTILE + wave * 256);
            }
        };
        if (n > 0) prefetch(h_cur, q_cur, 0);
        advance_nxt();

        // K and V fragments of the pair's 32 keys (B operands: column = key, k = head dim), through
        // this wavefront's quarter of tile buffer 1, which is idle until step 0 requests step 1's tiles
        bf16x8 kf[KS], vf[KS];
        {
            RowBlock<D> krows, vrows;
            krows.load(a.k + ktok0 * a.k_st + (int64_t)g * a.k_sh, a.k_st, wk_lo, sk - 1, lane);
            vrows.load(a.v + ktok0 * a.v_st + (int64_t)g * a.v_sh, a.v_st, wk_lo, sk - 1, lane);
            // (this kernel's fragment offsets point at row block j of a tile: wavefronts 2kb and 2kb+1 use
            // the two halves of one 64-row stretch, so the stretch's address serves both)
            char *stretch = smem + STEP + kb * (64 * L::ROWB);
            krows.fragments(stretch, j * 32, lo, kf, lane);
            vrows.fragments(stretch, j * 32, lo, vf, lane);
            __builtin_amdgcn_s_waitcnt(0xC07F);  // lgkmcnt(0): in registers before step 0's barrier frees the buffer
        }
        f32x16 accT[DB];  // dV^T (role 0) or dK^T (role 1): rows = head dim, column = key
#pragma unroll
        for (int d = 0; d < DB; d++)
#pragma unroll
            for (int i = 0; i < 16; i++) accT[d][i] = 0.f;

        auto step_fn = [&](auto bufc, int step) {
            constexpr int BUF = decltype(bufc)::value;
            const char *sQ = smem + BUF * STEP;
            const char *sG = sQ + QTILE;
            const float *sL = (const float *)(sQ + 2 * QTILE);  // lse2[64], -delta[64]
            const int q_lo = q_cur;
            // a block (32 queries x the pair's 32 keys) is empty when it lies past the end of the
            // sequence or wholly above the diagonal; both wavefronts of a pair agree on that
            auto empty = [&](int qb) {
                const int lo_ = q_lo + qb * 32;
                return lo_ >= s || (a.causal && lo_ + 31 + sh < wk_lo);
            };
            lo.pin();
            wait_vmem();
            __syncthreads();  // tile `step` is in LDS; the previous step's exchange slots are free
            // (the copies of the next tiles go out after phase 1's matrix instructions, not here: a
            // wavefront waits until its copy instructions are accepted, and behind the barrier that wait
            // would sit in front of matrix work that is ready to go; about 1 % on batches of short
            // sequences; the same move in the dQ kernel cost 2 %)

            // ---- phase 1: P and dS of query block j
            // (matrix phases run at raised wave priority, the arithmetic between them at the base one: when
            // both workgroups of a compute unit want the matrix pipe, the one already in a matrix phase
            // finishes it first instead of both crawling through it together; 2-3 % on this kernel)
            __builtin_amdgcn_s_setprio(2);
            uint32_t pp[8], dd[8];
            const int my_lo = q_lo + j * 32;
            if (!empty(j)) {
                // The dP accumulator starts at -delta of its rows (the scratch holds delta negated), so the
                // matrix instructions deliver dP - delta and the subtraction costs no vector instruction.
                f32x16 sacc, pacc;
#pragma unroll
                for (int i4 = 0; i4 < 4; i4++) {
                    const f32x4 d4 = *(const f32x4 *)(sL + 64 + j * 32 + 8 * i4 + 4 * hl);
#pragma unroll
                    for (int e = 0; e < 4; e++) {
                        sacc[4 * i4 + e] = 0.f;
                        pacc[4 * i4 + e] = d4[e];
                    }
                }
                {
                    // fragment n: k step n / 2 of the Q tile (n even) or the dO tile (n odd); read AH ahead
                    constexpr int AH = kReadAhead, N = 2 * KS;
                    bf16x8 fr[N];
                    auto rd = [&](int n) { return lds_nat((n & 1) ? sG : sQ, lo.nat[n >> 1]); };  // (rows of block j: see lo.nat above)
#pragma unroll
                    for (int n = 0; n < AH; n++) fr[n] = rd(n);
#pragma unroll
                    for (int n = 0; n < N; n++) {
                        if (n + AH < N) fr[n + AH] = rd(n + AH);
                        if (n & 1)
                            pacc = mfma32(fr[n], vf[n >> 1], pacc);
                        else
                            sacc = mfma32(fr[n], kf[n >> 1], sacc);
                    }
                }
                __builtin_amdgcn_s_setprio(0);
                if (__builtin_expect(step + 1 < n, 1)) prefetch(h_nxt, q_nxt, BUF ^ 1);
                // rows of the accumulator: query my_lo + 8*i4 + 4*hl + e
                const bool masked = (a.causal && my_lo + sh < wk_lo + 31) || (my_lo + 32 > s);
                auto probs = [&](auto maskc) {
                    constexpr bool MASK = decltype(maskc)::value;
#pragma unroll
                    for (int i4 = 0; i4 < 4; i4++) {
                        const f32x4 l4 = *(const f32x4 *)(sL + j * 32 + 8 * i4 + 4 * hl);
                        float p[4], ds[4];
#pragma unroll
                        for (int e = 0; e < 4; e++) {
                            p[e] = __builtin_amdgcn_exp2f(__builtin_fmaf(sacc[4 * i4 + e], a.scale_l2, -l4[e]));
                            if (MASK) {
                                const int qr = my_lo + 8 * i4 + 4 * hl + e;
                                p[e] = ((a.causal && qr + sh < kvrow) || qr >= s) ? 0.f : p[e];
                            }
                            ds[e] = p[e] * pacc[4 * i4 + e];
                        }
                        pp[2 * i4] = pack_bf16x2(p[0], p[1]);
                        pp[2 * i4 + 1] = pack_bf16x2(p[2], p[3]);
                        dd[2 * i4] = pack_bf16x2(ds[0], ds[1]);
                        dd[2 * i4 + 1] = pack_bf16x2(ds[2], ds[3]);
                    }
                };
                if (masked)
                    probs(std::true_type{});
                else
                    probs(std::false_type{});
                // hand the partner what it accumulates: role 0 gives dS, role 1 gives P
                char *slot = exch + (kb * 2 + j) * XSLOT + lane * 16;
                *(u32x4 *)(slot) = j ? u32x4{pp[0], pp[1], pp[2], pp[3]} : u32x4{dd[0], dd[1], dd[2], dd[3]};
                *(u32x4 *)(slot + 1024) = j ? u32x4{pp[4], pp[5], pp[6], pp[7]} : u32x4{dd[4], dd[5], dd[6], dd[7]};
            }
            if (empty(j) && step + 1 < n) prefetch(h_nxt, q_nxt, BUF ^ 1);  // no phase 1: the copies go out here
            __syncthreads();  // the partner's fragments are visible
            __builtin_amdgcn_s_setprio(2);

            // ---- phase 2: role 0: dV^T += dO^T P, role 1: dK^T += Q^T dS, both query blocks
            const char *sX = sQ;  // (+ QTILE for role 0, inside lo.tr)
#pragma unroll
            for (int qb = 0; qb < 2; qb++) {
                if (empty(qb)) continue;
                Frag8 f[2];
                if (qb == j) {  // this wavefront's own block: from registers
                    f[0].u = j ? u32x4{dd[0], dd[1], dd[2], dd[3]} : u32x4{pp[0], pp[1], pp[2], pp[3]};
                    f[1].u = j ? u32x4{dd[4], dd[5], dd[6], dd[7]} : u32x4{pp[4], pp[5], pp[6], pp[7]};
                } else {        // the partner's block: from its slot
                    const char *slot = exch + (kb * 2 + qb) * XSLOT + lane * 16;
                    f[0].u = *(const u32x4 *)(slot);
                    f[1].u = *(const u32x4 *)(slot + 1024);
                }
                {
                    constexpr int AH = kReadAhead, N = 2 * DB;  // fragment n: query half n / DB, head-dim block n % DB
                    bf16x8 fr[N];
                    auto rd = [&](int n) {
                        const int rowoff = (qb * 32 + (n / DB) * 16) * L::ROWB;
                        return lds_tr(sX, rowoff + lo.tr[n % DB][0], rowoff + lo.tr[n % DB][1]);
                    };
#pragma unroll
                    for (int n = 0; n < AH; n++) fr[n] = rd(n);
#pragma unroll
                    for (int n = 0; n < N; n++) {
                        if (n + AH < N) fr[n + AH] = rd(n + AH);
                        accT[n % DB] = mfma32(fr[n], f[n / DB].v, accT[n % DB]);
                    }
                }
            }
            __builtin_amdgcn_s_setprio(0);
            h_cur = h_nxt;
            q_cur = q_nxt;
            advance_nxt();
        };
        for (int step = 0; step < n; step += 2) {
            step_fn(std::integral_constant<int, 0>{}, step);
            if (step + 1 < n) step_fn(std::integral_constant<int, 1>{}, step + 1);
        }
        if (n >= kLateTicketSteps) deal.prefetch();
        if (nparts > 1) {
            split_store<DB>(a.pq.split_scratch + (int64_t)(slot + part) * kPartialBytes, accT, tid);
            if (!split_arrive(a.pq.split_flags + slot, nparts, &split_word, tid)) continue;  // a later part finishes the tile
#pragma unroll
            for (int d = 0; d < DB; d++)
#pragma unroll
                for (int i = 0; i < 16; i++) accT[d][i] = 0.f;
            for (int p = 0; p < nparts; p++)
                split_sum<DB>(a.pq.split_scratch + (int64_t)(slot + p) * kPartialBytes, accT, 1.0f, tid);
        }

        // role 0 writes dV rows, role 1 writes dK rows (scaled)
        char *const out = (char *)(j ? a.dk : a.dv);
        const int64_t ost = j ? a.dk_st : a.dv_st, osh = j ? a.dk_sh : a.dv_sh;
        const float mul = j ? a.scale : 1.0f;
        if (SHARD && (a.grad_f32 & 2)) {  // added to the partial sums the rows hold
            if (kvrow < sk) add_rowT_f32<DB>((float *)out + (ktok0 + kvrow) * ost + (int64_t)g * osh, accT, mul, hl);
        } else if (a.grad_f32) {
            if (kvrow < sk) store_rowT<DB>(out + ((ktok0 + kvrow) * ost + (int64_t)g * osh) * 4, true, accT, mul, hl);
        } else if (wk_lo < sk) {
            // through the Q/dO buffer the last step did not use (every wavefront is past its barriers)
            store_rowT_bf16_lds<DB>(smem + (n & 1) * STEP + wave * (32 * L::ROWB),
                                    (uint16_t *)out + (ktok0 + wk_lo) * ost + (int64_t)g * osh, ost,
                                    min(32, sk - wk_lo), accT, mul, lane);
        }
        // deal.advance() holds the barrier after which the tiles and the exchange slots are reused
    }
    deal.finish();
}

// ------------------------------------------------------------------------------ dQ
// SHARD = true: the rows' share of dQ that comes from one shard of the keys (see the dK/dV kernel): the
// log-sum-exp read here is that of the complete attention and `o` the complete output, so delta is the
// complete one; a part of a cut tile comes as an item of its own with its key range and shift.
template <int D, bool SHARD>
__global__ __launch_bounds__(kThreads, 2) void attn_bwd_dq_kernel(const AttnArgs a)
{
    typedef LdsTile<D> L;
    constexpr int KS = D / 16;
    constexpr int DB = D / 32;
    constexpr int TILE = kDqBk * L::ROWB;
    __shared__ __attribute__((aligned(1024))) char smem[4 * TILE];  // [buffer][K | V]

    const int tid = threadIdx.x;
    const int lane0 = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    LaneOffsets<D> lo;
    lo.init(lane0);
    __shared__ int deal_word, split_word;
    ItemDealer deal;

    for (int item = deal.first(a.pq, &deal_word, wave, lane0); item >= 0; item = deal.advance()) {
        // s: query rows of the sequence; sk: keys counted from the item's first one; rel: position of a
        // row among those keys minus its row index; tok0 / ktok0: first rows in q, o, dO / k, v
        int s, sk, rel, h, q0, ntiles, nparts, part, slot;
        int64_t tok0, ktok0;
        if constexpr (SHARD) {
            const flexsp_shard_item it = load_shard_item((const flexsp_shard_item *)a.pq.items, item);
            s = it.q_len; sk = it.k_len; rel = it.shift; h = it.head_parts & 0xffff; q0 = it.tile * kDqBq;
            tok0 = it.q_start; ktok0 = it.k_start;
            part = (it.head_parts >> 16) & 0xff; nparts = it.head_parts >> 24; slot = it.slot;
            const int kv_end = a.causal ? max(0, min(sk, q0 + kDqBq + rel)) : sk;  // keys some row of the tile sees
            ntiles = (kv_end + kDqBk - 1) / kDqBk;
        } else {
            const flexsp_item it = load_item(a.pq.items, item);
            s = it.seq_len; h = it.head; q0 = it.tile * kDqBq;
            tok0 = it.seq_start;
            // The item walks key tiles step_begin .. step_end-1 (all of them unless the tile was cut: then it
            // hands its partial dQ over).  From here on keys are counted from the item's first one: koff keys
            // are skipped, `sk` remain, and a row's own position among them is its row index minus koff.
            const int koff = it.step_begin * kDqBk;
            ntiles = it.step_end - it.step_begin; sk = s - koff; rel = -koff;
            ktok0 = tok0 + koff;
            nparts = it.parts & 0xffff; part = it.parts >> 16; slot = it.slot;
        }
        // opaque per-item copy of the lane id: per-lane address arithmetic of an item stays inside
        // the item instead of being hoisted out of this loop into long-lived registers
        int lane = lane0;
        asm volatile("" : "+v"(lane));
        const int r = lane & 31, hl = lane >> 5;
        const int g = h / a.G;
        const uint16_t *kbase = a.k + ktok0 * a.k_st + (int64_t)g * a.k_sh;
        const uint16_t *vbase = a.v + ktok0 * a.v_st + (int64_t)g * a.v_sh;
        const uint32_t goffk = tile_goff<D>(a.k_st, wave, lane), goffv = tile_goff<D>(a.v_st, wave, lane);
        auto prefetch = [&](int t, int buf) {
            char *dk = smem + buf * 2 * TILE, *dv = dk + TILE;
            if (__builtin_expect((t + 1) * kDqBk <= sk, 1)) {  // whole tile inside the sequence
                load_tile_async_fast<D, kDqBk>(dk, kbase + (int64_t)t * kDqBk * a.k_st, a.k_st, goffk, wave);
                load_tile_async_fast<D, kDqBk>(dv, vbase + (int64_t)t * kDqBk * a.v_st, a.v_st, goffv, wave);
            } else {
                load_tile_async<D, kDqBk>(dk, kbase, a.k_st, t * kDqBk, sk - 1, wave, lane);
                load_tile_async<D, kDqBk>(dv, vbase, a.v_st, t * kDqBk, sk - 1, wave, lane);
            }
        };
        if (!SHARD || ntiles > 0) prefetch(0, 0);  // (a tile of a shard's queries may see none of its keys)

        const int qrow = q0 + wave * 32 + r;
        const int wq_lo = q0 + wave * 32;
        const int wq_rel = wq_lo + rel;  // the wavefront's first row, counted like the keys
        const bool qok = qrow < s;
        bf16x8 qf[KS], gf[KS];  // B operands: column = query row, k = head dim
        // delta = dO . O of the row (the backward's preprocessing step, done here because this kernel
        // has the row's dO in registers anyway): this lane's half of the row, then the other half-wave's
        float dpart = 0.f;
        {
            // the three row blocks are requested together and pass one after the other through this
            // wavefront's quarter of tile buffer 1, which is idle until step 0 requests tile 1
            RowBlock<D> qrows, grows, orows;
            qrows.load(a.q + tok0 * a.q_st + (int64_t)h * a.q_sh, a.q_st, wq_lo, s - 1, lane);
            grows.load(a.dO + tok0 * a.do_st + (int64_t)h * a.do_sh, a.do_st, wq_lo, s - 1, lane);
            orows.load(a.o + tok0 * a.o_st + (int64_t)h * a.o_sh, a.o_st, wq_lo, s - 1, lane);
            char *region = smem + 2 * TILE + wave * (32 * L::ROWB);
            bf16x8 of[KS];
            qrows.fragments(region, 0, lo, qf, lane);
            grows.fragments(region, 0, lo, gf, lane);
            orows.fragments(region, 0, lo, of, lane);
            __builtin_amdgcn_s_waitcnt(0xC07F);  // lgkmcnt(0): in registers before step 0's barrier frees the buffer
#pragma unroll
            for (int ks = 0; ks < KS; ks++) {
                Frag8 fg, fo;
                fg.v = gf[ks];
                fo.v = of[ks];
#pragma unroll
                for (int i = 0; i < 4; i++) {
                    // (scalars first: a bit cast applied to a vector element in place reads element 0)
                    const uint32_t gw = fg.u[i], ow = fo.u[i];
                    dpart = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, gw), __builtin_bit_cast(bf16x2, ow),
                                                            dpart, false);
                }
            }
        }
        const float delta = halves_sum(dpart);
        // the log-sum-exp in base 2, so that the recomputation is one fma + exp2 per score; +inf makes
        // P = 0 for rows past the end of the sequence
        float lse2 = qok ? a.lse_in[(int64_t)h * a.T + tok0 + qrow] * 1.4426950408889634f : INFINITY;
        if constexpr (SHARD) lse2 = lse2 == -INFINITY ? INFINITY : lse2;  // a row that saw no key anywhere

        f32x16 dqT[DB];  // rows = head dim, column = query
#pragma unroll
        for (int db = 0; db < DB; db++)
#pragma unroll
            for (int i = 0; i < 16; i++) dqT[db][i] = 0.f;

        const int draw_t = ntiles >= kLateTicketSteps ? ntiles - 3 : 0;  // the step in which the next ticket is drawn
        auto step_fn = [&](auto bufc, int t) {
            constexpr int BUF = decltype(bufc)::value;
            const char *sK = smem + BUF * 2 * TILE;
            const char *sV = sK + TILE;
            const int kv0 = t * kDqBk;
            lo.pin();
            wait_vmem();
            __syncthreads();
            // the next item's ticket: three steps before a long item ends, in a short one's first step (see the forward kernel)
            if (t == draw_t) deal.prefetch();
            if (__builtin_expect(t + 1 < ntiles, 1)) prefetch(t + 1, BUF ^ 1);
            if (a.causal && kv0 > wq_rel + 31) return;

            const bool need_mask = SHARD ? ((a.causal && kv0 + kDqBk - 1 > wq_rel) || kv0 + kDqBk > sk)
                                         : (a.causal ? (kv0 + kDqBk - 1 > wq_rel) : (kv0 + kDqBk > sk));
            const int lim = SHARD ? (a.causal ? min(qrow + rel, sk - 1) : sk - 1) : (a.causal ? qrow + rel : sk - 1);
            // one 32-key block at a time (keeps the register count under half the file)
#pragma unroll
            for (int kb = 0; kb < 2; kb++) {
                if (a.causal && kv0 + kb * 32 > wq_rel + 31) continue;  // block wholly above the diagonal
                f32x16 sacc, pacc;
#pragma unroll
                for (int i = 0; i < 16; i++) sacc[i] = pacc[i] = 0.f;
                {
                    constexpr int AH = kReadAhead, N = 2 * KS;  // fragment n: k step n / 2 of the K tile (n even) or the V tile (n odd)
                    bf16x8 fr[N];
                    auto rd = [&](int n) { return lds_nat((n & 1) ? sV : sK, kb * 32 * L::ROWB + lo.nat[n >> 1]); };
#pragma unroll
                    for (int n = 0; n < AH; n++) fr[n] = rd(n);
#pragma unroll
                    for (int n = 0; n < N; n++) {
                        if (n + AH < N) fr[n + AH] = rd(n + AH);
                        if (n & 1)
                            pacc = mfma32(fr[n], gf[n >> 1], pacc);
                        else
                            sacc = mfma32(fr[n], qf[n >> 1], sacc);
                    }
                }
                uint32_t dd[8];
                auto dsfn = [&](auto maskc) {
                    constexpr bool MASK = decltype(maskc)::value;
#pragma unroll
                    for (int i = 0; i < 16; i += 2) {
                        float p0 = __builtin_amdgcn_exp2f(__builtin_fmaf(sacc[i], a.scale_l2, -lse2));
                        float p1 = __builtin_amdgcn_exp2f(__builtin_fmaf(sacc[i + 1], a.scale_l2, -lse2));
                        if (MASK) {
                            const int kv = kv0 + kb * 32 + 8 * (i >> 2) + 4 * hl + (i & 3);
                            p0 = kv > lim ? 0.f : p0;
                            p1 = kv + 1 > lim ? 0.f : p1;
                        }
                        dd[i >> 1] = pack_bf16x2(p0 * (pacc[i] - delta), p1 * (pacc[i + 1] - delta));
                    }
                };
                if (need_mask)
                    dsfn(std::true_type{});
                else
                    dsfn(std::false_type{});
                // dQ^T += K^T dS^T
                {
                    constexpr int AH = kReadAhead, N = 2 * DB;  // fragment n: key half n / DB, head-dim block n % DB
                    bf16x8 fr[N];
                    auto rd = [&](int n) {
                        const int rowoff = (kb * 32 + (n / DB) * 16) * L::ROWB;
                        return lds_tr(sK, rowoff + lo.tr[n % DB][0], rowoff + lo.tr[n % DB][1]);
                    };
#pragma unroll
                    for (int n = 0; n < AH; n++) fr[n] = rd(n);
#pragma unroll
                    for (int n = 0; n < N; n++) {
                        if (n + AH < N) fr[n + AH] = rd(n + AH);
                        const int hf = n / DB;
                        Frag8 df;
                        df.u = u32x4{dd[4 * hf], dd[4 * hf + 1], dd[4 * hf + 2], dd[4 * hf + 3]};
                        dqT[n % DB] = mfma32(fr[n], df.v, dqT[n % DB]);
                    }
                }
            }
        };
        if (ntiles <= 0) deal.prefetch();
        for (int t = 0; t < ntiles; t += 2) {
            step_fn(std::integral_constant<int, 0>{}, t);
            if (t + 1 < ntiles) step_fn(std::integral_constant<int, 1>{}, t + 1);
        }

        // delta and the base-2 log-sum-exp are kept for the dK/dV kernel, which runs after this one
        // (stored here, not where they are computed: a store in flight there would be waited for by
        // the first tile's wait for its copy)
        if (qok && hl == 0) {
            a.delta_out[(int64_t)h * a.T + tok0 + qrow] = -delta;  // negated: the dK/dV kernel starts its dP accumulator from it
            a.lse_out[(int64_t)h * a.T + tok0 + qrow] = lse2;
        }
        if (nparts > 1) {
            split_store<DB>(a.pq.split_scratch + (int64_t)(slot + part) * kPartialBytes, dqT, tid);
            if (!split_arrive(a.pq.split_flags + slot, nparts, &split_word, tid)) continue;  // a later part finishes the tile
#pragma unroll
            for (int db = 0; db < DB; db++)
#pragma unroll
                for (int i = 0; i < 16; i++) dqT[db][i] = 0.f;
            for (int p = 0; p < nparts; p++)
                split_sum<DB>(a.pq.split_scratch + (int64_t)(slot + p) * kPartialBytes, dqT, 1.0f, tid);
        }
        if (SHARD && (a.grad_f32 & 2)) {  // added to the partial sum the rows hold
            if (qok)
                add_rowT_f32<DB>((float *)a.dq + (tok0 + qrow) * a.dq_st + (int64_t)h * a.dq_sh, dqT, a.scale, hl);
        } else if (a.grad_f32) {
            if (qok)
                store_rowT<DB>((char *)a.dq + ((tok0 + qrow) * a.dq_st + (int64_t)h * a.dq_sh) * 4, true, dqT,
                               a.scale, hl);
        } else if (wq_lo < s) {
            // through the tile buffer the last step did not use (see the forward kernel)
            store_rowT_bf16_lds<DB>(smem + (ntiles & 1) * 2 * TILE + wave * (32 * L::ROWB),
                                    (uint16_t *)a.dq + (tok0 + wq_lo) * a.dq_st + (int64_t)h * a.dq_sh, a.dq_st,
                                    min(32, s - wq_lo), dqT, a.scale, lane);
        }
        // deal.advance() holds the barrier after which the LDS buffers are reused by the next item
    }
    deal.finish();
}

}  // namespace

hipError_t launch_attn_bwd_dkv(const AttnArgs &a, int D, int grid, hipStream_t s)
{
    if (D == 128)
        hipLaunchKernelGGL((attn_bwd_dkv_kernel<128, false>), dim3(grid), dim3(kThreads), 0, s, a);
    else
        hipLaunchKernelGGL((attn_bwd_dkv_kernel<64, false>), dim3(grid), dim3(kThreads), 0, s, a);
    return hipGetLastError();
}

hipError_t launch_attn_bwd_dq(const AttnArgs &a, int D, int grid, hipStream_t s)
{
    if (D == 128)
        hipLaunchKernelGGL((attn_bwd_dq_kernel<128, false>), dim3(grid), dim3(kThreads), 0, s, a);
    else
        hipLaunchKernelGGL((attn_bwd_dq_kernel<64, false>), dim3(grid), dim3(kThreads), 0, s, a);
    return hipGetLastError();
}

hipError_t launch_attn_bwd_dkv_kvshard(const AttnArgs &a, int D, int grid, hipStream_t s)
{
    if (D == 128)
        hipLaunchKernelGGL((attn_bwd_dkv_kernel<128, true>), dim3(grid), dim3(kThreads), 0, s, a);
    else
        hipLaunchKernelGGL((attn_bwd_dkv_kernel<64, true>), dim3(grid), dim3(kThreads), 0, s, a);
    return hipGetLastError();
}

hipError_t launch_attn_bwd_dq_kvshard(const AttnArgs &a, int D, int grid, hipStream_t s)
{
    if (D == 128)
        hipLaunchKernelGGL((attn_bwd_dq_kernel<128, true>), dim3(grid), dim3(kThreads), 0, s, a);
    else
        hipLaunchKernelGGL((attn_bwd_dq_kernel<64, true>), dim3(grid), dim3(kThreads), 0, s, a);
    return hipGetLastError();
}

}  // namespace flexsp
