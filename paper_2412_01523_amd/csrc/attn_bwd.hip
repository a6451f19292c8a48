// Backward of packed causal attention (gradient of paper Sec. 2.1.2, Eq. 3, per sequence
// of the packed stream) for gfx950.  With P = softmax(scale Q K^T) recomputed from the saved
// log-sum-exp, and delta_i = dO_i . O_i:
//     dV = P^T dO,   dP = dO V^T,   dS = P o (dP - delta),
//     dQ = scale dS K,   dK = scale dS^T Q.
// Three kernels, no floating-point atomics (results are deterministic):
//   delta   one pass over dO and O (HBM-bound);
//   dK/dV   one work item = 128 keys of one (sequence, kv head); loops over the query heads
//           of the group and over the query rows that see those keys; dK^T, dV^T stay in
//           registers, so grouped-query heads are summed without a reduction pass;
//   dQ      one work item = 128 query rows of one (sequence, head); loops over key tiles.
// The 32x32 accumulator keeps one COLUMN per lane, and only its ROW index can be contracted
// in a following MFMA.  Hence dK/dV computes S = Q K^T (rows = queries) and dQ computes
// S^T = K Q^T (rows = keys).  Operands whose contraction index runs along the rows of a
// row-major LDS tile are fetched with the LDS transpose read.
#include "attn_common.h"

namespace flexsp {
namespace {

// ------------------------------------------------------------------------------ delta
template <int D>
__global__ __launch_bounds__(256) void attn_bwd_delta_kernel(const AttnArgs a)
{
    constexpr int LPR = D / 8;        // lanes per row
    constexpr int RPB = 256 / LPR;    // rows per block
    const int64_t rows = (int64_t)a.T * a.Hq;
    const int sub = threadIdx.x % LPR;
    // block-uniform loop: lanes past the end still take part in the shuffles
    for (int64_t base = (int64_t)blockIdx.x * RPB; base < rows; base += (int64_t)gridDim.x * RPB) {
        const int64_t row = base + threadIdx.x / LPR;
        const bool ok = row < rows;
        const int64_t t = ok ? row / a.Hq : 0;
        const int h = ok ? (int)(row % a.Hq) : 0;
        u32x4 x = *(const u32x4 *)(a.o + t * a.o_st + (int64_t)h * a.o_sh + sub * 8);
        u32x4 y = *(const u32x4 *)(a.dO + t * a.do_st + (int64_t)h * a.do_sh + sub * 8);
        float acc = 0.f;
#pragma unroll
        for (int i = 0; i < 4; i++)
            acc += bf16_lo(x[i]) * bf16_lo(y[i]) + bf16_hi(x[i]) * bf16_hi(y[i]);
#pragma unroll
        for (int off = LPR / 2; off > 0; off >>= 1) acc += __shfl_xor(acc, off);
        if (ok && sub == 0) a.delta_out[(int64_t)h * a.T + t] = acc;
    }
}

// ------------------------------------------------------------------------------ dK / dV
template <int D>
struct DkvCfg {
    static constexpr int KS = D / 16;
    static constexpr int DB = D / 32;
    static constexpr int STRIDE = D + 8;   // Q / dO tile row stride (elements)
    static constexpr int CH = D / 8;
    static constexpr int BQ = kDkvBq;      // query rows staged per step
    static constexpr int NLD = BQ * CH / kThreads;
};

template <int D>
__global__ __launch_bounds__(kThreads, 1) void attn_bwd_dkv_kernel(const AttnArgs a)
{
    typedef DkvCfg<D> C;
    __shared__ __attribute__((aligned(16))) uint16_t sQ[C::BQ * C::STRIDE];
    __shared__ __attribute__((aligned(16))) uint16_t sG[C::BQ * C::STRIDE];
    __shared__ __attribute__((aligned(16))) float sLse[C::BQ];
    __shared__ __attribute__((aligned(16))) float sDel[C::BQ];
    __shared__ int s_item;

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int r = lane & 31, hl = lane >> 5;
    int cursor = 0;
    const float log2e = 1.4426950408889634f;

    for (;;) {
        if (tid == 0) s_item = queue_fetch(a.pq, cursor);
        __syncthreads();
        const int item = s_item;
        if (item < 0) break;
        const flexsp_item it = a.pq.items[item];
        const int s = it.seq_len, g = it.head;
        const int kv0 = it.tile * kDkvBk;
        const int64_t tok0 = it.seq_start;
        const int kvrow = kv0 + wave * 32 + r;  // this lane's key (column of S)
        const int wk_lo = kv0 + wave * 32;

        // K and V fragments of this wavefront's 32 keys (B operands: column = key, k = head dim)
        bf16x8 kf[C::KS], vf[C::KS];
        {
            const bool ok = kvrow < s;
            const uint16_t *kp = a.k + (tok0 + (ok ? kvrow : 0)) * a.k_st + (int64_t)g * a.k_sh + 8 * hl;
            const uint16_t *vp = a.v + (tok0 + (ok ? kvrow : 0)) * a.v_st + (int64_t)g * a.v_sh + 8 * hl;
#pragma unroll
            for (int ks = 0; ks < C::KS; ks++) {
                Frag8 f;
                f.u = ok ? *(const u32x4 *)(kp + 16 * ks) : u32x4{0, 0, 0, 0};
                kf[ks] = f.v;
                f.u = ok ? *(const u32x4 *)(vp + 16 * ks) : u32x4{0, 0, 0, 0};
                vf[ks] = f.v;
            }
        }
        f32x16 dkT[C::DB], dvT[C::DB];  // rows = head dim, column = key
#pragma unroll
        for (int db = 0; db < C::DB; db++)
#pragma unroll
            for (int i = 0; i < 16; i++) dkT[db][i] = dvT[db][i] = 0.f;

        const int qfirst = a.causal ? kv0 : 0;  // kv0 is a multiple of BQ
        const int nsteps = (s - qfirst + C::BQ - 1) / C::BQ;
        const int total = nsteps * a.G;

        u32x4 qreg[C::NLD], greg[C::NLD];
        float lreg = 0.f, dreg = 0.f;
        auto gload = [&](int step) {
            const int h = g * a.G + step / nsteps;
            const int qs = qfirst + (step % nsteps) * C::BQ;
            const uint16_t *qb = a.q + tok0 * a.q_st + (int64_t)h * a.q_sh;
            const uint16_t *gb = a.dO + tok0 * a.do_st + (int64_t)h * a.do_sh;
#pragma unroll
            for (int n = 0; n < C::NLD; n++) {
                int c = n * kThreads + tid;
                int row = c / C::CH, col = (c % C::CH) * 8;
                bool ok = qs + row < s;
                qreg[n] = ok ? *(const u32x4 *)(qb + (int64_t)(qs + row) * a.q_st + col) : u32x4{0, 0, 0, 0};
                greg[n] = ok ? *(const u32x4 *)(gb + (int64_t)(qs + row) * a.do_st + col) : u32x4{0, 0, 0, 0};
            }
            if (tid < C::BQ) {
                bool ok = qs + tid < s;
                // +inf log-sum-exp makes P = 0 for rows past the end of the sequence
                lreg = ok ? a.lse_in[(int64_t)h * a.T + tok0 + qs + tid] * log2e : INFINITY;
                dreg = ok ? a.delta_in[(int64_t)h * a.T + tok0 + qs + tid] : 0.f;
            }
        };
        auto lstore = [&]() {
#pragma unroll
            for (int n = 0; n < C::NLD; n++) {
                int c = n * kThreads + tid;
                int row = c / C::CH, col = (c % C::CH) * 8;
                *(u32x4 *)(sQ + row * C::STRIDE + col) = qreg[n];
                *(u32x4 *)(sG + row * C::STRIDE + col) = greg[n];
            }
            if (tid < C::BQ) {
                sLse[tid] = lreg;
                sDel[tid] = dreg;
            }
        };

        if (total > 0) gload(0);
        for (int step = 0; step < total; step++) {
            const int qs = qfirst + (step % nsteps) * C::BQ;
            __syncthreads();
            lstore();
            __syncthreads();
            if (step + 1 < total) gload(step + 1);
#pragma unroll
            for (int qb = 0; qb < C::BQ / 32; qb++) {
                const int q_lo = qs + qb * 32;  // first query row of this block
                if (q_lo >= s) continue;
                if (a.causal && q_lo + 31 < wk_lo) continue;  // all rows before all keys
                f32x16 sacc, pacc;
#pragma unroll
                for (int i = 0; i < 16; i++) sacc[i] = pacc[i] = 0.f;
#pragma unroll
                for (int ks = 0; ks < C::KS; ks++) {
                    bf16x8 qa = lds_frag(sQ, C::STRIDE, qb * 32, ks * 16, lane);
                    sacc = mfma32(qa, kf[ks], sacc);
                    bf16x8 ga = lds_frag(sG, C::STRIDE, qb * 32, ks * 16, lane);
                    pacc = mfma32(ga, vf[ks], pacc);
                }
                // rows of the accumulator: query q_lo + 8*(i/4) + 4*hl + i%4
                f32x4 l4[4], d4[4];
#pragma unroll
                for (int i4 = 0; i4 < 4; i4++) {
                    l4[i4] = *(const f32x4 *)(sLse + qb * 32 + 8 * i4 + 4 * hl);
                    d4[i4] = *(const f32x4 *)(sDel + qb * 32 + 8 * i4 + 4 * hl);
                }
                const bool need_mask = a.causal && (q_lo < wk_lo + 31);
                uint32_t pp[8], dd[8];
#pragma unroll
                for (int i = 0; i < 16; i += 2) {
                    float p0 = __builtin_amdgcn_exp2f(__builtin_fmaf(sacc[i], a.scale_l2, -l4[i >> 2][i & 3]));
                    float p1 = __builtin_amdgcn_exp2f(__builtin_fmaf(sacc[i + 1], a.scale_l2, -l4[i >> 2][(i + 1) & 3]));
                    if (need_mask) {
                        int qr = q_lo + 8 * (i >> 2) + 4 * hl + (i & 3);
                        if (qr < kvrow) p0 = 0.f;
                        if (qr + 1 < kvrow) p1 = 0.f;
                    }
                    float s0 = p0 * (pacc[i] - d4[i >> 2][i & 3]);
                    float s1 = p1 * (pacc[i + 1] - d4[i >> 2][(i + 1) & 3]);
                    pp[i >> 1] = pack_bf16x2(p0, p1);
                    dd[i >> 1] = pack_bf16x2(s0, s1);
                }
#pragma unroll
                for (int hf = 0; hf < 2; hf++) {
                    Frag8 pf, df;
                    pf.u = u32x4{pp[4 * hf], pp[4 * hf + 1], pp[4 * hf + 2], pp[4 * hf + 3]};
                    df.u = u32x4{dd[4 * hf], dd[4 * hf + 1], dd[4 * hf + 2], dd[4 * hf + 3]};
#pragma unroll
                    for (int db = 0; db < C::DB; db++) {
                        bf16x8 gt = lds_frag_tr(sG, C::STRIDE, qb * 32 + hf * 16, db * 32, lane);
                        dvT[db] = mfma32(gt, pf.v, dvT[db]);
                        bf16x8 qt = lds_frag_tr(sQ, C::STRIDE, qb * 32 + hf * 16, db * 32, lane);
                        dkT[db] = mfma32(qt, df.v, dkT[db]);
                    }
                }
            }
        }

        if (kvrow < s) {
            const int64_t eb = a.grad_f32 ? 4 : 2;
            store_rowT<C::DB>((char *)a.dk + ((tok0 + kvrow) * a.dk_st + (int64_t)g * a.dk_sh) * eb, a.grad_f32,
                              dkT, a.scale, hl);
            store_rowT<C::DB>((char *)a.dv + ((tok0 + kvrow) * a.dv_st + (int64_t)g * a.dv_sh) * eb, a.grad_f32,
                              dvT, 1.0f, hl);
        }
        __syncthreads();
    }
    if (tid == 0) queue_retire(a.pq);
}

// ------------------------------------------------------------------------------ dQ
template <int D>
struct DqCfg {
    static constexpr int KS = D / 16;
    static constexpr int DB = D / 32;
    static constexpr int KSTRIDE = D + 8;   // K tile: natural AND transpose reads
    static constexpr int VSTRIDE = D + 8;   // V tile: natural reads
    static constexpr int CH = D / 8;
    static constexpr int NLD = kDqBk * CH / kThreads;
};

template <int D>
__global__ __launch_bounds__(kThreads, 2) void attn_bwd_dq_kernel(const AttnArgs a)
{
    typedef DqCfg<D> C;
    __shared__ __attribute__((aligned(16))) uint16_t sK[kDqBk * C::KSTRIDE];
    __shared__ __attribute__((aligned(16))) uint16_t sV[kDqBk * C::VSTRIDE];
    __shared__ int s_item;

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int r = lane & 31, hl = lane >> 5;
    int cursor = 0;
    const float log2e = 1.4426950408889634f;

    for (;;) {
        if (tid == 0) s_item = queue_fetch(a.pq, cursor);
        __syncthreads();
        const int item = s_item;
        if (item < 0) break;
        const flexsp_item it = a.pq.items[item];
        const int s = it.seq_len, h = it.head, g = h / a.G;
        const int q0 = it.tile * kDqBq;
        const int64_t tok0 = it.seq_start;
        const int kv_end = a.causal ? min(s, q0 + kDqBq) : s;
        const int ntiles = (kv_end + kDqBk - 1) / kDqBk;
        const int qrow = q0 + wave * 32 + r;
        const int wq_lo = q0 + wave * 32;
        const bool qok = qrow < s;

        bf16x8 qf[C::KS], gf[C::KS];  // B operands: column = query row, k = head dim
        {
            const uint16_t *qp = a.q + (tok0 + (qok ? qrow : 0)) * a.q_st + (int64_t)h * a.q_sh + 8 * hl;
            const uint16_t *gp = a.dO + (tok0 + (qok ? qrow : 0)) * a.do_st + (int64_t)h * a.do_sh + 8 * hl;
#pragma unroll
            for (int ks = 0; ks < C::KS; ks++) {
                Frag8 f;
                f.u = qok ? *(const u32x4 *)(qp + 16 * ks) : u32x4{0, 0, 0, 0};
                qf[ks] = f.v;
                f.u = qok ? *(const u32x4 *)(gp + 16 * ks) : u32x4{0, 0, 0, 0};
                gf[ks] = f.v;
            }
        }
        const float lse2 = qok ? a.lse_in[(int64_t)h * a.T + tok0 + qrow] * log2e : INFINITY;
        const float delta = qok ? a.delta_in[(int64_t)h * a.T + tok0 + qrow] : 0.f;

        f32x16 dqT[C::DB];  // rows = head dim, column = query
#pragma unroll
        for (int db = 0; db < C::DB; db++)
#pragma unroll
            for (int i = 0; i < 16; i++) dqT[db][i] = 0.f;

        const uint16_t *kbase = a.k + tok0 * a.k_st + (int64_t)g * a.k_sh;
        const uint16_t *vbase = a.v + tok0 * a.v_st + (int64_t)g * a.v_sh;
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
        for (int t = 0; t < ntiles; t++) {
            const int kv0 = t * kDqBk;
            __syncthreads();
            lstore();
            __syncthreads();
            if (t + 1 < ntiles) gload(kv0 + kDqBk);
            if (a.causal && kv0 > wq_lo + 31) continue;

            f32x16 sacc[2], pacc[2];
#pragma unroll
            for (int kb = 0; kb < 2; kb++)
#pragma unroll
                for (int i = 0; i < 16; i++) sacc[kb][i] = pacc[kb][i] = 0.f;
#pragma unroll
            for (int ks = 0; ks < C::KS; ks++)
#pragma unroll
                for (int kb = 0; kb < 2; kb++) {
                    bf16x8 ka = lds_frag(sK, C::KSTRIDE, kb * 32, ks * 16, lane);
                    sacc[kb] = mfma32(ka, qf[ks], sacc[kb]);
                    bf16x8 va = lds_frag(sV, C::VSTRIDE, kb * 32, ks * 16, lane);
                    pacc[kb] = mfma32(va, gf[ks], pacc[kb]);
                }
            const bool need_mask = a.causal ? (kv0 + kDqBk - 1 > wq_lo) : (kv0 + kDqBk > s);
            const int lim = a.causal ? qrow : s - 1;
            uint32_t dd[2][8];
#pragma unroll
            for (int kb = 0; kb < 2; kb++)
#pragma unroll
                for (int i = 0; i < 16; i += 2) {
                    float p0 = __builtin_amdgcn_exp2f(__builtin_fmaf(sacc[kb][i], a.scale_l2, -lse2));
                    float p1 = __builtin_amdgcn_exp2f(__builtin_fmaf(sacc[kb][i + 1], a.scale_l2, -lse2));
                    if (need_mask) {
                        int kv = kv0 + kb * 32 + 8 * (i >> 2) + 4 * hl + (i & 3);
                        if (kv > lim) p0 = 0.f;
                        if (kv + 1 > lim) p1 = 0.f;
                    }
                    dd[kb][i >> 1] = pack_bf16x2(p0 * (pacc[kb][i] - delta), p1 * (pacc[kb][i + 1] - delta));
                }
            // dQ^T += K^T dS^T
#pragma unroll
            for (int kb = 0; kb < 2; kb++)
#pragma unroll
                for (int hf = 0; hf < 2; hf++) {
                    Frag8 df;
                    df.u = u32x4{dd[kb][4 * hf], dd[kb][4 * hf + 1], dd[kb][4 * hf + 2], dd[kb][4 * hf + 3]};
#pragma unroll
                    for (int db = 0; db < C::DB; db++) {
                        bf16x8 kt = lds_frag_tr(sK, C::KSTRIDE, kb * 32 + hf * 16, db * 32, lane);
                        dqT[db] = mfma32(kt, df.v, dqT[db]);
                    }
                }
        }

        if (qok) {
            const int64_t eb = a.grad_f32 ? 4 : 2;
            store_rowT<C::DB>((char *)a.dq + ((tok0 + qrow) * a.dq_st + (int64_t)h * a.dq_sh) * eb, a.grad_f32,
                              dqT, a.scale, hl);
        }
        __syncthreads();
    }
    if (tid == 0) queue_retire(a.pq);
}

}  // namespace

hipError_t launch_attn_bwd_delta(const AttnArgs &a, int D, hipStream_t s)
{
    int64_t rows = (int64_t)a.T * a.Hq;
    int rpb = 256 / (D / 8);
    int64_t blocks = (rows + rpb - 1) / rpb;
    if (blocks > 256 * 16) blocks = 256 * 16;
    if (blocks < 1) blocks = 1;
    if (D == 128)
        hipLaunchKernelGGL(attn_bwd_delta_kernel<128>, dim3((unsigned)blocks), dim3(256), 0, s, a);
    else
        hipLaunchKernelGGL(attn_bwd_delta_kernel<64>, dim3((unsigned)blocks), dim3(256), 0, s, a);
    return hipGetLastError();
}

hipError_t launch_attn_bwd_dkv(const AttnArgs &a, int D, int grid, hipStream_t s)
{
    if (D == 128)
        hipLaunchKernelGGL(attn_bwd_dkv_kernel<128>, dim3(grid), dim3(kThreads), 0, s, a);
    else
        hipLaunchKernelGGL(attn_bwd_dkv_kernel<64>, dim3(grid), dim3(kThreads), 0, s, a);
    return hipGetLastError();
}

hipError_t launch_attn_bwd_dq(const AttnArgs &a, int D, int grid, hipStream_t s)
{
    if (D == 128)
        hipLaunchKernelGGL(attn_bwd_dq_kernel<128>, dim3(grid), dim3(kThreads), 0, s, a);
    else
        hipLaunchKernelGGL(attn_bwd_dq_kernel<64>, dim3(grid), dim3(kThreads), 0, s, a);
    return hipGetLastError();
}

}  // namespace flexsp
