// Device helpers shared by the attention kernels: MFMA fragment types, the LDS
// transpose read, bf16 packing and the per-XCD work-queue fetch.
#pragma once

#include "flexsp_internal.h"

namespace flexsp {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;
typedef __attribute__((ext_vector_type(4))) short s16x4;

// v_mfma_f32_32x32x16_bf16, D = A(32x16) * B(16x32) + C.  Lane l (r = l % 32, hl = l / 32):
//   A: row r, k = 8*hl .. 8*hl+7          B: column r, k = 8*hl .. 8*hl+7
//   C/D register i: row 8*(i/4) + 4*hl + i%4, column r.
// Any permutation of the k slots is fine as long as A and B use the same one.
__device__ __forceinline__ f32x16 mfma32(bf16x8 a, bf16x8 b, f32x16 c)
{
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

union Frag8 {
    bf16x8 v;
    u32x4 u;
    s16x4 h[2];
    uint16_t s[8];
};

__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi)
{
    bf16x2 t;
    t[0] = (__bf16)lo;  // round to nearest even
    t[1] = (__bf16)hi;
    return __builtin_bit_cast(uint32_t, t);
}

__device__ __forceinline__ float bf16_lo(uint32_t u) { return __builtin_bit_cast(float, u << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t u) { return __builtin_bit_cast(float, u & 0xffff0000u); }

// ds_read_b64_tr_b16: the 16 lanes of a group each name 4 consecutive 16-bit elements;
// seen as a 4 x 16 block whose row r is supplied by lanes 4r .. 4r+3 of the group, lane i
// receives column i (4 elements, one per row).  `p` is this lane's source address.
__device__ __forceinline__ s16x4 lds_read_tr(const uint16_t *p)
{
    return __builtin_amdgcn_ds_read_tr16_b64_v4i16(
        (__attribute__((address_space(3))) s16x4 *)(uintptr_t)p);
}

// Operand fragment (A or B of mfma32) whose k index runs over the ROWS of a row-major LDS
// tile and whose free index (32 wide) runs over its columns: for lane l the fragment holds
// tile[row0 + kmap(j)][col0 + l % 32], j = 0..7, with kmap(j) = 4*hl + j for j < 4 and
// 8 + 4*hl + (j - 4) for j >= 4 -- the order in which a 32x32 accumulator keeps its rows,
// so an accumulator block can be the other operand without any shuffle.
__device__ __forceinline__ bf16x8 lds_frag_tr(const uint16_t *tile, int stride, int row0, int col0, int lane)
{
    int i = lane & 15, gg = lane >> 4;
    int hl = gg >> 1;
    const uint16_t *p = tile + (row0 + 4 * hl + (i >> 2)) * stride + col0 + 16 * (gg & 1) + 4 * (i & 3);
    Frag8 f;
    f.h[0] = lds_read_tr(p);
    f.h[1] = lds_read_tr(p + 8 * stride);
    return f.v;
}

// Operand fragment whose k index runs along the columns of a row-major LDS tile (natural
// read): tile[row0 + l % 32][col0 + 8*hl .. + 7].
__device__ __forceinline__ bf16x8 lds_frag(const uint16_t *tile, int stride, int row0, int col0, int lane)
{
    const uint16_t *p = tile + (row0 + (lane & 31)) * stride + col0 + 8 * (lane >> 5);
    Frag8 f;
    f.u = *(const u32x4 *)p;
    return f.v;
}

// Epilogue store of a transposed accumulator (rows = head dim, column = this lane's token):
// register group i4 of block db holds head-dim elements db*32 + 8*i4 + 4*hl .. +3.
// `row` points at element 0 of the token's row; values are multiplied by `mul` first.
template <int DB>
__device__ __forceinline__ void store_rowT(void *row, bool f32, const f32x16 (&acc)[DB], float mul, int hl)
{
#pragma unroll
    for (int db = 0; db < DB; db++)
#pragma unroll
        for (int i4 = 0; i4 < 4; i4++) {
            const int d = db * 32 + 8 * i4 + 4 * hl;
            if (f32) {
                f32x4 w = {acc[db][4 * i4] * mul, acc[db][4 * i4 + 1] * mul, acc[db][4 * i4 + 2] * mul,
                           acc[db][4 * i4 + 3] * mul};
                *(f32x4 *)((float *)row + d) = w;
            } else {
                u32x2 w;
                w[0] = pack_bf16x2(acc[db][4 * i4] * mul, acc[db][4 * i4 + 1] * mul);
                w[1] = pack_bf16x2(acc[db][4 * i4 + 2] * mul, acc[db][4 * i4 + 3] * mul);
                *(u32x2 *)((uint16_t *)row + d) = w;
            }
        }
}

// Work queue: one queue per XCD.  Workgroup w starts on queue w % nq (workgroups are
// dispatched round-robin over the XCDs, so that is its own XCD's queue) and moves on to the
// next queue when one runs dry.  Returns the item index or -1 when every queue is empty.
// `cursor` counts how many queues this workgroup has exhausted.
__device__ __forceinline__ int queue_fetch(const PassQueues &pq, int &cursor)
{
    while (cursor < pq.nq) {
        int qx = (int)((blockIdx.x + cursor) % pq.nq);
        int begin = pq.offsets[qx], end = pq.offsets[qx + 1];
        if (begin < end) {
            int got = atomicAdd(&pq.counters[qx], 1);
            if (begin + got < end) return begin + got;
        }
        cursor++;
    }
    return -1;
}

// Called by one thread of every workgroup after its last fetch.  The last workgroup to
// arrive puts all counters back to zero, so the plan is ready for the next launch.
__device__ __forceinline__ void queue_retire(const PassQueues &pq)
{
    __threadfence();
    int done = atomicAdd(&pq.counters[pq.nq], 1);
    if (done == (int)gridDim.x - 1) {
        for (int x = 0; x <= pq.nq; x++) atomicExch(&pq.counters[x], 0);
        __threadfence();
    }
}

}  // namespace flexsp
