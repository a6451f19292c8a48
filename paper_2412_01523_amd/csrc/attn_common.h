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

// acc + lo + hi of a packed bf16 pair (v_dot2_f32_bf16 against {1, 1}).
__device__ __forceinline__ float add_bf16x2(uint32_t pk, float acc)
{
    return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, pk), __builtin_bit_cast(bf16x2, 0x3f803f80u),
                                           acc, false);
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

// ------------------------------------------------------------------------------------------
// LDS tiles.  A tile holds rows of D bf16 (D*2 bytes, no padding) as 16-byte chunks; the chunk
// index is XOR-swizzled with a function of the row so that both access patterns below touch
// every bank once:
//   natural read  (ds_read_b128): 16 lanes read the same chunk of 16 consecutive rows;
//   transpose read (ds_read_b64_tr_b16): 32 lanes read 4 consecutive chunks of 4 consecutive rows.
// For D = 128 (16 chunks per row) the swizzle swaps the two 2-bit fields of row % 16; for D = 64
// (8 chunks, two rows per 256 bytes) it uses row bits 1..3.
template <int D>
struct LdsTile {
    static constexpr int CH = D / 8;    // 16-byte chunks per row
    static constexpr int ROWB = D * 2;  // bytes per row
    __device__ static __forceinline__ int sw(int row)
    {
        return D == 128 ? (((row & 3) << 2) | ((row >> 2) & 3)) : ((((row >> 1) & 1) << 2) | ((row >> 2) & 3));
    }
};

typedef __attribute__((address_space(3))) void lds_void_t;
typedef __attribute__((address_space(1))) const void glb_void_t;

// 16 bytes per lane straight from global memory into LDS: lane l's data lands at lds + 16*l.
// `lds` must be wave-uniform.  Completion is tracked by vmcnt.
// Issued as inline assembly on purpose: when the compiler knows that a copy into LDS is in
// flight it makes every later LDS read wait for ALL outstanding copies (it cannot tell that
// the copy fills the other buffer), which would stall each tile step on the prefetch of the
// next tile.  The one real dependency, tile t landed before step t reads it, is the explicit
// wait_vmem() + barrier at the top of a step.
__device__ __forceinline__ void global_to_lds16(const void *g, void *lds)
{
    const uint32_t dst = (uint32_t)(uintptr_t)lds;  // low half of a generic LDS pointer = LDS byte address
    asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" ::"v"(g), "s"(dst) : "memory");
}
// The same with the address split into a wave-uniform 64-bit base (scalar registers) and a
// 32-bit per-lane byte offset: the per-lane part of a tile copy is then one register for the
// whole kernel instead of one 64-bit address per copy instruction.
__device__ __forceinline__ void global_to_lds16(const void *base, uint32_t lane_off, void *lds)
{
    const uint32_t dst = (uint32_t)(uintptr_t)lds;
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1" ::"v"(lane_off), "s"(base), "s"(dst)
                 : "memory");
}
__device__ __forceinline__ void global_to_lds4(const void *g, void *lds)
{
    const uint32_t dst = (uint32_t)(uintptr_t)lds;
    asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dword %0, off" ::"v"(g), "s"(dst) : "memory");
}
__device__ __forceinline__ void wait_vmem() { __builtin_amdgcn_s_waitcnt(0x0F70); }  // vmcnt(0)

// Workgroup barrier that does NOT wait for this wavefront's outstanding global stores.  Used at
// the end of a work item, where __syncthreads() would stall every wavefront until the item's
// output rows have been acknowledged by memory (microseconds).  It orders LDS use only: a
// wavefront reaches it after the matrix instructions that consumed its last LDS reads were
// issued, so those reads have completed, and the next item may overwrite the tiles.
__device__ __forceinline__ void barrier_lds_only() { __builtin_amdgcn_s_barrier(); }

// Copies ROWS rows of a row-major global matrix (row r at g + r*stride elements, D bf16 each)
// into a swizzled LDS tile, asynchronously, with all 256 threads.  Row `first + r` is clamped to
// `last_valid`, so rows past the end of a sequence duplicate its last row (finite data; callers
// mask them).
template <int D, int ROWS>
__device__ __forceinline__ void load_tile_async(char *tile, const uint16_t *g, int32_t stride, int first,
                                                int last_valid, int wave, int lane)
{
    typedef LdsTile<D> L;
    constexpr int N = ROWS * L::CH / kThreads;
    static_assert(N >= 1 && ROWS * L::CH % kThreads == 0, "tile must split evenly over the workgroup");
#pragma unroll
    for (int n = 0; n < N; n++) {
        const int pos = n * kThreads + wave * 64 + lane;
        const int row = pos / L::CH;
        const int c = (pos % L::CH) ^ L::sw(row);
        const int grow = min(first + row, last_valid);
        global_to_lds16(g + (int64_t)grow * stride + c * 8, tile + (n * kThreads + wave * 64) * 16);
    }
}

// The same copy without the clamp, for tiles that lie wholly inside the sequence.  Chunk n of a
// lane lies kThreads/CH rows below chunk n-1 in the same (swizzled) column, because the swizzle
// has a period of 16 rows; so one per-lane byte offset (tile_goff, computed once per item) plus
// wave-uniform addresses describe the whole copy, and it costs no vector address arithmetic.
template <int D>
__device__ __forceinline__ uint32_t tile_goff(int32_t stride, int wave, int lane)
{
    typedef LdsTile<D> L;
    const int pos = wave * 64 + lane;
    const int row = pos / L::CH;
    const int c = (pos % L::CH) ^ L::sw(row);
    return (uint32_t)(row * (uint32_t)stride * 2u + c * 16);
}
template <int D, int ROWS>
__device__ __forceinline__ void load_tile_async_fast(char *tile, const uint16_t *g_tile, int32_t stride,
                                                     uint32_t goff, int wave)
{
    typedef LdsTile<D> L;
    static_assert((kThreads / L::CH) % 16 == 0, "rows per pass must be a multiple of the swizzle period");
#pragma unroll
    for (int n = 0; n < ROWS * L::CH / kThreads; n++)
        global_to_lds16(g_tile + (int64_t)n * (kThreads / L::CH) * stride, goff, tile + (n * kThreads + wave * 64) * 16);
}

// One of the ROWS*CH/kThreads copy instructions of load_tile_async_fast (n is a compile-time
// constant at every call site).  Lets a kernel place the copies of the next tile one by one
// between its matrix instructions: issued back to back by all wavefronts right after the
// barrier they queue up behind the 64 bytes per cycle a compute unit's load path delivers, and
// every wavefront stalls until its own have been accepted.
template <int D>
__device__ __forceinline__ void load_tile_async_fast_one(char *tile, const uint16_t *g_tile, int32_t stride,
                                                         uint32_t goff, int wave, int n)
{
    typedef LdsTile<D> L;
    global_to_lds16(g_tile + (int64_t)n * (kThreads / L::CH) * stride, goff, tile + (n * kThreads + wave * 64) * 16);
}

// Per-lane byte offsets of operand fragments inside a tile (computed once per kernel).
//   nat[ks]: fragment whose k index runs along the columns: rows rb*32 + l%32 (add rb*32*ROWB),
//            columns 16*ks + 8*hl .. +7.
//   tr[db][h]: fragment whose k index runs over ROWS (transpose read) and whose free index is
//            columns db*32 + l%32: lane's first (h=0) / second (h=1) 4-row read; for k slot j the
//            row is R0 + kmap(j), kmap(j) = 4*hl + j (j<4), 8 + 4*hl + (j-4) (j>=4): the order in
//            which a 32x32 accumulator keeps its rows, so an accumulator block can be the other
//            operand without a shuffle.  Add R0*ROWB with R0 a multiple of 16.
template <int D>
struct LaneOffsets {
    int nat[D / 16];
    int tr[D / 32][2];
    // Makes the offsets opaque to the optimiser at this point.  Called once per tile step: the
    // addresses of a step are then "offset register + compile-time constant", which folds into the
    // LDS instructions' immediate field, instead of being hoisted out of the tile loop as dozens
    // of precomputed address registers.  Emits no instruction.
    __device__ __forceinline__ void pin()
    {
#pragma unroll
        for (int ks = 0; ks < D / 16; ks++) asm volatile("" : "+v"(nat[ks]));
#pragma unroll
        for (int db = 0; db < D / 32; db++) {
            asm volatile("" : "+v"(tr[db][0]));
            asm volatile("" : "+v"(tr[db][1]));
        }
    }
    __device__ __forceinline__ void init(int lane)
    {
        typedef LdsTile<D> L;
        const int r = lane & 31, hl = lane >> 5;
#pragma unroll
        for (int ks = 0; ks < D / 16; ks++) nat[ks] = r * L::ROWB + (((2 * ks + hl) ^ L::sw(r)) << 4);
        const int i = lane & 15, gg = lane >> 4;
        const int cl = 2 * (gg & 1) + ((i & 3) >> 1);
#pragma unroll
        for (int db = 0; db < D / 32; db++)
#pragma unroll
            for (int h = 0; h < 2; h++) {
                const int row = 4 * hl + (i >> 2) + 8 * h;
                tr[db][h] = row * L::ROWB + (((4 * db + cl) ^ L::sw(row)) << 4) + (i & 1) * 8;
            }
    }
};

__device__ __forceinline__ bf16x8 lds_nat(const char *tile, int off)
{
    Frag8 f;
    f.u = *(const u32x4 *)(tile + off);
    return f.v;
}
__device__ __forceinline__ bf16x8 lds_tr(const char *tile, int off0, int off1)
{
    Frag8 f;
    f.h[0] = lds_read_tr((const uint16_t *)(tile + off0));
    f.h[1] = lds_read_tr((const uint16_t *)(tile + off1));
    return f.v;
}

// 32 consecutive rows of a row-major global matrix (D bf16 each) as the operand fragments of a
// wavefront: f[ks] of lane (r = l % 32, hl = l / 32) holds elements 16*ks + 8*hl .. +7 of row r.
// Loading a fragment straight from global memory makes every lane of an instruction touch a
// different row (32 rows, 32 bytes of each): the load path takes such an instruction apart lane by
// lane, and the 8 (D = 128) of them per operand cost a wavefront microseconds at the start of every
// work item.  Here the rows are read with whole-row instructions (lane l of piece n reads 16-byte
// chunk (64n + l) % CH of row (64n + l) / CH: 1 KiB contiguous per instruction for D = 128) and
// turned into fragments through a wave-private LDS region of 32 rows, laid out like a tile.
// Rows past `last_valid` read as zeros (callers never store their results).
template <int D>
struct RowBlock {
    typedef LdsTile<D> L;
    static constexpr int N = 32 * L::CH / 64;  // 16-byte pieces per lane
    u32x4 raw[N];
    // g: row 0 of the sequence at the wanted head (wave-uniform, like first and last_valid); issues
    // the loads, waits for nothing.  Buffer loads: one wave-uniform descriptor of the block (its first
    // row's address, the bytes up to the end of the sequence) and one per-lane byte offset serve all
    // pieces, so there is no per-lane 64-bit address arithmetic, and the bounds check of the hardware
    // returns zeros for rows past the sequence.
    __device__ __forceinline__ void load(const uint16_t *g, int64_t stride, int first, int last_valid, int lane)
    {
        const int nrows = min(last_valid - first + 1, 32);
        const uint32_t rowb = (uint32_t)stride * 2u;  // bytes from row to row
        const __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc(
            (void *)(g + (int64_t)first * stride), 0, nrows > 0 ? (int)(nrows * rowb) : 0, 0x00020000);
        const uint32_t off = (uint32_t)(lane / L::CH) * rowb + (uint32_t)(lane % L::CH) * 16u;
#pragma unroll
        for (int n = 0; n < N; n++) raw[n] = __builtin_amdgcn_raw_buffer_load_b128(rsrc, off, n * (64 / L::CH) * rowb, 0);
    }
    // The block is kept in rows row0 .. row0+31 (row0 a multiple of 32) of the tile-shaped LDS area
    // `tile`, which nobody else touches until this wavefront's next barrier; lo.nat must point at
    // those rows of a tile (kernels that fold a row offset into lo.nat pass the same offset here).
    __device__ __forceinline__ void fragments(char *tile, int row0, const LaneOffsets<D> &lo, bf16x8 (&f)[D / 16], int lane)
    {
        stage(tile, row0, lane);
        // (LDS instructions of one wavefront execute in order: the reads see the writes, and a later
        // call's writes to the same region come after these reads)
#pragma unroll
        for (int ks = 0; ks < D / 16; ks++) f[ks] = lds_nat(tile, lo.nat[ks]);
    }
    // The first half of fragments(): the block as 32 rows of a tile, for code that reads it with the
    // tile read patterns itself.
    __device__ __forceinline__ void stage(char *tile, int row0, int lane)
    {
        char *region = tile + row0 * L::ROWB;
#pragma unroll
        for (int n = 0; n < N; n++) {
            const int pos = n * 64 + lane;
            const int row = pos / L::CH;
            *(u32x4 *)(region + row * L::ROWB + (((pos % L::CH) ^ L::sw(row)) << 4)) = raw[n];
        }
    }
};

// max / sum across the two half-waves: every lane gets op(x[l % 32], x[l % 32 + 32]).
// v_permlane32_swap exchanges the upper half of its first operand with the lower half of its
// second; fed the same value twice it returns {x[l % 32], x[l % 32 + 32]} in every lane.
// (The two results are copied into scalars before the bit casts: casting the vector's elements
// in place made the compiler read element 0 twice.)
__device__ __forceinline__ void halves_both(float x, float &lo, float &hi)
{
    const unsigned a = __builtin_bit_cast(unsigned, x);
    auto r = __builtin_amdgcn_permlane32_swap(a, a, false, false);
    const unsigned r0 = r[0], r1 = r[1];
    lo = __builtin_bit_cast(float, r0);
    hi = __builtin_bit_cast(float, r1);
}
__device__ __forceinline__ float halves_max(float x)
{
    float lo, hi;
    halves_both(x, lo, hi);
    return fmaxf(lo, hi);
}
__device__ __forceinline__ float halves_sum(float x)
{
    float lo, hi;
    halves_both(x, lo, hi);
    return lo + hi;
}

// (Outputs are written with non-temporal stores here and below: they are not read again by the
// kernel that writes them, and the K/V and Q/dO tiles the workgroups share keep their place in L2;
// worth about 1 % on batches of short sequences.  The same hint on the per-item row loads cost up
// to 8 %.)
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
                __builtin_nontemporal_store(w, (f32x4 *)((float *)row + d));
            } else {
                u32x2 w;
                w[0] = pack_bf16x2(acc[db][4 * i4] * mul, acc[db][4 * i4 + 1] * mul);
                w[1] = pack_bf16x2(acc[db][4 * i4 + 2] * mul, acc[db][4 * i4 + 3] * mul);
                __builtin_nontemporal_store(w, (u32x2 *)((uint16_t *)row + d));
            }
        }
}

// The same for fp32 rows that already hold a partial sum: row += acc * mul (each lane owns its
// row's elements, so the read-modify-write races with nobody inside the kernel).
template <int DB>
__device__ __forceinline__ void add_rowT_f32(float *row, const f32x16 (&acc)[DB], float mul, int hl)
{
#pragma unroll
    for (int db = 0; db < DB; db++)
#pragma unroll
        for (int i4 = 0; i4 < 4; i4++) {
            f32x4 *p = (f32x4 *)(row + db * 32 + 8 * i4 + 4 * hl);
            f32x4 w = *p;
#pragma unroll
            for (int e = 0; e < 4; e++) w[e] += acc[db][4 * i4 + e] * mul;
            *p = w;
        }
}

// Epilogue store of a transposed accumulator as bf16 THROUGH LDS, so that global memory sees
// whole 16-byte pieces of contiguous rows instead of 8-byte pieces scattered over 32 rows (which
// the address coalescer handles one lane at a time: thousands of cycles per item).
//   acc      NB blocks; lane l holds token row l % 32, head-dim elements db*32 + 8*i4 + 4*hl + e
//   stage    wave-private LDS, 32 rows x ROWB bytes (ROWB = NB*64); chunk c of row r is kept at
//            position c ^ (r & (CH-1)) so that the column-wise writes spread over the banks
//   g        address of the first token row (this wavefront's row 0) + first head-dim element
//   stride   token stride in elements;  nrows  rows of this wavefront inside the sequence
template <int NB>
__device__ __forceinline__ void store_rowT_bf16_lds(char *stage, uint16_t *g, int64_t stride, int nrows,
                                                    const f32x16 (&acc)[NB], float mul, int lane)
{
    constexpr int ROWB = NB * 64;   // bytes per staged row
    constexpr int CH = ROWB / 16;   // 16-byte chunks per row
    // opaque copy: keeps the address arithmetic below here, inside the epilogue, instead of being
    // hoisted to the top of the kernel where its results would occupy registers for good
    asm volatile("" : "+v"(lane));
    const int r = lane & 31, hl = lane >> 5;
#pragma unroll
    for (int db = 0; db < NB; db++)
#pragma unroll
        for (int i4 = 0; i4 < 4; i4++) {
            u32x2 w;
            w[0] = pack_bf16x2(acc[db][4 * i4] * mul, acc[db][4 * i4 + 1] * mul);
            w[1] = pack_bf16x2(acc[db][4 * i4 + 2] * mul, acc[db][4 * i4 + 3] * mul);
            const int c = (4 * db + i4) ^ (r & (CH - 1));
            *(u32x2 *)(stage + r * ROWB + c * 16 + 8 * hl) = w;
        }
    // the wavefront reads back what it wrote: no barrier, just LDS ordering within the wave
#pragma unroll
    for (int n = 0; n < 32 * CH / 64; n++) {
        const int pos = n * 64 + lane;
        const int row = pos / CH;
        const int c = (pos % CH) ^ (row & (CH - 1));
        const u32x4 v = *(const u32x4 *)(stage + pos * 16);
        if (row < nrows) __builtin_nontemporal_store(v, (u32x4 *)(g + (int64_t)row * stride + c * 8));
    }
}

// Descriptor of item `idx` as wave-uniform (scalar) values.  The index is uniform, but the load
// itself is a vector load (the compiler cannot rule out that the kernel's own stores clobber the
// list), so without the readfirstlane every quantity derived from the descriptor - sequence
// length, tile bounds, loop trip counts, base addresses - would live in vector registers and
// every branch on them would be compiled as a divergent one.
__device__ __forceinline__ flexsp_item load_item(const flexsp_item *items, int idx)
{
    const flexsp_item v = items[idx];
    flexsp_item it;
    it.seq_start = __builtin_amdgcn_readfirstlane(v.seq_start);
    it.seq_len = __builtin_amdgcn_readfirstlane(v.seq_len);
    it.tile = __builtin_amdgcn_readfirstlane(v.tile);
    it.head = __builtin_amdgcn_readfirstlane(v.head);
    it.step_begin = __builtin_amdgcn_readfirstlane(v.step_begin);
    it.step_end = __builtin_amdgcn_readfirstlane(v.step_end);
    it.slot = __builtin_amdgcn_readfirstlane(v.slot);
    it.parts = __builtin_amdgcn_readfirstlane(v.parts);
    return it;
}

// ------------------------------------------------------------------------------------------
// Split tiles.  A tile whose inner loop was cut into parts (flexsp_item::parts names more than one) is finished
// by whichever part arrives last; nobody waits for anybody.  Every part
//   1. stores its accumulators to its own record of the plan's scratch (split_store),
//   2. waits until those stores have completed and counts itself in (split_arrive),
// and the part that finds all others counted already re-reads ALL records in part order, its own
// included (split_sum), so the sum is formed in one fixed order whichever part does it: results
// stay bitwise reproducible.  It also clears the counter for the next launch.
// The parts of a tile may run on different XCDs, whose L2 caches do not see each other's dirty
// lines.  A device-wide fence would write back and invalidate a whole L2 (and with it the K/V tiles
// every other workgroup of that XCD is streaming through it; measured: a batch with many cut tiles
// ran 30 % slower than with no cutting at all).  So the records are written and read with
// device-scope relaxed atomic accesses instead, which go through to memory and come from memory
// on their own and leave the caches alone; a record store is complete when its counter reaches zero.
// Record layout: value i of thread t at float index i * kThreads + t; the forward appends 2 floats
// per thread (row maximum, row sum) from index 64 * kThreads on.
__device__ __forceinline__ void split_put(float *p, float v)
{
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float split_get(const float *p)
{
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
template <int NB>
__device__ __forceinline__ void split_store(char *rec, const f32x16 (&acc)[NB], int tid)
{
    float *r = (float *)rec + tid;
#pragma unroll
    for (int b = 0; b < NB; b++)
#pragma unroll
        for (int i = 0; i < 16; i++) split_put(r + (b * 16 + i) * kThreads, acc[b][i]);
}
template <int NB>
__device__ __forceinline__ void split_sum(const char *rec, f32x16 (&acc)[NB], float mul, int tid)
{
    const float *r = (const float *)rec + tid;
    // every load of the record in flight, then the additions (these files are compiled in source
    // order: a load followed by its use would wait out one trip to memory per value)
    float v[NB * 16];
#pragma unroll
    for (int i = 0; i < NB * 16; i++) v[i] = split_get(r + i * kThreads);
#pragma unroll
    for (int b = 0; b < NB; b++)
#pragma unroll
        for (int i = 0; i < 16; i++) acc[b][i] += mul * v[b * 16 + i];
}
// Returns true in every thread of the workgroup iff this part is the last of its tile to arrive.
// Contains two workgroup barriers; `word` is an LDS word of the caller's.
__device__ __forceinline__ bool split_arrive(int32_t *flag, int nparts, int *word, int tid)
{
    __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0): this thread's record stores have completed
    __syncthreads();                     // ... and everybody's
    if (tid == 0) {
        const int seen = __hip_atomic_fetch_add(flag, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (seen == nparts - 1)  // everybody has arrived: ready for the next launch
            __hip_atomic_store(flag, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        *word = seen;
    }
    __syncthreads();
    return *(volatile int *)word == nparts - 1;  // the records are read after this, by the same kind of access
}

__device__ __forceinline__ flexsp_shard_item load_shard_item(const flexsp_shard_item *items, int idx)
{
    const flexsp_shard_item v = items[idx];
    flexsp_shard_item it;
    it.q_start = __builtin_amdgcn_readfirstlane(v.q_start);
    it.q_len = __builtin_amdgcn_readfirstlane(v.q_len);
    it.k_start = __builtin_amdgcn_readfirstlane(v.k_start);
    it.k_len = __builtin_amdgcn_readfirstlane(v.k_len);
    it.shift = __builtin_amdgcn_readfirstlane(v.shift);
    it.tile = __builtin_amdgcn_readfirstlane(v.tile);
    it.head_parts = __builtin_amdgcn_readfirstlane(v.head_parts);
    it.slot = __builtin_amdgcn_readfirstlane(v.slot);
    return it;
}

// Work distribution.  The plan holds one longest-first item list per XCD, balanced on the host.
// Workgroup w runs on XCD w % nq (workgroups are dispatched round-robin over the XCDs); that
// list is its home queue, and it is the (w / nq)-th of the W workgroups there.  Items are handed
// out as tickets: ticket l < W is workgroup l's first item (no memory access), tickets from W on
// come from one atomic counter per queue, longest item first, so the list is scheduled
// longest-processing-time-first against the run times as they really turn out.  The ticket for
// the NEXT item is drawn while an item runs (prefetch), so the counter's round trip (a few
// microseconds when 64 workgroups hit the same address) is hidden behind the item's work.  A
// workgroup whose home queue is empty takes items from the fullest of the other XCDs' queues
// and only stops when all are empty: the tail of the launch is spread over the whole chip.
// Only wavefront 0 talks to the counters; the item index reaches the others through one LDS
// word and the barrier that ends an item anyway.  The last workgroup to leave zeroes the
// counters, so a launch (or a graph replay of it) always finds them clear; launches that share
// a plan's counters must not overlap.
struct ItemDealer {
    const int32_t *offsets;
    int32_t *counters;  // kCounterStride apart (a line of their own each: they are hammered from all
                        // compute dies at once): [q] tickets drawn beyond the static ones, [nq] workgroups that left
    int *slot;          // LDS word
    int nq, q, wave, lane;
    int pending;        // wavefront 0, lane 0: ticket drawn ahead (offset from W of queue q)

    __device__ __forceinline__ int wgs_of(int qq) const { return ((int)gridDim.x - qq + nq - 1) / nq; }
    __device__ __forceinline__ int draw(int qq)  // wavefront 0 only; waits for the answer
    {
        int tk = 0;
        if (lane == 0) tk = atomicAdd(counters + qq * kCounterStride, 1);
        return __builtin_amdgcn_readfirstlane(tk);
    }
    // wavefront 0: an item of another queue, or -1 when all are empty.  Looks before it draws: one
    // load of all counters, then a ticket from the queue with the most items left (ties: the next in
    // ring order), again if somebody else emptied that queue meanwhile.  Drawing from the queues one
    // after the other instead made every leaving workgroup send a read-modify-write to every
    // counter: at the end of a pass thousands of them queue up on a handful of addresses, and the
    // loads of the items still running wait behind them (their last items took twice as long).
    __device__ __forceinline__ int steal()
    {
        // (every failed try means that another workgroup emptied a queue in between, so the tries
        // end by themselves; the bound is a belt to the braces)
        for (int tries = 0; tries < 4 * kMaxQueues; tries++) {
            // lanes 0 .. nq-1 (nq <= 8) look at one queue each; the key orders the queues by items left,
            // then by ring distance from this workgroup's queue, and carries the queue's number
            int l = lane;
            asm volatile("" : "+v"(l));  // (keeps this arithmetic here: it is loop-invariant and would be hoisted into long-lived registers)
            int key = 0;
            if (l < nq) {
                const int drawn = __hip_atomic_load(counters + l * kCounterStride, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                const int left = offsets[l + 1] - offsets[l] - wgs_of(l) - drawn;
                const int dist = l > q ? l - q : l - q + nq;  // 1 .. nq
                key = left > 0 ? (min(left, 0xFFFFF) << 8) | ((8 - dist) << 4) | l : 0;
            }
            // maximum over lanes 0 .. 7: lane ^ 1, lane ^ 2, then the mirrored half row
            key = max(key, __builtin_amdgcn_update_dpp(0, key, 0xB1, 0xF, 0xF, true));
            key = max(key, __builtin_amdgcn_update_dpp(0, key, 0x4E, 0xF, 0xF, true));
            key = max(key, __builtin_amdgcn_update_dpp(0, key, 0x141, 0xF, 0xF, true));
            key = __builtin_amdgcn_readfirstlane(key);
            if (key == 0) return -1;
            q = key & 15;
            const int idx = offsets[q] + wgs_of(q) + draw(q);
            if (idx < offsets[q + 1]) return idx;
        }
        return -1;
    }
    // hands wavefront 0's `idx` to the whole workgroup; contains the barrier that separates items
    __device__ __forceinline__ int publish(int idx)
    {
        if (wave == 0 && lane == 0) *slot = idx;
        __builtin_amdgcn_s_waitcnt(0xC07F);  // lgkmcnt(0): the LDS write is done (global stores may still be in flight)
        __builtin_amdgcn_s_barrier();
        const int v = *(volatile int *)slot;
        return __builtin_amdgcn_readfirstlane(v);
    }
    __device__ __forceinline__ int first(const PassQueues &pq, int *lds_word, int wave_, int lane_)
    {
        offsets = pq.offsets;
        counters = pq.counters;
        slot = lds_word;
        nq = pq.nq;
        wave = wave_;
        lane = lane_;
        q = (int)(blockIdx.x % pq.nq);
        pending = 0;
        int idx = -1;
        if (wave == 0) {
            idx = offsets[q] + (int)(blockIdx.x / pq.nq);
            if (idx >= offsets[q + 1]) idx = steal();
        }
        return publish(idx);
    }
    // call when an item starts: draws the ticket of the item after it
    __device__ __forceinline__ void prefetch()
    {
        if (wave == 0 && lane == 0) pending = atomicAdd(counters + q * kCounterStride, 1);
    }
    // call when an item is done (all of the workgroup's LDS reads issued): next item or -1
    __device__ __forceinline__ int advance()
    {
        int idx = -1;
        if (wave == 0) {
            idx = offsets[q] + wgs_of(q) + __builtin_amdgcn_readfirstlane(pending);
            if (idx >= offsets[q + 1]) idx = steal();
        }
        return publish(idx);
    }
    // call once, after the last item
    // The last workgroup to leave clears the counters for the next launch.  No fence: every ticket a
    // workgroup drew has come back before it gets here (it used the values), this counter's own
    // atomic orders the workgroups, and the clearing stores go to memory like the atomics do.  (A
    // device-scope fence writes back and invalidates the L2 of the compute die it runs on, once per
    // leaving workgroup: the workgroups still running then find their tiles gone from the cache.)
    __device__ __forceinline__ void finish()
    {
        if (wave == 0 && lane == 0) {
            if (atomicAdd(counters + nq * kCounterStride, 1) == (int)gridDim.x - 1)
                for (int i = 0; i <= nq; i++) __hip_atomic_store(counters + i * kCounterStride, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    }
};

}  // namespace flexsp
