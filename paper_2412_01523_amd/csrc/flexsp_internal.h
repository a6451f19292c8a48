// Internal declarations shared by the host code and the kernels of libflexsp.
// Nothing here is part of the public ABI (see include/flexsp.h).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <cmath>
#include <cstring>

#include "flexsp.h"

namespace flexsp {

// Tile shapes.  The plan builder and the kernels must agree on these.
constexpr int kFwdBq = 128;    // query rows per forward work item (4 waves x 32 rows)
constexpr int kFwdBk = 64;     // key rows staged in LDS per forward step
constexpr int kDqBq = 128;     // query rows per dQ work item
constexpr int kDqBk = 64;      // key rows per dQ step
constexpr int kDkvBk = 64;     // key rows per dK/dV work item (2 pairs of waves x 32 rows)
constexpr int kDkvBq = 64;     // query rows per dK/dV step
constexpr int kThreads = 256;  // every attention kernel runs 4 wavefronts per workgroup
constexpr int kMaxQueues = 8;  // one work queue per XCD
constexpr int kCounterStride = 32;  // int32 from one queue's ticket counter to the next: a 128-byte line each
constexpr int kLateTicketSteps = 16;  // items of at least this many steps draw the next ticket near their end

// Split tiles (see flexsp_item in flexsp.h): a part's partial result is one record of fp32 values,
// 64 per thread of the workgroup (the accumulators) plus, for the forward, each row's running
// maximum and sum.  kMinPartSteps: no part is made shorter than this many inner-loop steps (the
// hand-over costs about as much as two or three steps); at most kMaxParts parts per tile and
// kMaxSplitRecords records per pass.
constexpr int kPartialBytes = 64 * kThreads * 4 + 2 * kThreads * 4;  // 67 584 B
constexpr int kMinPartSteps = 16;
constexpr int kGroupMajorSteps = 24;  // sequences whose longest tile has at most this many steps are queued tile beside tile
constexpr int kLongPartSteps = 160;  // parts at least this long are aimed at 35 % of an even share instead of 75 %
constexpr int kMaxParts = 8;
constexpr int kMaxSplitRecords = 2048;

// Work item of the key-shard forward: query rows q_start .. q_start+q_len-1 of q / o / lse, shard
// keys k_start .. k_start+k_len-1 of k / v, shift = position of the first query in its sequence
// minus position of the shard's first key.  `tile` counts 128-row query tiles.
// A tile cut into parts (see flexsp_item) is listed once per part, each with its own key range and the
// shift that goes with it: head_parts = head | part << 16 | nparts << 24 (0 and 1 for a whole tile),
// slot = the tile's first partial-result record (-1 for a whole tile).
struct flexsp_shard_item {
    int32_t q_start, q_len, k_start, k_len, shift, tile, head_parts, slot;
};

struct PassQueues {
    const flexsp_item *items;  // device, all queues back to back
    const int32_t *offsets;    // device, nq + 1 boundaries into items
    int32_t *counters;         // device, nq fetch counters + 1 "workgroups done" counter, kCounterStride apart
    int32_t nq;
    int32_t *split_flags;      // device, one arrival counter per partial-result record (a tile uses its first record's)
    char *split_scratch;       // device, kPartialBytes per record
};

// Arguments of the attention kernels.  Strides are in elements; pointers already include
// the first head of the subset.
struct AttnArgs {
    const uint16_t *q, *k, *v, *o, *dO;
    uint16_t *out_o;
    void *dq, *dk, *dv;  // bf16 or fp32 elements, see grad_f32
    const float *lse_in, *delta_in;
    float *lse_out, *delta_out;
    // strides in elements; 32-bit (checked by the host) to keep the kernels' scalar registers free
    int32_t q_st, q_sh, k_st, k_sh, v_st, v_sh, o_st, o_sh, do_st, do_sh;
    int32_t dq_st, dq_sh, dk_st, dk_sh, dv_st, dv_sh;
    int32_t T;       // tokens in the packed stream (row length of lse / delta)
    int32_t Hq;      // query heads in the subset
    int32_t G;       // query heads per kv head
    int32_t causal;
    int32_t grad_f32;  // bit 0: gradients are stored as fp32 instead of bf16; bit 1 (key-shard kernels): added to what is there
    float scale;     // softmax scale
    float scale_l2;  // scale * log2(e)
    PassQueues pq;
};

// Launchers implemented next to their kernels.  All are asynchronous on `s`.
hipError_t launch_pack(const void *src, void *dst, int64_t T, int H, int D, int P, int eb,
                       bool unpack, hipStream_t s);
hipError_t launch_pack_many(int n, const void *const *src, void *const *dst, int64_t T, const int32_t *H, int D,
                            int P, int eb, bool unpack, hipStream_t s);
hipError_t launch_attn_fwd(const AttnArgs &a, int D, int grid, hipStream_t s);
hipError_t launch_attn_fwd_kvshard(const AttnArgs &a, int D, int grid, hipStream_t s);  // a.pq.items: flexsp_shard_item
hipError_t launch_lse_merge(const uint16_t *oa, const float *la, const uint16_t *ob, const float *lb, uint16_t *oo,
                            float *lo, int64_t T, int H, int D, int32_t oa_st, int32_t oa_sh, int32_t ob_st,
                            int32_t ob_sh, int32_t oo_st, int32_t oo_sh, hipStream_t s);
hipError_t launch_lse_merge_acc(float *oacc, float *lacc, const uint16_t *ob, const float *lb, uint16_t *ob16, int64_t T,
                                int H, int D, int32_t oa_st, int32_t oa_sh, int32_t ob_st, int32_t ob_sh, int32_t o16_st,
                                int32_t o16_sh, hipStream_t s);
hipError_t launch_attn_bwd_dkv(const AttnArgs &a, int D, int grid, hipStream_t s);
hipError_t launch_attn_bwd_dq(const AttnArgs &a, int D, int grid, hipStream_t s);
hipError_t launch_attn_bwd_dkv_kvshard(const AttnArgs &a, int D, int grid, hipStream_t s);  // a.pq.items: flexsp_shard_item;
hipError_t launch_attn_bwd_dq_kvshard(const AttnArgs &a, int D, int grid, hipStream_t s);   // a.grad_f32 bit 1: add to dq / dk / dv

// Host helpers shared by the files that hold entry points.
int ctx_device(const flexsp_ctx *ctx);        // HIP device of a context, -1 for a host-only one
int hip_status(hipError_t e);                 // records e for flexsp_last_hip_error, returns the flexsp_status for it
hipError_t static_scratch_init(int device);   // resolves the device's copy of the no-allocation scratch array

// A view the attention kernels can address: 16-byte aligned rows, strides that fit the kernels'
// 32-bit arithmetic (a per-lane byte offset spans up to 64 token rows).
inline bool view_ok(const flexsp_tensor &t)
{
    if (!t.ptr) return false;
    if (((uintptr_t)t.ptr & 15) != 0) return false;
    if (t.stride_token <= 0 || t.stride_head <= 0) return false;
    if ((t.stride_token % 8) != 0 || (t.stride_head % 8) != 0) return false;
    if (t.stride_token > (1 << 24) || t.stride_head > 0x3fffffff) return false;
    return true;
}

}  // namespace flexsp
