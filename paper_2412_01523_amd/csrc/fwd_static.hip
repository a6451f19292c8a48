// flexsp_attn_varlen_fwd_static: the forward of packed attention for callers that cannot
// allocate (code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc).
// It needs no plan: the work queues the forward kernel consumes are built ON THE DEVICE, from the
// device copy of cu_seqlens, into a file-scope array that every GPU the library runs on holds
// until the process ends.  The attention kernel itself is the one flexsp_attn_varlen_fwd launches.
#include <mutex>

#include "flexsp_internal.h"

using namespace flexsp;

namespace {

// ---------------------------------------------------------------------------- the scratch
constexpr int kStaticMaxItems = 65536;   // work items (128 query rows of one head each) per call
constexpr int kStaticMaxLevels = 4096;   // query tiles per sequence: sequences up to 524 288 tokens
constexpr int kCountersOff = 0;          // kMaxQueues ticket counters + "workgroups done", kCounterStride int32 apart
constexpr int kOffsetsOff = (kMaxQueues + 1) * kCounterStride * 4;  // int32[16]: kMaxQueues + 1 queue boundaries
constexpr int kStatusOff = kOffsetsOff + 64;  // int32[2]: items listed by the last call, 1 if its lengths were rejected
constexpr int kItemsOff = kStatusOff + 64;
constexpr size_t kScratchBytes = kItemsOff + (size_t)kStaticMaxItems * sizeof(flexsp_item);

// One copy per GPU, at its own address.  In host code this name is only a handle for
// hipGetSymbolAddress; kernels and copies use the resolved pointer (g_scratch_ptr).
static __device__ __align__(256) unsigned char scratch[kScratchBytes];

constexpr int kMaxDevices = 64;
void *g_scratch_ptr[kMaxDevices];
std::mutex g_scratch_mutex;

// ---------------------------------------------------------------------------- queue builder
// One workgroup lists every (sequence, query tile, head) item of the batch, most expensive first,
// and deals the list round-robin into the kMaxQueues queues the forward kernel reads, so every
// queue is itself ordered longest first and the queues are level.  "Expensive" is the number of
// key tiles an item walks: tile index + 1 when causal (level = tile index), the sequence's tile
// count otherwise (level = tile count - 1).  Levels are bucket-sorted with LDS counters; the order
// of items inside a level is whatever the atomics give, which does not affect any result (items are
// independent).  Lengths are validated here, on the device: a cu_seqlens that is not 0 = cu[0] <=
// cu[1] <= ... <= cu[B] <= T, a sequence with more than kStaticMaxLevels tiles or a batch with more
// than kStaticMaxItems items publishes an EMPTY list (the attention kernel then touches nothing)
// and raises the status word.
constexpr int kBuildThreads = 1024;

__global__ __launch_bounds__(kBuildThreads) void build_static_queue_kernel(const int32_t *cu, int B, int T, int heads,
                                                                            int causal, int tile_rows,
                                                                            unsigned char *scr)
{
    __shared__ int hist[kStaticMaxLevels + 2];   // sequences with exactly n tiles
    __shared__ int start[kStaticMaxLevels + 1];  // first list position of a level
    __shared__ int fill[kStaticMaxLevels + 1];   // (sequence, tile) pairs placed in a level so far
    __shared__ int s_maxnt, s_bad, s_total;
    int32_t *counters = (int32_t *)(scr + kCountersOff);
    int32_t *offsets = (int32_t *)(scr + kOffsetsOff);
    int32_t *status = (int32_t *)(scr + kStatusOff);
    flexsp_item *items = (flexsp_item *)(scr + kItemsOff);
    const int tid = threadIdx.x;

    for (int i = tid; i < kStaticMaxLevels + 2; i += kBuildThreads) hist[i] = 0;
    for (int i = tid; i < kStaticMaxLevels + 1; i += kBuildThreads) fill[i] = 0;
    if (tid == 0) {
        s_maxnt = 0;
        s_bad = (B > 0 && cu[0] != 0) ? 1 : 0;
        s_total = 0;
    }
    if (tid <= kMaxQueues) counters[tid * kCounterStride] = 0;  // every call starts with clear tickets
    __syncthreads();

    for (int b = tid; b < B; b += kBuildThreads) {
        const int lo = cu[b], hi = cu[b + 1];
        if (lo < 0 || hi < lo || hi > T) {
            atomicOr(&s_bad, 1);
            continue;
        }
        const int nt = (hi - lo + tile_rows - 1) / tile_rows;
        if (nt > kStaticMaxLevels) {
            atomicOr(&s_bad, 1);
            continue;
        }
        if (nt > 0) {
            atomicAdd(&hist[nt], 1);
            atomicMax(&s_maxnt, nt);
        }
    }
    __syncthreads();

    if (tid == 0) {
        // levels in decreasing order of cost; pos counts (sequence, tile) pairs, heads come later
        const int maxnt = s_maxnt;
        int64_t pos = 0;
        int longer = 0;  // causal: sequences with more than t tiles
        for (int t = maxnt - 1; t >= 0; t--) {
            start[t] = (int)pos;
            if (causal) {
                longer += hist[t + 1];
                pos += longer;
            } else {
                pos += (int64_t)hist[t + 1] * (t + 1);
            }
            if (pos * heads > kStaticMaxItems) {
                s_bad = 1;
                break;
            }
        }
        s_total = s_bad ? 0 : (int)pos * heads;
    }
    __syncthreads();

    const int total = s_total, nq = kMaxQueues;
    if (tid <= nq) {
        // queue x holds list positions x, x + nq, x + 2 nq, ...
        const int x = tid;
        offsets[x] = x * (total / nq) + min(x, total % nq);
    }
    if (tid == 0) {
        status[0] = total;
        status[1] = s_bad;
    }
    if (total == 0) return;

    // one wavefront per sequence, its lanes over the sequence's tiles
    const int wave = tid >> 6, lane = tid & 63, nwaves = kBuildThreads >> 6;
    for (int b = wave; b < B; b += nwaves) {
        const int lo = cu[b], len = cu[b + 1] - lo;
        const int nt = (len + tile_rows - 1) / tile_rows;
        for (int t = lane; t < nt; t += 64) {
            const int level = causal ? t : nt - 1;
            const int slot = atomicAdd(&fill[level], 1);
            const int p0 = (start[level] + slot) * heads;
            for (int h = 0; h < heads; h++) {
                const int p = p0 + h;
                const int x = p % nq;
                flexsp_item it;
                it.seq_start = lo;
                it.seq_len = len;
                it.tile = t;
                it.head = h;
                // whole tiles only: every 64-key step the tile's rows can see
                it.step_begin = 0;
                it.step_end = ((causal ? min(len, (t + 1) * tile_rows) : len) + kFwdBk - 1) / kFwdBk;
                it.slot = -1;
                it.parts = 1;
                items[x * (total / nq) + min(x, total % nq) + p / nq] = it;
            }
        }
    }
}

}  // namespace

namespace flexsp {

// Resolves this GPU's copy of the scratch array.  Called by flexsp_ctx_create with `device`
// current, once per device (later calls find the pointer).
hipError_t static_scratch_init(int device)
{
    if (device < 0 || device >= kMaxDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (g_scratch_ptr[device]) return hipSuccess;
    void *p = nullptr;
    hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (!p) return hipErrorInvalidSymbol;
    g_scratch_ptr[device] = p;
    return hipSuccess;
}

}  // namespace flexsp

extern "C" int flexsp_attn_varlen_fwd_static(flexsp_ctx *ctx, flexsp_tensor q, flexsp_tensor k, flexsp_tensor v,
                                             const int32_t *cu_seqlens_dev, int32_t B, int64_t T,
                                             int32_t head_begin, int32_t head_count, int32_t kv_head_begin,
                                             int32_t kv_head_count, int32_t D, int causal, float scale,
                                             flexsp_tensor o, float *lse, flexsp_stream stream)
{
    if (!ctx || !cu_seqlens_dev || !lse || B < 0 || T < 0) return FLEXSP_INVALID_ARGUMENT;
    if (head_begin < 0 || kv_head_begin < 0 || head_count <= 0 || kv_head_count <= 0 ||
        head_count % kv_head_count != 0)
        return FLEXSP_INVALID_ARGUMENT;
    if (!view_ok(q) || !view_ok(k) || !view_ok(v) || !view_ok(o) || !std::isfinite(scale))
        return FLEXSP_INVALID_ARGUMENT;
    if (D != 64 && D != 128) return FLEXSP_UNSUPPORTED;
    // the scratch array bounds the batch: every sequence adds at most one partial tile
    if (T > (int64_t)kStaticMaxLevels * kFwdBq ||
        ((T + kFwdBq - 1) / kFwdBq + B) * (int64_t)head_count > kStaticMaxItems)
        return FLEXSP_UNSUPPORTED;
    const int device = ctx_device(ctx);
    if (device < 0 || device >= kMaxDevices || !g_scratch_ptr[device]) return FLEXSP_NO_DEVICE;
    if (B == 0 || T == 0) return FLEXSP_OK;
    unsigned char *scr = (unsigned char *)g_scratch_ptr[device];
    hipStream_t s = (hipStream_t)stream;

    hipLaunchKernelGGL(build_static_queue_kernel, dim3(1), dim3(kBuildThreads), 0, s, cu_seqlens_dev, (int)B, (int)T,
                       (int)head_count, causal ? 1 : 0, kFwdBq, scr);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return hip_status(e);

    if (scale <= 0.f) scale = 1.0f / std::sqrt((float)D);
    AttnArgs a;
    std::memset(&a, 0, sizeof(a));
    a.q = (const uint16_t *)q.ptr + (int64_t)head_begin * q.stride_head;
    a.k = (const uint16_t *)k.ptr + (int64_t)kv_head_begin * k.stride_head;
    a.v = (const uint16_t *)v.ptr + (int64_t)kv_head_begin * v.stride_head;
    a.out_o = (uint16_t *)o.ptr + (int64_t)head_begin * o.stride_head;
    a.q_st = (int32_t)q.stride_token; a.q_sh = (int32_t)q.stride_head;
    a.k_st = (int32_t)k.stride_token; a.k_sh = (int32_t)k.stride_head;
    a.v_st = (int32_t)v.stride_token; a.v_sh = (int32_t)v.stride_head;
    a.o_st = (int32_t)o.stride_token; a.o_sh = (int32_t)o.stride_head;
    a.lse_out = lse;
    a.T = (int32_t)T; a.Hq = head_count; a.G = head_count / kv_head_count; a.causal = causal ? 1 : 0;
    a.scale = scale; a.scale_l2 = scale * 1.4426950408889634f;
    a.pq.items = (const flexsp_item *)(scr + kItemsOff);
    a.pq.offsets = (const int32_t *)(scr + kOffsetsOff);
    a.pq.counters = (int32_t *)(scr + kCountersOff);
    a.pq.nq = kMaxQueues;
    // the item count is known to the device only: a full persistent grid; workgroups without work leave
    e = launch_attn_fwd(a, D, flexsp_ctx_num_cu(ctx) * 2, s);
    return e == hipSuccess ? FLEXSP_OK : hip_status(e);
}
