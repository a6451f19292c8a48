// Host side of libflexsp: contexts, tile plans, argument validation and the extern "C"
// entry points declared in include/flexsp.h.  No kernel lives here.
#include <algorithm>
#include <cmath>
#include <cstring>
#include <new>
#include <vector>

#include "flexsp_internal.h"

using namespace flexsp;

struct EventPair {
    hipEvent_t start, stop;
    int kernel;
};

// Device memory of a plan plus the pinned host buffer its queues are uploaded from.  Slabs are
// recycled through the context: creating a plan per micro-batch then costs neither an allocation
// nor a device-wide synchronisation (hipFree), and the upload is an asynchronous copy.
struct PlanSlab {
    void *dev = nullptr;
    size_t dev_bytes = 0;
    void *host = nullptr;  // pinned
    size_t host_bytes = 0;
    hipEvent_t ready = nullptr;  // recorded on the upload stream after the copy
    hipEvent_t done = nullptr;   // recorded on the last stream that ran kernels on this slab
    bool done_valid = false;
};
constexpr size_t kSlabPoolMax = 16;  // free slabs kept by a context
constexpr size_t kSlabEager = 4;     // slabs a context makes rather than wait for a busy one ...
constexpr size_t kSlabEagerBytes = (size_t)1 << 30;  // ... while they hold less device memory than this

struct flexsp_ctx {
    int device;  // -1: host-only
    int num_cu;
    int num_xcd;
    hipStream_t upload = nullptr;  // non-blocking stream (default priority) for plan uploads
    std::vector<PlanSlab> slabs;   // free slabs
    size_t slabs_owned = 0;        // slabs alive: free ones and those held by plans
    size_t slab_bytes = 0;         // device memory of the slabs alive
    // profiling: a pool of event pairs created by flexsp_profile_start
    bool profiling;
    std::vector<EventPair> events;
    size_t events_used;
    int64_t dropped;
};

struct HostPass {
    std::vector<flexsp_item> items;     // queue order
    int64_t offsets[kMaxQueues + 1];    // queue boundaries
    int tile_rows;
    int32_t records = 0;                // partial-result records of split tiles
};

struct flexsp_plan {
    flexsp_ctx *ctx;
    int32_t B, Hq, Hkv, D, causal;
    int64_t T;
    std::vector<int32_t> cu;
    // key-shard plans (forward only): the shard's own boundaries and the position offsets
    bool kvshard = false;
    std::vector<int32_t> cu_k, shift;
    int64_t Tk = 0;
    HostPass pass[3];
    // device side (null for host-only plans): one allocation, carved up
    void *dev_base;
    size_t dev_bytes;
    PlanSlab slab;
    bool uploaded;            // the upload is known to have completed
    bool used, multi_stream;  // kernels were launched on this plan; on more than one stream
    hipStream_t last_stream;
    PassQueues dq[3];
    float *delta;
    size_t delta_bytes;
};

namespace {

thread_local int g_last_hip_error = 0;

int hip_fail(hipError_t e)
{
    g_last_hip_error = (int)e;
    return e == hipErrorOutOfMemory ? FLEXSP_OUT_OF_MEMORY : FLEXSP_HIP_ERROR;
}

inline int64_t cdiv(int64_t a, int64_t b) { return (a + b - 1) / b; }

// Workgroups an attention launch keeps resident: two per compute unit (a host-only context plans
// for the 256 compute units of the device it stands in for).
int workgroups_of(const flexsp_ctx *ctx) { return 2 * (ctx->num_cu > 0 ? ctx->num_cu : 256); }

void slab_free(PlanSlab &s)
{
    if (s.dev) (void)hipFree(s.dev);
    if (s.host) (void)hipHostFree(s.host);
    if (s.ready) (void)hipEventDestroy(s.ready);
    if (s.done) (void)hipEventDestroy(s.done);
    s = PlanSlab();
}

// A slab with at least the given sizes.  Among the adequate ones in the pool, one whose last
// kernels have already finished is preferred (the smallest such): its queues can be uploaded at
// once, while the kernels of the plan destroyed a moment ago still run.  Taking back the slab just
// released instead would put every step's upload behind the previous step's last kernel and in
// front of its own first one, an idle gap per step.  When every adequate slab is still in use
// and the context owns fewer than kSlabEager slabs (and less than kSlabEagerBytes in them), a new one
// is made (a quarter larger than asked, so that the next, slightly different batch fits too).
// Beyond that the HOST waits here for the busy slab released longest ago: a caller that builds a
// plan per micro-batch is thereby held kSlabEager steps ahead of the GPU at most, which keeps the
// GPU fed just as well as running ahead without bound does.  Both alternatives were measured and
// stall the GPU for 6-9 ms each time: making slabs as the host runs further ahead (allocating
// device and pinned memory in the middle of a run), and ordering the upload behind the busy
// slab's kernels with an event on the upload stream (the first such cross-stream waits after an
// idle period).  With the host-side wait, allocations end with the first kSlabEager plans of a run
// and no stream ever waits for an event that is not complete yet.
hipError_t slab_get(flexsp_ctx *ctx, size_t dev_bytes, size_t host_bytes, PlanSlab &out)
{
    int best = -1, best_busy = -1;
    for (size_t i = 0; i < ctx->slabs.size(); i++) {
        const PlanSlab &s = ctx->slabs[i];
        if (s.dev_bytes < dev_bytes || s.host_bytes < host_bytes) continue;
        const bool idle = !s.done_valid || hipEventQuery(s.done) == hipSuccess;
        // idle: the smallest adequate one; busy: the first in the list, which was released first
        if (idle) {
            if (best < 0 || s.dev_bytes < ctx->slabs[best].dev_bytes) best = (int)i;
        } else if (best_busy < 0) {
            best_busy = (int)i;
        }
    }
    if (best < 0 && best_busy >= 0 && (ctx->slabs_owned >= kSlabEager || ctx->slab_bytes + dev_bytes > kSlabEagerBytes))
        best = best_busy;
    if (best >= 0) {
        out = ctx->slabs[best];
        ctx->slabs.erase(ctx->slabs.begin() + best);
        if (best == best_busy) {
            hipError_t e = hipEventSynchronize(out.done);
            if (e != hipSuccess) return e;
        }
        out.done_valid = false;  // its kernels are over: nothing to order the upload behind
        // the previous upload from this pinned buffer must be over before the host refills it
        return hipEventSynchronize(out.ready);
    }
    PlanSlab s;
    s.dev_bytes = dev_bytes + dev_bytes / 4 + 256;
    s.host_bytes = host_bytes + host_bytes / 4 + 256;
    hipError_t e = hipMalloc(&s.dev, s.dev_bytes);
    if (e == hipSuccess) e = hipHostMalloc(&s.host, s.host_bytes, hipHostMallocDefault);
    if (e == hipSuccess) e = hipEventCreateWithFlags(&s.ready, hipEventDisableTiming);
    if (e == hipSuccess) e = hipEventCreateWithFlags(&s.done, hipEventDisableTiming);
    if (e != hipSuccess) {
        slab_free(s);
        return e;
    }
    ctx->slabs_owned++;
    ctx->slab_bytes += s.dev_bytes;
    out = s;
    return hipSuccess;
}

// Called by the hot entry points before they launch on `stream`: the kernels must see the
// uploaded queues.  Once the upload is known to be complete this is one flag test.
hipError_t plan_before_launch(flexsp_plan *plan, hipStream_t stream)
{
    if (!plan->uploaded) {
        hipError_t q = hipEventQuery(plan->slab.ready);
        if (q == hipSuccess) {
            plan->uploaded = true;
        } else if (q == hipErrorNotReady) {
            hipError_t e = hipStreamWaitEvent(stream, plan->slab.ready, 0);
            if (e != hipSuccess) return e;
        } else {
            return q;
        }
    }
    if (plan->used && plan->last_stream != stream) plan->multi_stream = true;
    plan->used = true;
    plan->last_stream = stream;
    return hipSuccess;
}

// Brackets one kernel launch with a pair of events while profiling is on.
struct Timed {
    flexsp_ctx *ctx;
    hipStream_t stream;
    EventPair *ev;
    Timed(flexsp_ctx *c, int kernel, hipStream_t s) : ctx(c), stream(s), ev(nullptr)
    {
        if (!c->profiling) return;
        if (c->events_used >= c->events.size()) {
            c->dropped++;
            return;
        }
        ev = &c->events[c->events_used++];
        ev->kernel = kernel;
        (void)hipEventRecord(ev->start, stream);
    }
    ~Timed()
    {
        if (ev) (void)hipEventRecord(ev->stop, stream);
    }
};

struct Work {
    flexsp_item it;
    int64_t cost;   // inner-loop steps of this item
    int32_t group;  // (sequence, head) group id
};

void distribute(std::vector<Work> &work, const std::vector<int64_t> &group_cost, int nq, int n_wg, int tile_rows,
                HostPass &out, int spare = 0);

// Builds one pass: lists the items, spreads whole (sequence, head) groups over the queues
// (largest group first onto the least loaded queue, so tiles that read the same K/V run on
// one XCD and share its L2), then orders each queue by decreasing cost (short sequences: tile beside tile, see distribute) so that the long
// tail of a batch starts first and short items fill the gaps at the end.
void build_pass(const std::vector<int32_t> &cu, int B, int heads, int group_mult, int tile_rows,
                int step_rows, bool causal, bool key_major, int nq, int n_wg, HostPass &out)
{
    std::vector<Work> work;
    std::vector<int64_t> group_cost;
    {
        size_t total = 0;
        for (int b = 0; b < B; b++) total += (size_t)cdiv(std::max(cu[b + 1] - cu[b], 0), tile_rows);
        work.reserve(total * heads);
        group_cost.reserve((size_t)B * heads);
    }
    for (int b = 0; b < B; b++) {
        int32_t s = cu[b + 1] - cu[b];
        if (s <= 0) continue;
        int32_t nt = (int32_t)cdiv(s, tile_rows);
        for (int h = 0; h < heads; h++) {
            int32_t gid = (int32_t)group_cost.size();
            int64_t gc = 0;
            for (int32_t t = 0; t < nt; t++) {
                int64_t cost;
                if (!key_major) {
                    // query tile t: keys 0 .. min(s, (t+1)*tile_rows) - 1 when causal
                    int64_t keys = causal ? std::min<int64_t>(s, (int64_t)(t + 1) * tile_rows) : s;
                    cost = cdiv(keys, step_rows);
                } else {
                    // key tile t: queries from the tile's first key to the end when causal
                    int64_t first = causal ? (int64_t)t * tile_rows : 0;
                    cost = cdiv(s - first, step_rows) * group_mult;
                }
                Work w;
                w.it.seq_start = cu[b];
                w.it.seq_len = s;
                w.it.tile = t;
                w.it.head = h;
                w.cost = cost;
                w.group = gid;
                work.push_back(w);
                gc += cost;
            }
            group_cost.push_back(gc);
        }
    }
    distribute(work, group_cost, nq, n_wg, tile_rows, out);
}

// Cuts tiles that would outlast an even share of the pass into parts (see flexsp_item): with W =
// total steps / workgroups, a tile of c steps becomes ceil(c / L) parts of equal length (at most
// kMaxParts, none shorter than kMinPartSteps), where the part length aimed at is L = 3W/4 while that
// is at most kLongPartSteps, then kLongPartSteps, and 0.35 W once that is longer still: a part costs
// its hand-over (a few steps' time) whatever its length, so short parts are kept few and long ones
// are made finer, which evens out the end of the pass.  Longest-first scheduling alone
// finishes no earlier than the longest item, which for a batch of few heads and one dominant
// sequence is several times the even share: the compute units that run out of work wait for it.
// `spare`: tiles of up to this many even shares are left whole (0: every tile longer than a part is cut).
void split_long_items(std::vector<Work> &work, int n_wg, int spare, HostPass &out)
{
    out.records = 0;
    int64_t total = 0;
    for (Work &w : work) {
        w.it.step_begin = 0;
        w.it.step_end = (int32_t)w.cost;
        w.it.slot = -1;
        w.it.parts = 1;
        total += w.cost;
    }
    const int64_t share = total / std::max(n_wg, 1);
    const int64_t target = std::max<int64_t>(
        std::min(share * 3 / 4, std::max<int64_t>(share * 35 / 100, kLongPartSteps)), kMinPartSteps);
    const size_t n0 = work.size();
    for (size_t i = 0; i < n0; i++) {
        const int64_t c = work[i].cost;
        if (c < 2 * kMinPartSteps || c <= target || c <= spare * share) continue;
        int k = (int)std::min<int64_t>(std::min<int64_t>(cdiv(c, target), kMaxParts), c / kMinPartSteps);
        if (k < 2 || out.records + k > kMaxSplitRecords) continue;
        const int32_t slot = out.records;
        out.records += k;
        for (int p = 0; p < k; p++) {
            Work w = work[i];
            w.it.step_begin = (int32_t)((int64_t)p * c / k);
            w.it.step_end = (int32_t)((int64_t)(p + 1) * c / k);
            w.it.slot = slot;
            w.it.parts = (p << 16) | k;
            w.cost = w.it.step_end - w.it.step_begin;
            if (p == 0)
                work[i] = w;
            else
                work.push_back(w);
        }
    }
}

// Spreads listed work over the queues and orders every queue longest first (see build_pass).
void distribute(std::vector<Work> &work, const std::vector<int64_t> &group_cost, int nq, int n_wg, int tile_rows,
                HostPass &out, int spare)
{
    split_long_items(work, n_wg, spare, out);
    // groups -> queues
    std::vector<int32_t> order(group_cost.size());
    for (size_t i = 0; i < order.size(); i++) order[i] = (int32_t)i;
    std::stable_sort(order.begin(), order.end(),
                     [&](int32_t a, int32_t b) { return group_cost[a] > group_cost[b]; });
    std::vector<int64_t> load(nq, 0);
    std::vector<int32_t> queue_of(group_cost.size(), 0);
    for (int32_t g : order) {
        int best = 0;
        for (int x = 1; x < nq; x++)
            if (load[x] < load[best]) best = x;
        queue_of[g] = best;
        load[best] += group_cost[g];
    }
    // item -> queue: its group's queue.  Each queue's members are kept in order of decreasing
    // cost; the order comes from one stable counting sort of all items (costs are small integers),
    // not from comparison sorts: a plan is built per micro-batch, on the host's time.
    const size_t n = work.size();
    std::vector<int32_t> item_queue(n);
    for (size_t i = 0; i < n; i++) item_queue[i] = queue_of[work[i].group];
    std::vector<int32_t> by_cost(n);  // item indices, most expensive first, ties in list order
    {
        int64_t maxc = 0;
        for (const Work &w : work) maxc = std::max(maxc, w.cost);
        if (maxc <= (int64_t)(4 * n + 1024)) {
            std::vector<int32_t> start((size_t)maxc + 2, 0);
            for (const Work &w : work) start[(size_t)(maxc - w.cost) + 1]++;
            for (size_t c = 1; c < start.size(); c++) start[c] += start[c - 1];
            for (size_t i = 0; i < n; i++) by_cost[(size_t)start[(size_t)(maxc - work[i].cost)]++] = (int32_t)i;
        } else {  // a few enormous items: the table would be larger than the list
            for (size_t i = 0; i < n; i++) by_cost[i] = (int32_t)i;
            std::stable_sort(by_cost.begin(), by_cost.end(),
                             [&](int32_t a, int32_t b) { return work[a].cost > work[b].cost; });
        }
    }
    std::vector<std::vector<int32_t>> members(nq);
    for (int x = 0; x < nq; x++) members[x].reserve(n / nq + 16);
    for (int32_t idx : by_cost) members[item_queue[idx]].push_back(idx);
    // Level the queues by moving the cheapest items of the fullest queue to the emptiest one (a
    // group that outweighs a whole queue's share, e.g. one dominant sequence with few heads, is
    // split this way; only the moved items lose L2 affinity).
    // Moved items wait in a side list per receiving queue and are merged in once (one insertion
    // into a sorted list per move costs a memmove each, thousands of times when six heavy groups
    // meet eight queues).
    auto dearer = [&](int32_t a, int32_t b) { return work[a].cost > work[b].cost; };
    std::vector<std::vector<int32_t>> incoming(nq);
    auto merge_in = [&](int x) {
        if (incoming[x].empty()) return;
        std::stable_sort(incoming[x].begin(), incoming[x].end(), dearer);
        std::vector<int32_t> merged(members[x].size() + incoming[x].size());
        std::merge(members[x].begin(), members[x].end(), incoming[x].begin(), incoming[x].end(), merged.begin(),
                   dearer);
        members[x].swap(merged);
        incoming[x].clear();
    };
    for (size_t guard = 0; guard < n; guard++) {
        int hi = 0, lo_ = 0;
        for (int x = 1; x < nq; x++) {
            if (load[x] > load[hi]) hi = x;
            if (load[x] < load[lo_]) lo_ = x;
        }
        merge_in(hi);  // (rare: a queue that received items has become the fullest)
        if (members[hi].empty()) break;
        const int32_t cand = members[hi].back();
        const int64_t c = work[cand].cost;
        if (load[hi] - c < load[lo_] + c) break;  // moving would not narrow the gap
        members[hi].pop_back();
        load[hi] -= c;
        load[lo_] += c;
        incoming[lo_].push_back(cand);
    }
    for (int x = 0; x < nq; x++) merge_in(x);
    // Order inside a queue.  Items of long sequences stay longest first.  The tiles of a SHORT sequence
    // (none of more than kGroupMajorSteps steps) are put side by side, where the longest of them would
    // stand: the workgroups of the XCD then take them at about the same time and share the sequence's
    // rows in L2, instead of each meeting them cold (batches of 256- to 1 024-token sequences: 2-4 %
    // faster; no effect where long sequences carry the work).  The queue still ends with its cheapest items.
    {
        std::vector<int64_t> gmax(group_cost.size(), 0);
        for (const Work &w : work) gmax[w.group] = std::max(gmax[w.group], w.cost);
        auto rank = [&](int32_t i) { return gmax[work[i].group] > kGroupMajorSteps ? work[i].cost : gmax[work[i].group]; };
        for (int x = 0; x < nq; x++)
            std::stable_sort(members[x].begin(), members[x].end(), [&](int32_t a, int32_t b) {
                const int64_t ra = rank(a), rb = rank(b);
                if (ra != rb) return ra > rb;
                const int32_t ga = work[a].group, gb = work[b].group;
                const bool sa = gmax[ga] <= kGroupMajorSteps, sb = gmax[gb] <= kGroupMajorSteps;
                if (sa != sb) return sb;              // at equal rank: items of long sequences first
                if (!sa) return false;                // two of those: as they were (stable)
                if (ga != gb) return ga < gb;         // short sequences: one after the other,
                return work[a].cost > work[b].cost;   // each with its dearest tile first
            });
    }
    out.items.resize(n);
    size_t at = 0;
    for (int x = 0; x <= kMaxQueues; x++) out.offsets[x] = (int64_t)n;
    for (int x = 0; x < nq; x++) {
        out.offsets[x] = (int64_t)at;
        for (int32_t idx : members[x]) out.items[at++] = work[idx].it;
    }
    out.offsets[nq] = (int64_t)n;
    out.tile_rows = tile_rows;
}

int check_attn_common(flexsp_ctx *ctx, flexsp_plan *plan, const int32_t *cu_dev, int32_t head_begin,
                      int32_t head_count, int32_t kv_head_begin, int32_t kv_head_count, int causal)
{
    (void)cu_dev;  // the plan carries the lengths; the device copy is not read by the plan-based calls
    if (!ctx || !plan) return FLEXSP_INVALID_ARGUMENT;
    if (plan->ctx != ctx || plan->kvshard) return FLEXSP_PLAN_MISMATCH;
    if (head_begin < 0 || kv_head_begin < 0 || head_count <= 0 || kv_head_count <= 0)
        return FLEXSP_INVALID_ARGUMENT;
    if (head_count % kv_head_count != 0) return FLEXSP_INVALID_ARGUMENT;
    if (head_count != plan->Hq || kv_head_count != plan->Hkv || (causal != 0) != (plan->causal != 0))
        return FLEXSP_PLAN_MISMATCH;
    if (ctx->device < 0 || !plan->dev_base) return FLEXSP_NO_DEVICE;
    return FLEXSP_OK;
}

// Puts a freshly built plan's queues on the device (nothing to do for a host-only context): one
// slab, carved into [items x3][offsets x3][counters x3][delta, lse2].  Items of a key-shard plan are
// written in their wider device form.  On failure the plan is deleted and a status returned.
int plan_upload(flexsp_ctx *ctx, flexsp_plan *p)
{
    for (int i = 0; i < 3; i++) std::memset(&p->dq[i], 0, sizeof(PassQueues));
    if (ctx->device < 0) return FLEXSP_OK;
    const size_t item_bytes = p->kvshard ? sizeof(flexsp_shard_item) : sizeof(flexsp_item);
    {

        // one allocation: [items x3][offsets x3][counters x3][delta]
        int nq = ctx->num_xcd;
        size_t off = 0, item_off[3], offs_off[3], ctr_off[3];
        auto align = [](size_t x) { return (x + 255) & ~(size_t)255; };
        for (int i = 0; i < 3; i++) {
            item_off[i] = off;
            off = align(off + p->pass[i].items.size() * item_bytes);
        }
        for (int i = 0; i < 3; i++) {
            offs_off[i] = off;
            off = align(off + (nq + 1) * sizeof(int32_t));
        }
        for (int i = 0; i < 3; i++) {
            ctr_off[i] = off;
            off = align(off + (nq + 1) * kCounterStride * sizeof(int32_t));
        }
        size_t flag_off[3], part_off[3];
        for (int i = 0; i < 3; i++) {
            flag_off[i] = off;
            off = align(off + (size_t)p->pass[i].records * sizeof(int32_t));
        }
        size_t head_bytes = off;
        size_t delta_off = off;
        off = align(off + p->delta_bytes + 512);  // the dK/dV kernel reads up to 63 floats past a row's end
        for (int i = 0; i < 3; i++) {
            part_off[i] = off;
            off = align(off + (size_t)p->pass[i].records * kPartialBytes);
        }
        hipError_t e = hipSetDevice(ctx->device);
        if (e == hipSuccess) e = slab_get(ctx, off ? off : 256, head_bytes ? head_bytes : 256, p->slab);
        if (e != hipSuccess) {
            delete p;
            return hip_fail(e);
        }
        p->dev_base = p->slab.dev;
        p->dev_bytes = off;
        char *stage = (char *)p->slab.host;
        std::memset(stage, 0, head_bytes);  // also the ticket counters: every plan starts with them clear
        for (int i = 0; i < 3; i++) {
            if (p->kvshard) {
                // the host list names a sequence by its index (seq_start); the device item carries its ranges
                flexsp_shard_item *d = (flexsp_shard_item *)(stage + item_off[i]);
                for (size_t n = 0; n < p->pass[i].items.size(); n++) {
                    const flexsp_item &it = p->pass[i].items[n];
                    const int b = it.seq_start;
                    // a part of a cut tile: the keys of its steps only, positions counted from its first key
                    const int32_t np = it.parts & 0xffff, part = it.parts >> 16;  // (whole tiles only in the dK/dV pass)
                    const int32_t skip = np > 1 ? it.step_begin * kFwdBk : 0;
                    int32_t k_len = p->cu_k[b + 1] - p->cu_k[b];
                    if (np > 1 && part + 1 < np) k_len = std::min(k_len, it.step_end * kFwdBk);
                    d[n] = flexsp_shard_item{p->cu[b], p->cu[b + 1] - p->cu[b], p->cu_k[b] + skip, k_len - skip,
                                             p->shift[b] - skip, it.tile, it.head | (part << 16) | (np << 24), it.slot};
                }
            } else if (!p->pass[i].items.empty()) {
                std::memcpy(stage + item_off[i], p->pass[i].items.data(),
                            p->pass[i].items.size() * sizeof(flexsp_item));
            }
            int32_t *o = (int32_t *)(stage + offs_off[i]);
            for (int x = 0; x <= nq; x++) o[x] = (int32_t)p->pass[i].offsets[x];
            p->dq[i].items = (const flexsp_item *)((char *)p->dev_base + item_off[i]);
            p->dq[i].offsets = (const int32_t *)((char *)p->dev_base + offs_off[i]);
            p->dq[i].counters = (int32_t *)((char *)p->dev_base + ctr_off[i]);
            p->dq[i].nq = nq;
            p->dq[i].split_flags = (int32_t *)((char *)p->dev_base + flag_off[i]);
            p->dq[i].split_scratch = (char *)p->dev_base + part_off[i];
        }
        // asynchronous upload on the context's own stream, after the kernels of the slab's previous
        // plan; the hot calls make their stream wait for `ready` (or find it complete already)
        if (p->slab.done_valid) e = hipStreamWaitEvent(ctx->upload, p->slab.done, 0);
        if (e == hipSuccess && head_bytes)
            e = hipMemcpyAsync(p->dev_base, stage, head_bytes, hipMemcpyHostToDevice, ctx->upload);
        if (e == hipSuccess) e = hipEventRecord(p->slab.ready, ctx->upload);
        if (e != hipSuccess) {
            (void)hipStreamSynchronize(ctx->upload);
            ctx->slab_bytes -= p->slab.dev_bytes;
            slab_free(p->slab);
            ctx->slabs_owned--;
            delete p;
            return hip_fail(e);
        }
        p->slab.done_valid = false;
        p->delta = (float *)((char *)p->dev_base + delta_off);
    }
    return FLEXSP_OK;
}

int grid_for(const flexsp_ctx *ctx, const HostPass &p, int per_cu)
{
    int64_t n = (int64_t)p.items.size();
    int64_t g = (int64_t)ctx->num_cu * per_cu;
    if (n < g) g = ((n + ctx->num_xcd - 1) / ctx->num_xcd) * ctx->num_xcd;
    return (int)std::max<int64_t>(g, 1);
}

}  // namespace

namespace flexsp {
int ctx_device(const flexsp_ctx *ctx) { return ctx ? ctx->device : -1; }
int hip_status(hipError_t e) { return hip_fail(e); }
}  // namespace flexsp

extern "C" {

const char *flexsp_strerror(int status)
{
    switch (status) {
    case FLEXSP_OK: return "ok";
    case FLEXSP_INVALID_ARGUMENT: return "invalid argument";
    case FLEXSP_UNSUPPORTED: return "unsupported configuration";
    case FLEXSP_PLAN_MISMATCH: return "arguments do not match the plan";
    case FLEXSP_HIP_ERROR: return "HIP runtime error";
    case FLEXSP_OUT_OF_MEMORY: return "out of memory";
    case FLEXSP_NO_DEVICE: return "no usable gfx950 device";
    default: return "unknown status";
    }
}

int flexsp_last_hip_error(void) { return g_last_hip_error; }

const char *flexsp_version(void) { return "0.1"; }

int flexsp_ctx_create(flexsp_ctx **out, int device)
{
    if (!out || device < -1) return FLEXSP_INVALID_ARGUMENT;
    *out = nullptr;
    flexsp_ctx *c = new (std::nothrow) flexsp_ctx;
    if (!c) return FLEXSP_OUT_OF_MEMORY;
    c->device = device;
    c->num_cu = 0;
    c->num_xcd = kMaxQueues;
    c->profiling = false;
    c->events_used = 0;
    c->dropped = 0;
    if (device >= 0) {
        int n = 0;
        hipError_t e = hipGetDeviceCount(&n);
        if (e != hipSuccess || device >= n) {
            delete c;
            g_last_hip_error = (int)e;
            return FLEXSP_NO_DEVICE;
        }
        hipDeviceProp_t pr;
        e = hipGetDeviceProperties(&pr, device);
        if (e != hipSuccess) {
            delete c;
            return hip_fail(e);
        }
        if (std::strncmp(pr.gcnArchName, "gfx950", 6) != 0) {
            delete c;
            return FLEXSP_NO_DEVICE;
        }
        c->num_cu = pr.multiProcessorCount;
        e = hipSetDevice(device);
        if (e == hipSuccess) e = hipStreamCreateWithFlags(&c->upload, hipStreamNonBlocking);
        if (e == hipSuccess) e = static_scratch_init(device);  // this device is current here
        if (e != hipSuccess) {
            if (c->upload) (void)hipStreamDestroy(c->upload);
            delete c;
            return hip_fail(e);
        }
    }
    *out = c;
    return FLEXSP_OK;
}

void flexsp_ctx_destroy(flexsp_ctx *ctx)
{
    if (!ctx) return;
    if (ctx->device >= 0) (void)hipSetDevice(ctx->device);
    for (EventPair &e : ctx->events) {
        (void)hipEventDestroy(e.start);
        (void)hipEventDestroy(e.stop);
    }
    if (ctx->device >= 0) {
        if (!ctx->slabs.empty()) (void)hipDeviceSynchronize();  // kernels of destroyed plans may still run
        for (PlanSlab &s : ctx->slabs) slab_free(s);
        if (ctx->upload) (void)hipStreamDestroy(ctx->upload);
    }
    delete ctx;
}

int flexsp_profile_start(flexsp_ctx *ctx, int32_t max_launches)
{
    if (!ctx || max_launches <= 0) return FLEXSP_INVALID_ARGUMENT;
    if (ctx->device < 0) return FLEXSP_NO_DEVICE;
    try {
        ctx->events.reserve((size_t)max_launches);
    } catch (const std::bad_alloc &) {
        return FLEXSP_OUT_OF_MEMORY;
    }
    {
        hipError_t r = hipSetDevice(ctx->device);  // events belong to the device that is current when they are made
        if (r != hipSuccess) return hip_fail(r);
    }
    while (ctx->events.size() < (size_t)max_launches) {
        EventPair e;
        e.kernel = 0;
        hipError_t r = hipEventCreate(&e.start);
        if (r != hipSuccess) return hip_fail(r);
        r = hipEventCreate(&e.stop);
        if (r != hipSuccess) {
            (void)hipEventDestroy(e.start);
            return hip_fail(r);
        }
        ctx->events.push_back(e);
    }
    ctx->events_used = 0;
    ctx->dropped = 0;
    ctx->profiling = true;
    return FLEXSP_OK;
}

int flexsp_profile_stop(flexsp_ctx *ctx, flexsp_profile *out)
{
    if (!ctx || !out) return FLEXSP_INVALID_ARGUMENT;
    if (ctx->device < 0) return FLEXSP_NO_DEVICE;
    std::memset(out, 0, sizeof(*out));
    ctx->profiling = false;
    for (size_t i = 0; i < ctx->events_used; i++) {
        EventPair &e = ctx->events[i];
        hipError_t r = hipEventSynchronize(e.stop);
        if (r != hipSuccess) return hip_fail(r);
        float ms = 0.f;
        r = hipEventElapsedTime(&ms, e.start, e.stop);
        if (r != hipSuccess) return hip_fail(r);
        out->ms[e.kernel] += ms;
        out->launches[e.kernel]++;
    }
    out->dropped = ctx->dropped;
    ctx->events_used = 0;
    return FLEXSP_OK;
}

int flexsp_ctx_num_cu(const flexsp_ctx *ctx) { return ctx ? ctx->num_cu : 0; }
int flexsp_ctx_num_xcd(const flexsp_ctx *ctx) { return ctx ? ctx->num_xcd : 0; }

int flexsp_plan_create(flexsp_ctx *ctx, const int32_t *cu, int32_t B, int32_t Hq, int32_t Hkv,
                       int32_t D, int causal, flexsp_plan **out)
{
    if (!out) return FLEXSP_INVALID_ARGUMENT;
    *out = nullptr;
    if (!ctx || !cu || B < 0 || Hq <= 0 || Hkv <= 0 || D <= 0) return FLEXSP_INVALID_ARGUMENT;
    if (Hq % Hkv != 0) return FLEXSP_INVALID_ARGUMENT;
    if (cu[0] != 0) return FLEXSP_INVALID_ARGUMENT;
    for (int b = 0; b < B; b++)
        if (cu[b + 1] < cu[b]) return FLEXSP_INVALID_ARGUMENT;
    if (D != 64 && D != 128) return FLEXSP_UNSUPPORTED;
    flexsp_plan *p = new (std::nothrow) flexsp_plan;
    if (!p) return FLEXSP_OUT_OF_MEMORY;
    p->ctx = ctx;
    p->B = B; p->Hq = Hq; p->Hkv = Hkv; p->D = D; p->causal = causal ? 1 : 0;
    p->T = cu[B];
    p->dev_base = nullptr; p->dev_bytes = 0; p->delta = nullptr;
    p->uploaded = false; p->used = false; p->multi_stream = false; p->last_stream = nullptr;
    p->delta_bytes = 2 * (size_t)p->T * Hq * sizeof(float);  // delta and log2-domain LSE, [Hq, T] each
    try {
        p->cu.assign(cu, cu + B + 1);
        const int nq = ctx->num_xcd, n_wg = workgroups_of(ctx);
        build_pass(p->cu, B, Hq, 1, kFwdBq, kFwdBk, causal != 0, false, nq, n_wg, p->pass[FLEXSP_PASS_FWD]);
        build_pass(p->cu, B, Hkv, Hq / Hkv, kDkvBk, kDkvBq, causal != 0, true, nq, n_wg, p->pass[FLEXSP_PASS_BWD_DKV]);
        build_pass(p->cu, B, Hq, 1, kDqBq, kDqBk, causal != 0, false, nq, n_wg, p->pass[FLEXSP_PASS_BWD_DQ]);
    } catch (const std::bad_alloc &) {
        delete p;
        return FLEXSP_OUT_OF_MEMORY;
    }
    {
        int rc = plan_upload(ctx, p);
        if (rc) return rc;
    }
    *out = p;
    return FLEXSP_OK;
}

int flexsp_plan_create_kvshard(flexsp_ctx *ctx, const int32_t *cu_q, const int32_t *cu_k, const int32_t *shift,
                               int32_t B, int32_t Hq, int32_t Hkv, int32_t D, int causal, flexsp_plan **out)
{
    if (!out) return FLEXSP_INVALID_ARGUMENT;
    *out = nullptr;
    if (!ctx || !cu_q || !cu_k || (!shift && B > 0) || B < 0 || Hq <= 0 || Hkv <= 0 || D <= 0)
        return FLEXSP_INVALID_ARGUMENT;
    if (Hq % Hkv != 0 || cu_q[0] != 0 || cu_k[0] != 0) return FLEXSP_INVALID_ARGUMENT;
    for (int b = 0; b < B; b++) {
        if (cu_q[b + 1] < cu_q[b] || cu_k[b + 1] < cu_k[b]) return FLEXSP_INVALID_ARGUMENT;
        // positions are token counts: |shift| beyond 2^30 would overflow the kernels' 32-bit arithmetic
        if (shift[b] > (1 << 30) || shift[b] < -(1 << 30)) return FLEXSP_INVALID_ARGUMENT;
    }
    if (D != 64 && D != 128) return FLEXSP_UNSUPPORTED;
    if (Hq > 0xffff) return FLEXSP_UNSUPPORTED;  // a device item keeps the head in 16 bits
    flexsp_plan *p = new (std::nothrow) flexsp_plan;
    if (!p) return FLEXSP_OUT_OF_MEMORY;
    p->ctx = ctx;
    p->B = B; p->Hq = Hq; p->Hkv = Hkv; p->D = D; p->causal = causal ? 1 : 0;
    p->T = cu_q[B];
    p->Tk = cu_k[B];
    p->kvshard = true;
    p->dev_base = nullptr; p->dev_bytes = 0; p->delta = nullptr;
    p->uploaded = false; p->used = false; p->multi_stream = false; p->last_stream = nullptr;
    p->delta_bytes = 2 * (size_t)p->T * Hq * sizeof(float);  // delta and log2-domain LSE of the query rows
    static_assert(kFwdBq == kDqBq && kFwdBk == kDqBk, "the forward's and the dQ kernel's shard items are listed alike");
    try {
        p->cu.assign(cu_q, cu_q + B + 1);
        p->cu_k.assign(cu_k, cu_k + B + 1);
        p->shift.assign(shift, shift + B);
        // forward and dQ kernel: items (sequence index, query tile, head); cost = key tiles the tile's rows can see
        for (int pass : {FLEXSP_PASS_FWD, FLEXSP_PASS_BWD_DQ}) {
            std::vector<Work> work;
            std::vector<int64_t> group_cost;
            for (int b = 0; b < B; b++) {
                const int32_t sq = cu_q[b + 1] - cu_q[b], sk = cu_k[b + 1] - cu_k[b];
                if (sq <= 0) continue;
                const int32_t nt = (int32_t)cdiv(sq, kFwdBq);
                for (int h = 0; h < Hq; h++) {
                    const int32_t gid = (int32_t)group_cost.size();
                    int64_t gc = 0;
                    for (int32_t t = 0; t < nt; t++) {
                        int64_t keys = sk;
                        if (causal) keys = std::max<int64_t>(0, std::min<int64_t>(sk, (int64_t)(t + 1) * kFwdBq + shift[b]));
                        Work w;
                        w.it.seq_start = b;  // the sequence INDEX (see plan_upload); its ranges are in cu / cu_k / shift
                        w.it.seq_len = sq;
                        w.it.tile = t;
                        w.it.head = h;
                        w.cost = cdiv(keys, kFwdBk) + 1;  // an item without visible keys still writes its rows
                        w.group = gid;
                        work.push_back(w);
                        gc += w.cost;
                    }
                    group_cost.push_back(gc);
                }
            }
            // (a tile is cut only when it would outlast TWO even shares: with a share of a few dozen steps, as
            // on a micro-batch split over a ring, the hand-over of the parts costs more than the wait for a
            // tile that is a little longer than the rest)
            distribute(work, group_cost, ctx->num_xcd, workgroups_of(ctx), kFwdBq, p->pass[pass], 2);
        }
        // dK/dV kernel: items (sequence index, key tile of the shard, kv head); cost = steps of 64 query rows
        // from the first row that sees the tile, for every query head of the group.  Not cut into parts.
        {
            std::vector<Work> work;
            std::vector<int64_t> group_cost;
            const int G = Hq / Hkv;
            for (int b = 0; b < B; b++) {
                const int32_t sq = cu_q[b + 1] - cu_q[b], sk = cu_k[b + 1] - cu_k[b];
                if (sk <= 0) continue;
                const int32_t nt = (int32_t)cdiv(sk, kDkvBk);
                for (int g = 0; g < Hkv; g++) {
                    const int32_t gid = (int32_t)group_cost.size();
                    int64_t gc = 0;
                    for (int32_t t = 0; t < nt; t++) {
                        int64_t qfirst = 0;
                        if (causal) qfirst = std::max<int64_t>(0, (int64_t)t * kDkvBk - shift[b]) / kDkvBq * kDkvBq;
                        Work w;
                        w.it.seq_start = b;
                        w.it.seq_len = sk;
                        w.it.tile = t;
                        w.it.head = g;
                        w.cost = std::max<int64_t>(0, cdiv((int64_t)sq - qfirst, kDkvBq)) * G + 1;  // (the rows are written even if nobody sees them)
                        w.group = gid;
                        work.push_back(w);
                        gc += w.cost;
                    }
                    group_cost.push_back(gc);
                }
            }
            // (one "workgroup" whose share no tile exceeds: nothing is cut)
            distribute(work, group_cost, ctx->num_xcd, 1, kDkvBk, p->pass[FLEXSP_PASS_BWD_DKV], 1);
        }
    } catch (const std::bad_alloc &) {
        delete p;
        return FLEXSP_OUT_OF_MEMORY;
    }
    {
        int rc = plan_upload(ctx, p);
        if (rc) return rc;
    }
    *out = p;
    return FLEXSP_OK;
}

void flexsp_plan_destroy(flexsp_plan *plan)
{
    if (!plan) return;
    if (plan->dev_base) {
        flexsp_ctx *ctx = plan->ctx;
        (void)hipSetDevice(ctx->device);
        PlanSlab s = plan->slab;
        // whoever gets this slab next must come after the kernels still running on it
        s.done_valid = false;
        if (plan->used) {
            if (plan->multi_stream || hipEventRecord(s.done, plan->last_stream) != hipSuccess)
                (void)hipDeviceSynchronize();
            else
                s.done_valid = true;
        }
        if (ctx->slabs.size() < kSlabPoolMax) {
            try {
                ctx->slabs.push_back(s);
            } catch (const std::bad_alloc &) {
                if (s.done_valid) (void)hipEventSynchronize(s.done);
                (void)hipEventSynchronize(s.ready);
                ctx->slab_bytes -= s.dev_bytes;
                slab_free(s);
                ctx->slabs_owned--;
            }
        } else {
            if (s.done_valid) (void)hipEventSynchronize(s.done);
            (void)hipEventSynchronize(s.ready);
            ctx->slab_bytes -= s.dev_bytes;
            slab_free(s);
            ctx->slabs_owned--;
        }
    }
    delete plan;
}

int64_t flexsp_plan_num_items(const flexsp_plan *plan, int pass)
{
    if (!plan || pass < 0 || pass > 2) return FLEXSP_INVALID_ARGUMENT;
    return (int64_t)plan->pass[pass].items.size();
}

int flexsp_plan_get_items(const flexsp_plan *plan, int pass, flexsp_item *items, int64_t capacity,
                          int64_t *queue_offsets)
{
    if (!plan || pass < 0 || pass > 2) return FLEXSP_INVALID_ARGUMENT;
    const HostPass &hp = plan->pass[pass];
    if (capacity < (int64_t)hp.items.size() || (!items && !hp.items.empty())) return FLEXSP_INVALID_ARGUMENT;
    if (!hp.items.empty()) std::memcpy(items, hp.items.data(), hp.items.size() * sizeof(flexsp_item));
    if (queue_offsets)
        for (int x = 0; x <= plan->ctx->num_xcd; x++) queue_offsets[x] = hp.offsets[x];
    return FLEXSP_OK;
}

int flexsp_plan_tile_rows(const flexsp_plan *plan, int pass)
{
    if (!plan || pass < 0 || pass > 2) return FLEXSP_INVALID_ARGUMENT;
    return plan->pass[pass].tile_rows;
}

size_t flexsp_attn_bwd_workspace_bytes(const flexsp_plan *plan) { return plan ? plan->delta_bytes : 0; }

static int permute_entry(flexsp_ctx *ctx, const void *src, void *dst, int64_t T, int32_t H, int32_t D,
                         int32_t P, int32_t eb, flexsp_stream stream, bool unpack)
{
    if (T < 0 || H <= 0 || D <= 0 || P <= 0 || eb <= 0) return FLEXSP_INVALID_ARGUMENT;
    if (H % P != 0) return FLEXSP_INVALID_ARGUMENT;
    if (eb != 1 && eb != 2 && eb != 4 && eb != 8 && eb != 16) return FLEXSP_UNSUPPORTED;
    if (!ctx) return FLEXSP_INVALID_ARGUMENT;
    if (T == 0) return FLEXSP_OK;
    if (!src || !dst) return FLEXSP_INVALID_ARGUMENT;
    int64_t bytes = T * H * D * eb;
    const char *s = (const char *)src;
    const char *d = (const char *)dst;
    if (s < d + bytes && d < s + bytes) return FLEXSP_INVALID_ARGUMENT;  // overlap
    if (((uintptr_t)src | (uintptr_t)dst) % (uintptr_t)eb) return FLEXSP_INVALID_ARGUMENT;
    if (ctx->device < 0) return FLEXSP_NO_DEVICE;
    hipError_t e;
    {
        Timed tm(ctx, unpack ? FLEXSP_K_UNPACK : FLEXSP_K_PACK, (hipStream_t)stream);
        e = launch_pack(src, dst, T, H, D, P, eb, unpack, (hipStream_t)stream);
    }
    return e == hipSuccess ? FLEXSP_OK : hip_fail(e);
}

static int permute_many_entry(flexsp_ctx *ctx, int32_t n, const void *const *src, void *const *dst, int64_t T,
                              const int32_t *H, int32_t D, int32_t P, int32_t eb, flexsp_stream stream, bool unpack)
{
    if (n < 0 || n > FLEXSP_PACK_MANY_MAX || (n > 0 && (!src || !dst || !H))) return FLEXSP_INVALID_ARGUMENT;
    if (T < 0 || D <= 0 || P <= 0 || eb <= 0) return FLEXSP_INVALID_ARGUMENT;
    if (eb != 1 && eb != 2 && eb != 4 && eb != 8 && eb != 16) return FLEXSP_UNSUPPORTED;
    if (!ctx) return FLEXSP_INVALID_ARGUMENT;
    for (int i = 0; i < n; i++)
        if (H[i] <= 0 || H[i] % P != 0) return FLEXSP_INVALID_ARGUMENT;
    if (T == 0 || n == 0) return FLEXSP_OK;
    // every source against every destination: none may overlap
    for (int i = 0; i < n; i++) {
        if (!src[i] || !dst[i]) return FLEXSP_INVALID_ARGUMENT;
        if (((uintptr_t)src[i] | (uintptr_t)dst[i]) % (uintptr_t)eb) return FLEXSP_INVALID_ARGUMENT;
    }
    for (int i = 0; i < n; i++)
        for (int j = 0; j < n; j++) {
            const char *s = (const char *)src[i], *d = (const char *)dst[j];
            const int64_t sb = T * H[i] * D * eb, db = T * H[j] * D * eb;
            if (s < d + db && d < s + sb) return FLEXSP_INVALID_ARGUMENT;
            if (i < j) {
                const char *d2 = (const char *)dst[i];
                if (d2 < d + db && d < d2 + sb) return FLEXSP_INVALID_ARGUMENT;  // two destinations overlap
            }
        }
    if (ctx->device < 0) return FLEXSP_NO_DEVICE;
    hipError_t e;
    {
        Timed tm(ctx, unpack ? FLEXSP_K_UNPACK : FLEXSP_K_PACK, (hipStream_t)stream);
        e = launch_pack_many(n, src, dst, T, H, D, P, eb, unpack, (hipStream_t)stream);
    }
    return e == hipSuccess ? FLEXSP_OK : hip_fail(e);
}

int flexsp_pack_many(flexsp_ctx *ctx, int32_t n, const void *const *src, void *const *dst, int64_t T,
                     const int32_t *H, int32_t D, int32_t P, int32_t eb, flexsp_stream stream)
{
    return permute_many_entry(ctx, n, src, dst, T, H, D, P, eb, stream, false);
}

int flexsp_unpack_many(flexsp_ctx *ctx, int32_t n, const void *const *src, void *const *dst, int64_t T,
                       const int32_t *H, int32_t D, int32_t P, int32_t eb, flexsp_stream stream)
{
    return permute_many_entry(ctx, n, src, dst, T, H, D, P, eb, stream, true);
}

int flexsp_pack(flexsp_ctx *ctx, const void *src, void *dst, int64_t T, int32_t H, int32_t D, int32_t P,
                int32_t eb, flexsp_stream stream)
{
    return permute_entry(ctx, src, dst, T, H, D, P, eb, stream, false);
}

int flexsp_unpack(flexsp_ctx *ctx, const void *src, void *dst, int64_t T, int32_t H, int32_t D, int32_t P,
                  int32_t eb, flexsp_stream stream)
{
    return permute_entry(ctx, src, dst, T, H, D, P, eb, stream, true);
}

int flexsp_attn_varlen_fwd(flexsp_ctx *ctx, flexsp_plan *plan, flexsp_tensor q, flexsp_tensor k,
                           flexsp_tensor v, const int32_t *cu_dev, int32_t head_begin, int32_t head_count,
                           int32_t kv_head_begin, int32_t kv_head_count, int causal, float scale,
                           flexsp_tensor o, float *lse, flexsp_stream stream)
{
    int rc = check_attn_common(ctx, plan, cu_dev, head_begin, head_count, kv_head_begin, kv_head_count, causal);
    if (rc == FLEXSP_NO_DEVICE) {
        // still report bad views first, so host-only tests can see them
        if (!view_ok(q) || !view_ok(k) || !view_ok(v) || !view_ok(o) || !lse) return FLEXSP_INVALID_ARGUMENT;
        return rc;
    }
    if (rc) return rc;
    if (!view_ok(q) || !view_ok(k) || !view_ok(v) || !view_ok(o) || !lse) return FLEXSP_INVALID_ARGUMENT;
    if (!std::isfinite(scale)) return FLEXSP_INVALID_ARGUMENT;
    if (plan->pass[FLEXSP_PASS_FWD].items.empty()) return FLEXSP_OK;
    {
        hipError_t pe = plan_before_launch(plan, (hipStream_t)stream);
        if (pe != hipSuccess) return hip_fail(pe);
    }
    if (scale <= 0.f) scale = 1.0f / std::sqrt((float)plan->D);
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
    a.T = (int32_t)plan->T; a.Hq = plan->Hq; a.G = plan->Hq / plan->Hkv; a.causal = plan->causal;
    a.scale = scale; a.scale_l2 = scale * 1.4426950408889634f;
    a.pq = plan->dq[FLEXSP_PASS_FWD];
    hipError_t e;
    {
        Timed tm(ctx, FLEXSP_K_FWD, (hipStream_t)stream);
        e = launch_attn_fwd(a, plan->D, grid_for(ctx, plan->pass[FLEXSP_PASS_FWD], 2), (hipStream_t)stream);
    }
    return e == hipSuccess ? FLEXSP_OK : hip_fail(e);
}

int flexsp_attn_varlen_fwd_kvshard(flexsp_ctx *ctx, flexsp_plan *plan, flexsp_tensor q, flexsp_tensor k,
                                   flexsp_tensor v, int32_t head_begin, int32_t head_count, int32_t kv_head_begin,
                                   int32_t kv_head_count, int causal, float scale, flexsp_tensor o, float *lse,
                                   flexsp_stream stream)
{
    if (!ctx || !plan) return FLEXSP_INVALID_ARGUMENT;
    if (plan->ctx != ctx || !plan->kvshard) return FLEXSP_PLAN_MISMATCH;
    if (head_begin < 0 || kv_head_begin < 0 || head_count <= 0 || kv_head_count <= 0 ||
        head_count % kv_head_count != 0)
        return FLEXSP_INVALID_ARGUMENT;
    if (head_count != plan->Hq || kv_head_count != plan->Hkv || (causal != 0) != (plan->causal != 0))
        return FLEXSP_PLAN_MISMATCH;
    if (!view_ok(q) || !view_ok(k) || !view_ok(v) || !view_ok(o) || !lse || !std::isfinite(scale))
        return FLEXSP_INVALID_ARGUMENT;
    if (ctx->device < 0 || !plan->dev_base) return FLEXSP_NO_DEVICE;
    if (plan->pass[FLEXSP_PASS_FWD].items.empty()) return FLEXSP_OK;
    {
        hipError_t pe = plan_before_launch(plan, (hipStream_t)stream);
        if (pe != hipSuccess) return hip_fail(pe);
    }
    if (scale <= 0.f) scale = 1.0f / std::sqrt((float)plan->D);
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
    a.T = (int32_t)plan->T; a.Hq = plan->Hq; a.G = plan->Hq / plan->Hkv; a.causal = plan->causal;
    a.scale = scale; a.scale_l2 = scale * 1.4426950408889634f;
    a.pq = plan->dq[FLEXSP_PASS_FWD];
    hipError_t e;
    {
        Timed tm(ctx, FLEXSP_K_FWD, (hipStream_t)stream);
        e = launch_attn_fwd_kvshard(a, plan->D, grid_for(ctx, plan->pass[FLEXSP_PASS_FWD], 2), (hipStream_t)stream);
    }
    return e == hipSuccess ? FLEXSP_OK : hip_fail(e);
}

int flexsp_attn_varlen_fwd_kvshard_acc(flexsp_ctx *ctx, flexsp_plan *plan, flexsp_tensor q, flexsp_tensor k,
                                       flexsp_tensor v, int32_t head_begin, int32_t head_count, int32_t kv_head_begin,
                                       int32_t kv_head_count, int causal, float scale, flexsp_tensor o_acc,
                                       float *lse_acc, flexsp_tensor o_bf16, flexsp_stream stream)
{
    if (!ctx || !plan) return FLEXSP_INVALID_ARGUMENT;
    if (plan->ctx != ctx || !plan->kvshard) return FLEXSP_PLAN_MISMATCH;
    if (head_begin < 0 || kv_head_begin < 0 || head_count <= 0 || kv_head_count <= 0 ||
        head_count % kv_head_count != 0)
        return FLEXSP_INVALID_ARGUMENT;
    if (head_count != plan->Hq || kv_head_count != plan->Hkv || (causal != 0) != (plan->causal != 0))
        return FLEXSP_PLAN_MISMATCH;
    if (!view_ok(q) || !view_ok(k) || !view_ok(v) || !view_ok(o_acc) || (o_bf16.ptr && !view_ok(o_bf16)) || !lse_acc ||
        !std::isfinite(scale))
        return FLEXSP_INVALID_ARGUMENT;
    if (ctx->device < 0 || !plan->dev_base) return FLEXSP_NO_DEVICE;
    if (plan->pass[FLEXSP_PASS_FWD].items.empty()) return FLEXSP_OK;
    {
        hipError_t pe = plan_before_launch(plan, (hipStream_t)stream);
        if (pe != hipSuccess) return hip_fail(pe);
    }
    if (scale <= 0.f) scale = 1.0f / std::sqrt((float)plan->D);
    AttnArgs a;
    std::memset(&a, 0, sizeof(a));
    a.q = (const uint16_t *)q.ptr + (int64_t)head_begin * q.stride_head;
    a.k = (const uint16_t *)k.ptr + (int64_t)kv_head_begin * k.stride_head;
    a.v = (const uint16_t *)v.ptr + (int64_t)kv_head_begin * v.stride_head;
    // the kernel's fold mode: the fp32 running result travels in the fields the forward does not use otherwise
    a.dq = (float *)o_acc.ptr + (int64_t)head_begin * o_acc.stride_head;
    a.dq_st = (int32_t)o_acc.stride_token; a.dq_sh = (int32_t)o_acc.stride_head;
    a.delta_out = lse_acc;
    if (o_bf16.ptr) {
        a.out_o = (uint16_t *)o_bf16.ptr + (int64_t)head_begin * o_bf16.stride_head;
        a.o_st = (int32_t)o_bf16.stride_token; a.o_sh = (int32_t)o_bf16.stride_head;
    }
    a.q_st = (int32_t)q.stride_token; a.q_sh = (int32_t)q.stride_head;
    a.k_st = (int32_t)k.stride_token; a.k_sh = (int32_t)k.stride_head;
    a.v_st = (int32_t)v.stride_token; a.v_sh = (int32_t)v.stride_head;
    a.T = (int32_t)plan->T; a.Hq = plan->Hq; a.G = plan->Hq / plan->Hkv; a.causal = plan->causal;
    a.scale = scale; a.scale_l2 = scale * 1.4426950408889634f;
    a.pq = plan->dq[FLEXSP_PASS_FWD];
    hipError_t e;
    {
        Timed tm(ctx, FLEXSP_K_FWD, (hipStream_t)stream);
        e = launch_attn_fwd_kvshard(a, plan->D, grid_for(ctx, plan->pass[FLEXSP_PASS_FWD], 2), (hipStream_t)stream);
    }
    return e == hipSuccess ? FLEXSP_OK : hip_fail(e);
}

int flexsp_attn_varlen_bwd_kvshard(flexsp_ctx *ctx, flexsp_plan *plan, flexsp_tensor q, flexsp_tensor k,
                                   flexsp_tensor v, flexsp_tensor o, flexsp_tensor dO, const float *lse,
                                   int32_t head_begin, int32_t head_count, int32_t kv_head_begin,
                                   int32_t kv_head_count, int causal, float scale, flexsp_tensor dq, flexsp_tensor dk,
                                   flexsp_tensor dv, int32_t grad_dtype, int32_t accumulate, flexsp_stream stream)
{
    if (!ctx || !plan) return FLEXSP_INVALID_ARGUMENT;
    if (plan->ctx != ctx || !plan->kvshard) return FLEXSP_PLAN_MISMATCH;
    if (head_begin < 0 || kv_head_begin < 0 || head_count <= 0 || kv_head_count <= 0) return FLEXSP_INVALID_ARGUMENT;
    if (head_count % kv_head_count != 0) return FLEXSP_INVALID_ARGUMENT;
    if (head_count != plan->Hq || kv_head_count != plan->Hkv || (causal != 0) != (plan->causal != 0))
        return FLEXSP_PLAN_MISMATCH;
    if (grad_dtype != FLEXSP_BF16 && grad_dtype != FLEXSP_F32) return FLEXSP_UNSUPPORTED;
    if (accumulate != 0 && accumulate != 1) return FLEXSP_INVALID_ARGUMENT;
    if (accumulate && grad_dtype != FLEXSP_F32) return FLEXSP_UNSUPPORTED;  // partial sums are kept in fp32
    const bool views = view_ok(q) && view_ok(k) && view_ok(v) && view_ok(o) && view_ok(dO) && view_ok(dq) &&
                       view_ok(dk) && view_ok(dv) && lse;
    if (!views || !std::isfinite(scale)) return FLEXSP_INVALID_ARGUMENT;
    if (ctx->device < 0 || !plan->dev_base) return FLEXSP_NO_DEVICE;
    if (plan->pass[FLEXSP_PASS_BWD_DQ].items.empty() && plan->pass[FLEXSP_PASS_BWD_DKV].items.empty()) return FLEXSP_OK;
    {
        hipError_t pe = plan_before_launch(plan, (hipStream_t)stream);
        if (pe != hipSuccess) return hip_fail(pe);
    }
    if (scale <= 0.f) scale = 1.0f / std::sqrt((float)plan->D);
    AttnArgs a;
    std::memset(&a, 0, sizeof(a));
    a.q = (const uint16_t *)q.ptr + (int64_t)head_begin * q.stride_head;
    a.k = (const uint16_t *)k.ptr + (int64_t)kv_head_begin * k.stride_head;
    a.v = (const uint16_t *)v.ptr + (int64_t)kv_head_begin * v.stride_head;
    a.o = (const uint16_t *)o.ptr + (int64_t)head_begin * o.stride_head;
    a.dO = (const uint16_t *)dO.ptr + (int64_t)head_begin * dO.stride_head;
    const int64_t gb = grad_dtype == FLEXSP_F32 ? 4 : 2;
    a.grad_f32 = (grad_dtype == FLEXSP_F32 ? 1 : 0) | (accumulate ? 2 : 0);
    a.dq = (char *)dq.ptr + (int64_t)head_begin * dq.stride_head * gb;
    a.dk = (char *)dk.ptr + (int64_t)kv_head_begin * dk.stride_head * gb;
    a.dv = (char *)dv.ptr + (int64_t)kv_head_begin * dv.stride_head * gb;
    a.q_st = (int32_t)q.stride_token; a.q_sh = (int32_t)q.stride_head;
    a.k_st = (int32_t)k.stride_token; a.k_sh = (int32_t)k.stride_head;
    a.v_st = (int32_t)v.stride_token; a.v_sh = (int32_t)v.stride_head;
    a.o_st = (int32_t)o.stride_token; a.o_sh = (int32_t)o.stride_head;
    a.do_st = (int32_t)dO.stride_token; a.do_sh = (int32_t)dO.stride_head;
    a.dq_st = (int32_t)dq.stride_token; a.dq_sh = (int32_t)dq.stride_head;
    a.dk_st = (int32_t)dk.stride_token; a.dk_sh = (int32_t)dk.stride_head;
    a.dv_st = (int32_t)dv.stride_token; a.dv_sh = (int32_t)dv.stride_head;
    float *lse2 = plan->delta + (size_t)plan->T * plan->Hq;
    a.T = (int32_t)plan->T; a.Hq = plan->Hq; a.G = plan->Hq / plan->Hkv; a.causal = plan->causal;
    a.scale = scale; a.scale_l2 = scale * 1.4426950408889634f;
    hipStream_t s = (hipStream_t)stream;
    hipError_t e = hipSuccess;
    // as in flexsp_attn_varlen_bwd: the dQ kernel leaves delta and the base-2 log-sum-exp of its rows in
    // the plan's scratch for the dK/dV kernel
    a.lse_in = lse;
    a.lse_out = lse2;
    a.delta_out = plan->delta;
    a.pq = plan->dq[FLEXSP_PASS_BWD_DQ];
    if (!plan->pass[FLEXSP_PASS_BWD_DQ].items.empty()) {
        Timed tm(ctx, FLEXSP_K_BWD_DQ, s);
        e = launch_attn_bwd_dq_kvshard(a, plan->D, grid_for(ctx, plan->pass[FLEXSP_PASS_BWD_DQ], 2), s);
    }
    if (e != hipSuccess) return hip_fail(e);
    a.lse_in = lse2;
    a.delta_in = plan->delta;
    a.pq = plan->dq[FLEXSP_PASS_BWD_DKV];
    if (!plan->pass[FLEXSP_PASS_BWD_DKV].items.empty()) {
        Timed tm(ctx, FLEXSP_K_BWD_DKV, s);
        e = launch_attn_bwd_dkv_kvshard(a, plan->D, grid_for(ctx, plan->pass[FLEXSP_PASS_BWD_DKV], 2), s);
    }
    return e == hipSuccess ? FLEXSP_OK : hip_fail(e);
}

int flexsp_lse_merge(flexsp_ctx *ctx, flexsp_tensor o_a, const float *lse_a, flexsp_tensor o_b, const float *lse_b,
                     flexsp_tensor o_out, float *lse_out, int64_t T, int32_t H, int32_t D, flexsp_stream stream)
{
    if (!ctx || T < 0 || H <= 0 || D <= 0) return FLEXSP_INVALID_ARGUMENT;
    if (D != 64 && D != 128) return FLEXSP_UNSUPPORTED;  // (a row's pieces then share one wavefront: in-place use is safe)
    if (T == 0) return FLEXSP_OK;
    if (!view_ok(o_a) || !view_ok(o_b) || !view_ok(o_out) || !lse_a || !lse_b || !lse_out)
        return FLEXSP_INVALID_ARGUMENT;
    if (T * (int64_t)H * (D / 8) >= ((int64_t)1 << 31)) return FLEXSP_UNSUPPORTED;
    if (ctx->device < 0) return FLEXSP_NO_DEVICE;
    hipError_t e = launch_lse_merge((const uint16_t *)o_a.ptr, lse_a, (const uint16_t *)o_b.ptr, lse_b,
                                    (uint16_t *)o_out.ptr, lse_out, T, H, D, (int32_t)o_a.stride_token,
                                    (int32_t)o_a.stride_head, (int32_t)o_b.stride_token, (int32_t)o_b.stride_head,
                                    (int32_t)o_out.stride_token, (int32_t)o_out.stride_head, (hipStream_t)stream);
    return e == hipSuccess ? FLEXSP_OK : hip_fail(e);
}

int flexsp_lse_merge_acc(flexsp_ctx *ctx, flexsp_tensor o_acc, float *lse_acc, flexsp_tensor o_b, const float *lse_b,
                         flexsp_tensor o_bf16, int64_t T, int32_t H, int32_t D, flexsp_stream stream)
{
    if (!ctx || T < 0 || H <= 0 || D <= 0) return FLEXSP_INVALID_ARGUMENT;
    if (D != 64 && D != 128) return FLEXSP_UNSUPPORTED;
    if (T == 0) return FLEXSP_OK;
    if (!view_ok(o_acc) || !view_ok(o_b) || (o_bf16.ptr && !view_ok(o_bf16)) || !lse_acc || !lse_b)
        return FLEXSP_INVALID_ARGUMENT;
    if (T * (int64_t)H * (D / 8) >= ((int64_t)1 << 31)) return FLEXSP_UNSUPPORTED;
    if (ctx->device < 0) return FLEXSP_NO_DEVICE;
    hipError_t e = launch_lse_merge_acc((float *)o_acc.ptr, lse_acc, (const uint16_t *)o_b.ptr, lse_b, (uint16_t *)o_bf16.ptr,
                                        T, H, D, (int32_t)o_acc.stride_token, (int32_t)o_acc.stride_head,
                                        (int32_t)o_b.stride_token, (int32_t)o_b.stride_head,
                                        o_bf16.ptr ? (int32_t)o_bf16.stride_token : 0,
                                        o_bf16.ptr ? (int32_t)o_bf16.stride_head : 0, (hipStream_t)stream);
    return e == hipSuccess ? FLEXSP_OK : hip_fail(e);
}

int flexsp_attn_varlen_bwd(flexsp_ctx *ctx, flexsp_plan *plan, flexsp_tensor q, flexsp_tensor k,
                           flexsp_tensor v, flexsp_tensor o, flexsp_tensor dO, const float *lse,
                           const int32_t *cu_dev, int32_t head_begin, int32_t head_count,
                           int32_t kv_head_begin, int32_t kv_head_count, int causal, float scale,
                           flexsp_tensor dq, flexsp_tensor dk, flexsp_tensor dv, int32_t grad_dtype,
                           flexsp_stream stream)
{
    int rc = check_attn_common(ctx, plan, cu_dev, head_begin, head_count, kv_head_begin, kv_head_count, causal);
    bool views = view_ok(q) && view_ok(k) && view_ok(v) && view_ok(o) && view_ok(dO) && view_ok(dq) &&
                 view_ok(dk) && view_ok(dv) && lse;
    if (rc == FLEXSP_NO_DEVICE && !views) return FLEXSP_INVALID_ARGUMENT;
    if ((rc == FLEXSP_OK || rc == FLEXSP_NO_DEVICE) && grad_dtype != FLEXSP_BF16 && grad_dtype != FLEXSP_F32)
        return FLEXSP_UNSUPPORTED;
    if (rc) return rc;
    if (!views || !std::isfinite(scale)) return FLEXSP_INVALID_ARGUMENT;
    if (plan->pass[FLEXSP_PASS_FWD].items.empty()) return FLEXSP_OK;
    {
        hipError_t pe = plan_before_launch(plan, (hipStream_t)stream);
        if (pe != hipSuccess) return hip_fail(pe);
    }
    if (scale <= 0.f) scale = 1.0f / std::sqrt((float)plan->D);
    AttnArgs a;
    std::memset(&a, 0, sizeof(a));
    a.q = (const uint16_t *)q.ptr + (int64_t)head_begin * q.stride_head;
    a.k = (const uint16_t *)k.ptr + (int64_t)kv_head_begin * k.stride_head;
    a.v = (const uint16_t *)v.ptr + (int64_t)kv_head_begin * v.stride_head;
    a.o = (const uint16_t *)o.ptr + (int64_t)head_begin * o.stride_head;
    a.dO = (const uint16_t *)dO.ptr + (int64_t)head_begin * dO.stride_head;
    const int64_t gb = grad_dtype == FLEXSP_F32 ? 4 : 2;
    a.grad_f32 = grad_dtype == FLEXSP_F32;
    a.dq = (char *)dq.ptr + (int64_t)head_begin * dq.stride_head * gb;
    a.dk = (char *)dk.ptr + (int64_t)kv_head_begin * dk.stride_head * gb;
    a.dv = (char *)dv.ptr + (int64_t)kv_head_begin * dv.stride_head * gb;
    a.q_st = (int32_t)q.stride_token; a.q_sh = (int32_t)q.stride_head;
    a.k_st = (int32_t)k.stride_token; a.k_sh = (int32_t)k.stride_head;
    a.v_st = (int32_t)v.stride_token; a.v_sh = (int32_t)v.stride_head;
    a.o_st = (int32_t)o.stride_token; a.o_sh = (int32_t)o.stride_head;
    a.do_st = (int32_t)dO.stride_token; a.do_sh = (int32_t)dO.stride_head;
    a.dq_st = (int32_t)dq.stride_token; a.dq_sh = (int32_t)dq.stride_head;
    a.dk_st = (int32_t)dk.stride_token; a.dk_sh = (int32_t)dk.stride_head;
    a.dv_st = (int32_t)dv.stride_token; a.dv_sh = (int32_t)dv.stride_head;
    float *lse2 = plan->delta + (size_t)plan->T * plan->Hq;
    a.T = (int32_t)plan->T; a.Hq = plan->Hq; a.G = plan->Hq / plan->Hkv; a.causal = plan->causal;
    a.scale = scale; a.scale_l2 = scale * 1.4426950408889634f;
    hipStream_t s = (hipStream_t)stream;
    hipError_t e;
    // The dQ kernel runs first: it holds every query row's dO in registers, so it also computes
    // delta = dO . O and the log-sum-exp in base 2 for its rows and leaves both in the plan's
    // scratch for the dK/dV kernel (no separate preprocessing launch).
    a.lse_in = lse;
    a.lse_out = lse2;
    a.delta_out = plan->delta;
    a.pq = plan->dq[FLEXSP_PASS_BWD_DQ];
    {
        Timed tm(ctx, FLEXSP_K_BWD_DQ, s);
        e = launch_attn_bwd_dq(a, plan->D, grid_for(ctx, plan->pass[FLEXSP_PASS_BWD_DQ], 2), s);
    }
    if (e != hipSuccess) return hip_fail(e);
    a.lse_in = lse2;
    a.delta_in = plan->delta;
    a.pq = plan->dq[FLEXSP_PASS_BWD_DKV];
    {
        Timed tm(ctx, FLEXSP_K_BWD_DKV, s);
        e = launch_attn_bwd_dkv(a, plan->D, grid_for(ctx, plan->pass[FLEXSP_PASS_BWD_DKV], 2), s);
    }
    return e == hipSuccess ? FLEXSP_OK : hip_fail(e);
}

}  // extern "C"
