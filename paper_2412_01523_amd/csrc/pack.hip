// Layout permute kernels: sequence-sharded [T, H, D] <-> head-sharded [P, T, H/P, D]
// (the local half of the exchanges in paper Sec. 2.1.2, Eq. 2 and Eq. 4).
//
// HBM-bound bit copy.  The SEQUENCE-sharded side is walked linearly, so one side of every access
// is perfectly contiguous and the other side splits into P streams (one per slab), each
// contiguous in runs of (H/P)*D*elem_bytes bytes (1 KiB for 4 heads x 128 x bf16: one 16-byte
// access per lane of a wavefront).  Walking the head-sharded side instead would make every
// workgroup that runs at the same time read the same 1/P-wide window of each token row, which
// concentrates the traffic on a fraction of the memory channels.
#include "flexsp_internal.h"

namespace flexsp {
namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
template <int VB> struct VecOf;
template <> struct VecOf<16> { typedef u32x4 type; };
template <> struct VecOf<8> { typedef u32x2 type; };
template <> struct VecOf<4> { typedef uint32_t type; };
template <> struct VecOf<2> { typedef uint16_t type; };
template <> struct VecOf<1> { typedef uint8_t type; };

constexpr int kPackThreads = 256;
constexpr int kPackMany = 4;  // tensors per launch of the multi-tensor form

// Units are vectors of VB bytes.  rc = vectors per (token, slab) run, row = vectors per
// token on the sequence-sharded side (= P * rc), slab = T * rc vectors per slab.  One vector
// per thread and one 4 KiB stretch per workgroup measured fastest (more vectors per thread
// lose 5-15 %).  IDX is the integer type of a vector index (32-bit whenever the tensor has
// fewer than 2^31 vectors); shifts replace the divisions when rc and row are powers of two.
template <int VB, bool UNPACK, typename IDX>
__global__ __launch_bounds__(kPackThreads) void permute_kernel(
    const typename VecOf<VB>::type *__restrict__ src, typename VecOf<VB>::type *__restrict__ dst,
    IDX total, IDX slab, IDX row, IDX rc, int row_shift, int rc_shift)
{
    const IDX c = (IDX)blockIdx.x * kPackThreads + threadIdx.x;  // sequence-sharded index
    if (c >= total) return;
    IDX t, e, r, w;
    if (row_shift >= 0) {
        t = c >> row_shift;
        e = c & (row - 1);
    } else {
        t = c / row;  // token
        e = c - t * row;
    }
    if (rc_shift >= 0) {
        r = e >> rc_shift;
        w = e & (rc - 1);
    } else {
        r = e / rc;  // slab (peer)
        w = e - r * rc;
    }
    const IDX o = r * slab + t * rc + w;  // head-sharded index
    if (UNPACK)
        __builtin_nontemporal_store(__builtin_nontemporal_load(&src[o]), &dst[c]);
    else
        __builtin_nontemporal_store(__builtin_nontemporal_load(&src[c]), &dst[o]);
}

// Several tensors in one launch (blockIdx.y picks the tensor): the same walk, 16-byte vectors and
// 32-bit indices only.  Saves the launches in between and lets one tensor's last workgroups
// overlap the next one's first.
struct ManyArgs {
    const u32x4 *src[kPackMany];
    u32x4 *dst[kPackMany];
    uint32_t total[kPackMany], slab[kPackMany], row[kPackMany], rc[kPackMany];
    int row_shift[kPackMany], rc_shift[kPackMany];
};
// (the tensor index is resolved by a chain of compile-time cases: indexing the by-value argument
// arrays with a run-time value would move them to scratch memory)
template <bool UNPACK, int Y>
__device__ __forceinline__ void permute_one_of_many(const ManyArgs &m, uint32_t c)
{
    if (c >= m.total[Y]) return;
    const uint32_t row = m.row[Y], rc = m.rc[Y];
    uint32_t t, e, r, w;
    if (m.row_shift[Y] >= 0) {
        t = c >> m.row_shift[Y];
        e = c & (row - 1);
    } else {
        t = c / row;
        e = c - t * row;
    }
    if (m.rc_shift[Y] >= 0) {
        r = e >> m.rc_shift[Y];
        w = e & (rc - 1);
    } else {
        r = e / rc;
        w = e - r * rc;
    }
    const uint32_t o = r * m.slab[Y] + t * rc + w;
    if (UNPACK)
        __builtin_nontemporal_store(__builtin_nontemporal_load(&m.src[Y][o]), &m.dst[Y][c]);
    else
        __builtin_nontemporal_store(__builtin_nontemporal_load(&m.src[Y][c]), &m.dst[Y][o]);
}
template <bool UNPACK>
__global__ __launch_bounds__(kPackThreads) void permute_many_kernel(const ManyArgs m)
{
    static_assert(kPackMany == 4, "one case per tensor below");
    const uint32_t c = blockIdx.x * kPackThreads + threadIdx.x;
    switch (blockIdx.y) {
    case 0: permute_one_of_many<UNPACK, 0>(m, c); break;
    case 1: permute_one_of_many<UNPACK, 1>(m, c); break;
    case 2: permute_one_of_many<UNPACK, 2>(m, c); break;
    default: permute_one_of_many<UNPACK, 3>(m, c); break;
    }
}

inline int shift_of(int64_t x)
{
    if (x <= 0 || (x & (x - 1)) != 0) return -1;
    int sft = 0;
    while (((int64_t)1 << sft) < x) sft++;
    return sft;
}

template <int VB, typename IDX>
hipError_t launch_idx(const void *src, void *dst, int64_t total, int64_t slab, int64_t row, int64_t rc,
                      bool unpack, hipStream_t s)
{
    typedef typename VecOf<VB>::type V;
    int64_t blocks = (total + kPackThreads - 1) / kPackThreads;
    if (blocks > 0x7fffffff) return hipErrorInvalidValue;
    if (unpack)
        hipLaunchKernelGGL((permute_kernel<VB, true, IDX>), dim3((unsigned)blocks), dim3(kPackThreads), 0, s,
                           (const V *)src, (V *)dst, (IDX)total, (IDX)slab, (IDX)row, (IDX)rc, shift_of(row),
                           shift_of(rc));
    else
        hipLaunchKernelGGL((permute_kernel<VB, false, IDX>), dim3((unsigned)blocks), dim3(kPackThreads), 0, s,
                           (const V *)src, (V *)dst, (IDX)total, (IDX)slab, (IDX)row, (IDX)rc, shift_of(row),
                           shift_of(rc));
    return hipGetLastError();
}

template <int VB>
hipError_t launch_vb(const void *src, void *dst, int64_t bytes, int64_t T, int64_t run_bytes, int P,
                     bool unpack, hipStream_t s)
{
    int64_t total = bytes / VB;
    int64_t rc = run_bytes / VB;
    int64_t slab = T * rc, row = (int64_t)P * rc;
    if (total + kPackThreads < ((int64_t)1 << 31))
        return launch_idx<VB, uint32_t>(src, dst, total, slab, row, rc, unpack, s);
    return launch_idx<VB, int64_t>(src, dst, total, slab, row, rc, unpack, s);
}

}  // namespace

hipError_t launch_pack(const void *src, void *dst, int64_t T, int H, int D, int P, int eb, bool unpack,
                       hipStream_t s)
{
    int64_t run_bytes = (int64_t)(H / P) * D * eb;
    int64_t bytes = T * P * run_bytes;
    if (bytes == 0) return hipSuccess;
    uintptr_t bits = (uintptr_t)src | (uintptr_t)dst | (uintptr_t)run_bytes;
    if ((bits & 15) == 0) return launch_vb<16>(src, dst, bytes, T, run_bytes, P, unpack, s);
    if ((bits & 7) == 0) return launch_vb<8>(src, dst, bytes, T, run_bytes, P, unpack, s);
    if ((bits & 3) == 0) return launch_vb<4>(src, dst, bytes, T, run_bytes, P, unpack, s);
    if ((bits & 1) == 0) return launch_vb<2>(src, dst, bytes, T, run_bytes, P, unpack, s);
    return launch_vb<1>(src, dst, bytes, T, run_bytes, P, unpack, s);
}

// n tensors [T, H[i], D] with the same T, D, P and element size.  One launch when every tensor
// qualifies for 16-byte vectors and 32-bit indices, otherwise one launch per tensor.
hipError_t launch_pack_many(int n, const void *const *src, void *const *dst, int64_t T, const int32_t *H, int D,
                            int P, int eb, bool unpack, hipStream_t s)
{
    ManyArgs m;
    bool fast = n <= kPackMany;
    int64_t most = 0;
    for (int i = 0; i < n && fast; i++) {
        const int64_t run_bytes = (int64_t)(H[i] / P) * D * eb, bytes = T * P * run_bytes;
        const uintptr_t bits = (uintptr_t)src[i] | (uintptr_t)dst[i] | (uintptr_t)run_bytes;
        const int64_t total = bytes / 16;
        if ((bits & 15) != 0 || total + kPackThreads >= ((int64_t)1 << 31)) {
            fast = false;
            break;
        }
        const int64_t rc = run_bytes / 16;
        m.src[i] = (const u32x4 *)src[i];
        m.dst[i] = (u32x4 *)dst[i];
        m.total[i] = (uint32_t)total;
        m.rc[i] = (uint32_t)rc;
        m.slab[i] = (uint32_t)(T * rc);
        m.row[i] = (uint32_t)((int64_t)P * rc);
        m.row_shift[i] = shift_of((int64_t)P * rc);
        m.rc_shift[i] = shift_of(rc);
        most = total > most ? total : most;
    }
    if (!fast) {
        for (int i = 0; i < n; i++) {
            hipError_t e = launch_pack(src[i], dst[i], T, H[i], D, P, eb, unpack, s);
            if (e != hipSuccess) return e;
        }
        return hipSuccess;
    }
    if (most == 0) return hipSuccess;
    for (int i = n; i < kPackMany; i++) {
        m.src[i] = nullptr; m.dst[i] = nullptr;
        m.total[i] = 0; m.slab[i] = 0; m.row[i] = 1; m.rc[i] = 1; m.row_shift[i] = 0; m.rc_shift[i] = 0;
    }
    const dim3 grid((unsigned)((most + kPackThreads - 1) / kPackThreads), (unsigned)n);
    if (unpack)
        hipLaunchKernelGGL(permute_many_kernel<true>, grid, dim3(kPackThreads), 0, s, m);
    else
        hipLaunchKernelGGL(permute_many_kernel<false>, grid, dim3(kPackThreads), 0, s, m);
    return hipGetLastError();
}

}  // namespace flexsp
