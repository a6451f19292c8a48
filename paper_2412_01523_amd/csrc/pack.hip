// Layout permute kernels: sequence-sharded [T, H, D] <-> head-sharded [P, T, H/P, D]
// (the local half of the exchanges in paper Sec. 2.1.2, Eq. 2 and Eq. 4).
//
// HBM-bound bit copy.  The head-sharded side is walked linearly, so one side of every
// access is perfectly contiguous and the other side is contiguous in runs of
// (H/P)*D*elem_bytes bytes (1 KiB for 4 heads x 128 x bf16: one 16-byte access per lane of
// a wavefront).  Each thread keeps UNROLL independent 16-byte loads in flight.
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
constexpr int kPackUnroll = 8;

// Units are vectors of VB bytes.  rc = vectors per (token, slab) run, row = vectors per
// token on the sequence-sharded side (= P * rc), slab = T * rc vectors per slab.
// rc_shift >= 0 when rc is a power of two.
template <int VB, bool UNPACK>
__global__ __launch_bounds__(kPackThreads) void permute_kernel(
    const typename VecOf<VB>::type *__restrict__ src, typename VecOf<VB>::type *__restrict__ dst,
    int64_t total, int64_t slab, int64_t row, int32_t rc, int32_t rc_shift)
{
    typedef typename VecOf<VB>::type V;
    const int64_t tile = (int64_t)kPackThreads * kPackUnroll;
    for (int64_t base = (int64_t)blockIdx.x * tile; base < total; base += (int64_t)gridDim.x * tile) {
        int64_t lin[kPackUnroll], str[kPackUnroll];
        V val[kPackUnroll];
#pragma unroll
        for (int u = 0; u < kPackUnroll; u++) {
            int64_t c = base + (int64_t)u * kPackThreads + threadIdx.x;  // head-sharded index
            lin[u] = c;
            int64_t r = c / slab;  // slab (peer) index
            int64_t e = c - r * slab;
            int64_t t, w;
            if (rc_shift >= 0) {
                t = e >> rc_shift;
                w = e & (rc - 1);
            } else {
                t = e / rc;
                w = e - t * rc;
            }
            str[u] = t * row + r * rc + w;  // sequence-sharded index
        }
#pragma unroll
        for (int u = 0; u < kPackUnroll; u++)
            if (lin[u] < total) val[u] = __builtin_nontemporal_load(&src[UNPACK ? lin[u] : str[u]]);
#pragma unroll
        for (int u = 0; u < kPackUnroll; u++)
            if (lin[u] < total) __builtin_nontemporal_store(val[u], &dst[UNPACK ? str[u] : lin[u]]);
    }
}

template <int VB>
hipError_t launch_vb(const void *src, void *dst, int64_t bytes, int64_t T, int64_t run_bytes, int P,
                     bool unpack, hipStream_t s)
{
    typedef typename VecOf<VB>::type V;
    int64_t total = bytes / VB;
    int32_t rc = (int32_t)(run_bytes / VB);
    int32_t shift = -1;
    if ((rc & (rc - 1)) == 0) {
        shift = 0;
        while ((1 << shift) < rc) shift++;
    }
    int64_t slab = T * rc, row = (int64_t)P * rc;
    int64_t tile = (int64_t)kPackThreads * kPackUnroll;
    int64_t blocks = (total + tile - 1) / tile;
    if (blocks > 256 * 32) blocks = 256 * 32;
    if (unpack)
        hipLaunchKernelGGL((permute_kernel<VB, true>), dim3((unsigned)blocks), dim3(kPackThreads), 0, s,
                           (const V *)src, (V *)dst, total, slab, row, rc, shift);
    else
        hipLaunchKernelGGL((permute_kernel<VB, false>), dim3((unsigned)blocks), dim3(kPackThreads), 0, s,
                           (const V *)src, (V *)dst, total, slab, row, rc, shift);
    return hipGetLastError();
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

}  // namespace flexsp
