// Measurement support of libdvm (Section 6.1 of the paper measures run time and compile time apart):
//   dvm_encode_timed  times dvm_encode itself with the monotonic clock, no language binding in between;
//   dvm_copy_kernel   a plain copy kernel of this library's own, the bandwidth ceiling of a load-store loop on
//                     the device that the interpreter's figures are quoted against.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <time.h>

#include "../../include/dvm.h"
#include "dvm_internal.h"

extern "C" int dvm_encode_timed(const dvm_ctx *ctx, const dvm_prog *prog, const dvm_shape *in_shapes, int n_in,
                                const dvm_shape *out_layout, void *bytecode, size_t cap, size_t *len, int reps, int64_t *ns) {
    if (reps < 1 || !ns) return dvm_set_error(DVM_E_ARGS, "dvm_encode_timed: reps and ns");
    int st = DVM_OK;
    for (int r = 0; r < reps; ++r) {
        struct timespec t0, t1;
        clock_gettime(CLOCK_MONOTONIC, &t0);
        st = dvm_encode(ctx, prog, in_shapes, n_in, out_layout, bytecode, cap, len, nullptr);
        clock_gettime(CLOCK_MONOTONIC, &t1);
        ns[r] = (int64_t)(t1.tv_sec - t0.tv_sec) * 1000000000ll + (t1.tv_nsec - t0.tv_nsec);
        if (st != DVM_OK) return st;
    }
    return st;
}

namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
constexpr int COPY_THREADS = 256;
constexpr int COPY_UNROLL = 4;                                      // 16-byte accesses per lane and tile
constexpr size_t COPY_TILE_BYTES = (size_t)COPY_THREADS * COPY_UNROLL * 16;   // 16 KiB

// One tile = 256 lanes x 4 accesses of 16 bytes, each access of a wave covering 1 KiB contiguous; all loads of a
// tile are issued before its first store.  Tiles go to the workgroups blocked or interleaved.
template <bool INTERLEAVED>
__global__ void __launch_bounds__(COPY_THREADS) dvm_copy_tiles(const u32x4 *__restrict__ src, u32x4 *__restrict__ dst, uint64_t ntiles) {
    uint64_t lo, hi, step;
    if (INTERLEAVED) {
        lo = blockIdx.x; hi = ntiles; step = gridDim.x;
    } else {
        const uint64_t m = (ntiles + gridDim.x - 1) / gridDim.x;
        lo = m * blockIdx.x; hi = lo + m < ntiles ? lo + m : ntiles; step = 1;
    }
    for (uint64_t t = lo; t < hi; t += step) {
        const uint64_t base = t * (COPY_THREADS * COPY_UNROLL) + threadIdx.x;
        u32x4 v[COPY_UNROLL];
#pragma unroll
        for (int u = 0; u < COPY_UNROLL; ++u) v[u] = __builtin_nontemporal_load(&src[base + u * COPY_THREADS]);
#pragma unroll
        for (int u = 0; u < COPY_UNROLL; ++u) __builtin_nontemporal_store(v[u], &dst[base + u * COPY_THREADS]);
    }
}

}  // namespace

extern "C" int dvm_copy_kernel(const dvm_ctx *ctx, void *dst, const void *src, size_t bytes, int assignment, void *hip_stream) {
    if (!ctx || !dst || !src) return dvm_set_error(DVM_E_ARGS, "dvm_copy_kernel: null argument");
    if (dvm_ctx_device(ctx) < 0) return dvm_set_error(DVM_E_ARGS, "dvm_copy_kernel: context was created without a device");
    if (bytes == 0 || bytes % COPY_TILE_BYTES != 0) return dvm_set_error(DVM_E_ARGS, "dvm_copy_kernel: size must be a positive multiple of 16 KiB");
    if (((uintptr_t)dst | (uintptr_t)src) & 15) return dvm_set_error(DVM_E_ALIGN, "dvm_copy_kernel: pointers must be 16-byte aligned");
    if (assignment != DVM_ASSIGN_BLOCKED && assignment != DVM_ASSIGN_INTERLEAVED) return dvm_set_error(DVM_E_ARGS, "dvm_copy_kernel: unknown tile assignment");
    const uint64_t ntiles = bytes / COPY_TILE_BYTES;
    int n_cu = 256;
    dvm_ctx_planner_get(ctx, &n_cu, nullptr);
    uint64_t grid = (uint64_t)n_cu * 8;             // eight resident workgroups of four waves per compute unit
    if (grid > ntiles) grid = ntiles;
    if (assignment == DVM_ASSIGN_INTERLEAVED)
        hipLaunchKernelGGL(dvm_copy_tiles<true>, dim3((unsigned)grid), dim3(COPY_THREADS), 0, (hipStream_t)hip_stream, (const u32x4 *)src, (u32x4 *)dst, ntiles);
    else
        hipLaunchKernelGGL(dvm_copy_tiles<false>, dim3((unsigned)grid), dim3(COPY_THREADS), 0, (hipStream_t)hip_stream, (const u32x4 *)src, (u32x4 *)dst, ntiles);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return dvm_set_error(DVM_E_HIP, hipGetErrorString(e));
    return DVM_OK;
}
