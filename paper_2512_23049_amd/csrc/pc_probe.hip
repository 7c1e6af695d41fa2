// Achievable-peak probes: what this GPU sustains for the two resources the attention kernels
// are priced against, measured the same way the kernels are (events on the caller's stream).
// They belong to the benchmark, not to the attention path; nothing else in the library calls them.
#include <hip/hip_runtime.h>

#include <cstdint>

#include "../../include/pc_probe.h"

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

constexpr int PROBE_CHAINS = 4;          // independent accumulators per wave: no MFMA waits for another
constexpr int PROBE_UNROLL = 4;          // MFMAs per chain per loop trip
constexpr int PROBE_SETS = 8;            // operand fragment sets a wave cycles through

// Every wave runs iters * 16 MFMAs (32x32x16 bf16) on operand fragments read once from
// `operands` (set s, lane l: 32 bytes at ((s * 64 + l) * 32), A then B).  Consecutive MFMAs take
// different A and B fragments (MFMA i of a loop trip: A set i mod 8, B set 3 i mod 8, so the 16 MFMAs
// of a trip see 16 different (A, B) pairs) and the accumulators change all the time: the matrix
// core's inputs toggle from one instruction to the next as they do in an attention loop.  The
// power a matrix core draws, and with it the clock the chip holds, depends on how many operand
// bits toggle, so the caller chooses the data: all-zero operands give the datasheet rate, random
// ones the rate real data can reach.
__global__ __launch_bounds__(256) void pc_probe_mfma_kernel(const uint4 *__restrict__ operands,
                                                            int iters, float *sink) {
    const int lane = threadIdx.x & 63;
    bf16x8 a[PROBE_SETS], b[PROBE_SETS];
    f32x16 acc[PROBE_CHAINS];
#pragma unroll
    for (int s = 0; s < PROBE_SETS; ++s) {
        a[s] = __builtin_bit_cast(bf16x8, operands[(s * 64 + lane) * 2]);
        b[s] = __builtin_bit_cast(bf16x8, operands[(s * 64 + lane) * 2 + 1]);
    }
#pragma unroll
    for (int c = 0; c < PROBE_CHAINS; ++c)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[c][r] = 0.f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int u = 0; u < PROBE_UNROLL; ++u)
#pragma unroll
            for (int c = 0; c < PROBE_CHAINS; ++c) {
                const int i = u * PROBE_CHAINS + c;
                acc[c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i % PROBE_SETS], b[(3 * i) % PROBE_SETS], acc[c], 0, 0, 0);
            }
    }
    float s = 0.f;
#pragma unroll
    for (int c = 0; c < PROBE_CHAINS; ++c)
#pragma unroll
        for (int r = 0; r < 16; ++r) s += acc[c][r];
    if (s == 123456.789f) sink[0] = s;   // keeps the loop alive; practically never true
}

// Streaming read: every lane takes 16 bytes per load, four loads in flight, consecutive lanes
// consecutive addresses, the grid striding over the buffer.
__global__ __launch_bounds__(256) void pc_probe_read_kernel(const u32x4 *__restrict__ src, int64_t n16,
                                                            float *sink) {
    u32x4 acc = {0u, 0u, 0u, 0u};
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    for (; i + 3 * stride < n16; i += 4 * stride) {
        const u32x4 p = __builtin_nontemporal_load(src + i);
        const u32x4 q = __builtin_nontemporal_load(src + i + stride);
        const u32x4 r = __builtin_nontemporal_load(src + i + 2 * stride);
        const u32x4 t = __builtin_nontemporal_load(src + i + 3 * stride);
        acc ^= p ^ q ^ r ^ t;
    }
    for (; i < n16; i += stride) acc ^= __builtin_nontemporal_load(src + i);
    if ((acc.x ^ acc.y ^ acc.z ^ acc.w) == 0x9e3779b9u && acc.x == 0x7f4a7c15u) sink[0] = 1.f;
}

struct EventPair {
    hipEvent_t t0 = nullptr, t1 = nullptr;
    hipError_t create() {
        hipError_t e = hipEventCreate(&t0);
        return e != hipSuccess ? e : hipEventCreate(&t1);
    }
    ~EventPair() {
        if (t0) (void)hipEventDestroy(t0);
        if (t1) (void)hipEventDestroy(t1);
    }
};

int32_t compute_units(int *cus) {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return PC_PROBE_ERR_HIP;
    if (hipDeviceGetAttribute(cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) return PC_PROBE_ERR_HIP;
    return *cus > 0 ? PC_PROBE_OK : PC_PROBE_ERR_HIP;
}

}  // namespace

extern "C" {

int32_t pc_probe_mfma_bf16(const void *operands, int64_t operand_bytes, int32_t iters, int32_t waves_per_simd,
                           int32_t reps, float *sink, double *tflops, void *stream) {
    if (!operands || !sink || !tflops) return PC_PROBE_ERR_INVALID_ARG;
    if (operand_bytes < (int64_t)PROBE_SETS * 64 * 32) return PC_PROBE_ERR_SHAPE;
    if (iters < 1 || iters > (1 << 16) || reps < 1 || reps > 100) return PC_PROBE_ERR_INVALID_ARG;   // at most ~2 s of GPU time
    if (waves_per_simd < 1 || waves_per_simd > 2) return PC_PROBE_ERR_INVALID_ARG;
    int cus = 0;
    if (int32_t rc = compute_units(&cus)) return rc;
    hipStream_t st = (hipStream_t)stream;
    EventPair ev;
    if (ev.create() != hipSuccess) return PC_PROBE_ERR_HIP;
    const int grid = cus * waves_per_simd;              // a workgroup is four waves, one per SIMD
    const uint4 *ops = (const uint4 *)operands;
    pc_probe_mfma_kernel<<<grid, 256, 0, st>>>(ops, iters, sink);          // untimed first launch
    if (hipEventRecord(ev.t0, st) != hipSuccess) return PC_PROBE_ERR_HIP;
    for (int r = 0; r < reps; ++r) pc_probe_mfma_kernel<<<grid, 256, 0, st>>>(ops, iters, sink);
    if (hipEventRecord(ev.t1, st) != hipSuccess) return PC_PROBE_ERR_HIP;
    if (hipEventSynchronize(ev.t1) != hipSuccess) return PC_PROBE_ERR_HIP;
    if (hipGetLastError() != hipSuccess) return PC_PROBE_ERR_HIP;
    float ms = 0.f;
    if (hipEventElapsedTime(&ms, ev.t0, ev.t1) != hipSuccess || ms <= 0.f) return PC_PROBE_ERR_HIP;
    const double flop = (double)grid * 4 * (double)iters * PROBE_CHAINS * PROBE_UNROLL * (2.0 * 32 * 32 * 16);
    *tflops = flop * reps / (ms * 1e-3) / 1e12;
    return PC_PROBE_OK;
}

int32_t pc_probe_hbm_read(const void *src, int64_t bytes, int32_t reps, float *sink, double *gb_per_s,
                          void *stream) {
    if (!src || !sink || !gb_per_s) return PC_PROBE_ERR_INVALID_ARG;
    if (bytes < 16 || (bytes & 15) || ((uintptr_t)src & 15)) return PC_PROBE_ERR_SHAPE;
    if (reps < 1 || reps > 100) return PC_PROBE_ERR_INVALID_ARG;
    int cus = 0;
    if (int32_t rc = compute_units(&cus)) return rc;
    hipStream_t st = (hipStream_t)stream;
    EventPair ev;
    if (ev.create() != hipSuccess) return PC_PROBE_ERR_HIP;
    const int grid = cus * 8;
    const u32x4 *p = (const u32x4 *)src;
    pc_probe_read_kernel<<<grid, 256, 0, st>>>(p, bytes / 16, sink);       // untimed first launch
    if (hipEventRecord(ev.t0, st) != hipSuccess) return PC_PROBE_ERR_HIP;
    for (int r = 0; r < reps; ++r) pc_probe_read_kernel<<<grid, 256, 0, st>>>(p, bytes / 16, sink);
    if (hipEventRecord(ev.t1, st) != hipSuccess) return PC_PROBE_ERR_HIP;
    if (hipEventSynchronize(ev.t1) != hipSuccess) return PC_PROBE_ERR_HIP;
    if (hipGetLastError() != hipSuccess) return PC_PROBE_ERR_HIP;
    float ms = 0.f;
    if (hipEventElapsedTime(&ms, ev.t0, ev.t1) != hipSuccess || ms <= 0.f) return PC_PROBE_ERR_HIP;
    *gb_per_s = (double)bytes * reps / (ms * 1e-3) / 1e9;
    return PC_PROBE_OK;
}

}  // extern "C"
