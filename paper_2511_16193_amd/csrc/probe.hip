// Micro-benchmarks that give the rooflines of this very GPU, as opposed to the data sheet's: a register-only bf16
// MFMA loop, a plain device copy and read, and a loop that shows whether matrix and vector instructions overlap.
// The benchmark reports every kernel's rate against the first three.
// Declared in include/specverify_ops.h.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/specverify.h"
#include "../../include/specverify_ops.h"
#include "common.h"

namespace sv {

typedef __attribute__((ext_vector_type(16))) float floatx16;

// One wave per SIMD, eight independent 32x32 accumulators, operands held in registers for the whole loop: nothing
// but the matrix unit is busy.  The operands come from memory once (random values make the multipliers toggle, and
// the chip's clock then settles well below what all-zero operands allow).
__global__ __launch_bounds__(256, 1) void probe_mfma_kernel(const sv::u32x4* __restrict__ operands, float* __restrict__ sink, int iters) {
    const int t = blockIdx.x * 256 + threadIdx.x;
    sv::bf16x8 a[4], b[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        a[i] = __builtin_bit_cast(sv::bf16x8, operands[(int64_t)t * 8 + i]);
        b[i] = __builtin_bit_cast(sv::bf16x8, operands[(int64_t)t * 8 + 4 + i]);
    }
    floatx16 acc[8];
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[i][e] = 0.f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 8; ++i) acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i & 3], b[i >> 1], acc[i], 0, 0, 0);
    }
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int e = 0; e < 16; ++e) s += acc[i][e];
    sink[t] = s;
}

// Do the matrix unit and the vector ALU of a SIMD work at the same time?  MODE 0: `iters` rounds of eight independent
// v_mfma_f32_16x16x32_bf16; MODE 1: `iters` rounds of 8 * NV independent v_fma_f32; MODE 2: both, NV FMAs after each
// MFMA.  Operands in registers; 64 * WAVES threads per work-group give one or two waves per SIMD.
template <int MODE, int NV>
__global__ __launch_bounds__(512) void probe_mix_kernel(float* __restrict__ sink, int iters, float seed) {
    floatx4 acc[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) acc[i] = floatx4{0.f, 0.f, 0.f, 0.f};
    sv::bf16x8 a, b;
#pragma unroll
    for (int i = 0; i < 8; ++i) { a[i] = (__bf16)(threadIdx.x * 0.001f + i); b[i] = (__bf16)(seed + i); }
    float v[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) v[i] = seed + i + threadIdx.x;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int m = 0; m < 8; ++m) {
            if (MODE != 1) acc[m] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, acc[m], 0, 0, 0);
            if (MODE != 0) {
#pragma unroll
                for (int j = 0; j < NV; ++j) v[(m + j) & 7] = __builtin_fmaf(v[(m + j) & 7], 1.0001f, 0.5f);
            }
            if (MODE == 2) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                __builtin_amdgcn_sched_group_barrier(0x002, NV, 0);
            }
        }
    }
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < 8; ++i) s += acc[i][0] + acc[i][1] + acc[i][2] + acc[i][3] + v[i];
    sink[blockIdx.x * blockDim.x + threadIdx.x] = s;
}

// Plain copy, 16 bytes per lane, grid-stride: what a stream of reads and writes reaches on this part.
__global__ __launch_bounds__(256) void probe_copy_kernel(const sv::u32x4* __restrict__ src, sv::u32x4* __restrict__ dst, size_t n16) {
    const size_t stride = (size_t)gridDim.x * 256;
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += stride) dst[i] = src[i];
}

// Plain read, 16 bytes per lane, eight loads in flight per lane, grid-stride: what a read-only stream reaches (the
// verify attention is one).  The xor of what was read goes to `sink` only if it matches a value it never has, so
// that the loads are not optimised away and nothing is written.
__global__ __launch_bounds__(256) void probe_read_kernel(const sv::u32x4* __restrict__ src, unsigned* __restrict__ sink, size_t n16) {
    const size_t stride = (size_t)gridDim.x * 256;
    size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    sv::u32x4 acc = {0, 0, 0, 0};
    for (; i + 7 * stride < n16; i += 8 * stride) {
        sv::u32x4 v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) v[u] = __builtin_nontemporal_load(src + i + u * stride);
#pragma unroll
        for (int u = 0; u < 8; ++u) acc ^= v[u];
    }
    for (; i < n16; i += stride) acc ^= src[i];
    if ((acc.x ^ acc.y ^ acc.z ^ acc.w) == 0x9E3779B9u) sink[0] = 1;
}

struct EventPair {
    hipEvent_t a = nullptr, b = nullptr;
    bool ok() { return hipEventCreate(&a) == hipSuccess && hipEventCreate(&b) == hipSuccess; }
    ~EventPair() { if (a) (void)hipEventDestroy(a); if (b) (void)hipEventDestroy(b); }
};

}  // namespace sv

using namespace sv;

extern "C" int sv_probe_mfma_bf16(const void* operands, size_t operand_bytes, float* sink, int iters, void* stream,
                                  double* tflops) {
    constexpr int kBlocks = 256;                          // one work-group per CU, one wave per SIMD
    if (!operands || !sink || !tflops || iters <= 0 || operand_bytes < (size_t)kBlocks * 256 * 8 * 16) return SV_EINVAL;
    hipStream_t st = (hipStream_t)stream;
    EventPair ev;
    if (!ev.ok()) return SV_EHIP;
    hipLaunchKernelGGL(probe_mfma_kernel, dim3(kBlocks), dim3(256), 0, st, (const sv::u32x4*)operands, sink, iters / 8 + 1);   // warm-up
    if (hipEventRecord(ev.a, st) != hipSuccess) return SV_EHIP;
    hipLaunchKernelGGL(probe_mfma_kernel, dim3(kBlocks), dim3(256), 0, st, (const sv::u32x4*)operands, sink, iters);
    if (hipEventRecord(ev.b, st) != hipSuccess || hipEventSynchronize(ev.b) != hipSuccess || hipGetLastError() != hipSuccess) return SV_EHIP;
    float ms = 0.f;
    if (hipEventElapsedTime(&ms, ev.a, ev.b) != hipSuccess || !(ms > 0.f)) return SV_EHIP;
    *tflops = (double)kBlocks * 4 * iters * 8 * (2.0 * 32 * 32 * 16) / (ms * 1e-3) / 1e12;
    return SV_OK;
}

// Runs `launch(grid)` reps times for each of a few grid sizes (after one warm-up launch each) and returns the best
// time of one repetition in milliseconds (< 0 on error): the probes report what the part can do, not what one
// particular launch shape does.
template <typename F>
static double best_of_grids(hipStream_t st, int reps, F launch) {
    EventPair ev;
    if (!ev.ok()) return -1.0;
    double best = -1.0;
    for (int blocks : {1024, 2048, 4096, 8192, 16384}) {
        launch(blocks);
        if (hipEventRecord(ev.a, st) != hipSuccess) return -1.0;
        for (int r = 0; r < reps; ++r) launch(blocks);
        if (hipEventRecord(ev.b, st) != hipSuccess || hipEventSynchronize(ev.b) != hipSuccess || hipGetLastError() != hipSuccess) return -1.0;
        float ms = 0.f;
        if (hipEventElapsedTime(&ms, ev.a, ev.b) != hipSuccess || !(ms > 0.f)) return -1.0;
        if (best < 0.0 || ms / reps < best) best = ms / reps;
    }
    return best;
}

extern "C" int sv_probe_hbm_copy(const void* src, void* dst, size_t bytes, int reps, void* stream, double* gbs_each_way) {
    if (!src || !dst || !gbs_each_way || bytes < (1u << 20) || bytes % 16 != 0 || reps <= 0 || ((uintptr_t)src & 15) || ((uintptr_t)dst & 15))
        return SV_EINVAL;
    hipStream_t st = (hipStream_t)stream;
    const size_t n16 = bytes / 16;
    const double ms = best_of_grids(st, reps, [&](int blocks) {
        hipLaunchKernelGGL(probe_copy_kernel, dim3(blocks), dim3(256), 0, st, (const sv::u32x4*)src, (sv::u32x4*)dst, n16);
    });
    if (ms < 0.0) return SV_EHIP;
    *gbs_each_way = (double)bytes / (ms * 1e-3) / 1e9;
    return SV_OK;
}

extern "C" int sv_probe_hbm_read(const void* src, size_t bytes, int reps, void* sink, void* stream, double* gbs) {
    if (!src || !sink || !gbs || bytes < (1u << 20) || bytes % 16 != 0 || reps <= 0 || ((uintptr_t)src & 15)) return SV_EINVAL;
    hipStream_t st = (hipStream_t)stream;
    const size_t n16 = bytes / 16;
    const double ms = best_of_grids(st, reps, [&](int blocks) {
        hipLaunchKernelGGL(probe_read_kernel, dim3(blocks), dim3(256), 0, st, (const sv::u32x4*)src, (unsigned*)sink, n16);
    });
    if (ms < 0.0) return SV_EHIP;
    *gbs = (double)bytes / (ms * 1e-3) / 1e9;
    return SV_OK;
}

// Times, in milliseconds, of the three modes of probe_mix_kernel (MFMAs alone, FMAs alone, both woven) on 256
// work-groups of `waves_per_simd` * 4 waves; out_ms[3].
extern "C" int sv_probe_mfma_valu(float* sink, int iters, int valu_per_mfma, int waves_per_simd, void* stream, double* out_ms) {
    if (!sink || !out_ms || iters <= 0 || (waves_per_simd != 1 && waves_per_simd != 2) ||
        (valu_per_mfma != 2 && valu_per_mfma != 4 && valu_per_mfma != 6))
        return SV_EINVAL;
    hipStream_t st = (hipStream_t)stream;
    const dim3 grid(256), block(256 * waves_per_simd);
    auto timed = [&](auto kern, double& ms_out) -> int {
        EventPair ev;
        if (!ev.ok()) return SV_EHIP;
        hipLaunchKernelGGL(kern, grid, block, 0, st, sink, iters / 8 + 1, 1.0f);       // warm-up
        if (hipEventRecord(ev.a, st) != hipSuccess) return SV_EHIP;
        hipLaunchKernelGGL(kern, grid, block, 0, st, sink, iters, 1.0f);
        if (hipEventRecord(ev.b, st) != hipSuccess || hipEventSynchronize(ev.b) != hipSuccess || hipGetLastError() != hipSuccess) return SV_EHIP;
        float ms = 0.f;
        if (hipEventElapsedTime(&ms, ev.a, ev.b) != hipSuccess) return SV_EHIP;
        ms_out = ms;
        return SV_OK;
    };
    int rc = SV_OK;
    switch (valu_per_mfma) {
        case 2:
            if ((rc = timed(probe_mix_kernel<0, 2>, out_ms[0])) || (rc = timed(probe_mix_kernel<1, 2>, out_ms[1])) || (rc = timed(probe_mix_kernel<2, 2>, out_ms[2]))) return rc;
            break;
        case 4:
            if ((rc = timed(probe_mix_kernel<0, 4>, out_ms[0])) || (rc = timed(probe_mix_kernel<1, 4>, out_ms[1])) || (rc = timed(probe_mix_kernel<2, 4>, out_ms[2]))) return rc;
            break;
        default:
            if ((rc = timed(probe_mix_kernel<0, 6>, out_ms[0])) || (rc = timed(probe_mix_kernel<1, 6>, out_ms[1])) || (rc = timed(probe_mix_kernel<2, 6>, out_ms[2]))) return rc;
            break;
    }
    return SV_OK;
}
