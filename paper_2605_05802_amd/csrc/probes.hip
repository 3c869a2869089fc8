// Measured ceilings of the chip this process runs on, for the roofline report: what a pure streaming
// read, a plain copy and a register-resident bf16 matrix-core loop achieve, next to the published peaks.
// Auxiliaries of the boundary (sr_probe_*); nothing on the rollout path calls them.
#include <functional>

#include "sr_internal.h"

namespace sr {
namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// Every wavefront streams its own contiguous run with 16-byte loads, eight in flight per lane, with the
// non-temporal hint the weight-streaming kernels use (NT) or with default loads.
template <bool NT>
__global__ __launch_bounds__(256) void probe_read_kernel(const u32x4 *__restrict__ src, size_t vec_per_wave, u32x4 *sink) {
    const size_t wave = (size_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    const u32x4 *p = src + wave * vec_per_wave + (threadIdx.x & 63);
    u32x4 acc = {0, 0, 0, 0};
    for (size_t i = 0; i < vec_per_wave; i += 8 * 64) {
        u32x4 v[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) v[j] = NT ? __builtin_nontemporal_load(p + i + j * 64) : p[i + j * 64];
#pragma unroll
        for (int j = 0; j < 8; ++j) acc ^= v[j];
    }
    if (acc.x == 0x9E3779B9u && acc.y == 0x7F4A7C15u) *sink = acc;      // never true for the zero-filled buffer
}

__global__ __launch_bounds__(256) void probe_copy_kernel(const u32x4 *__restrict__ src, u32x4 *__restrict__ dst,
                                                         size_t vec_per_wave) {
    const size_t wave = (size_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    const size_t base = wave * vec_per_wave + (threadIdx.x & 63);
    for (size_t i = 0; i < vec_per_wave; i += 8 * 64) {
        u32x4 v[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) v[j] = src[base + i + j * 64];
#pragma unroll
        for (int j = 0; j < 8; ++j) dst[base + i + j * 64] = v[j];
    }
}

// Four independent 32x32x16 accumulator chains per wavefront, operands in registers: nothing but the matrix pipe.
__global__ __launch_bounds__(256) void probe_mfma_kernel(float *out, int iters) {
    bf16x8 a, b;
#pragma unroll
    for (int i = 0; i < 8; ++i) { a[i] = (__bf16)(0.001f * (threadIdx.x & 63) + i); b[i] = (__bf16)(0.5f * i); }
    f32x16 acc[4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 16; ++j) acc[i][j] = 0.f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 4; ++i) acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[i], 0, 0, 0);
    }
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < 4; ++i) s += acc[i][0];
    out[(size_t)blockIdx.x * 256 + threadIdx.x] = s;
}

int time_launches(hipStream_t st, int iters, double *ms_per_launch, const std::function<void()> &launch) {
    hipEvent_t e0, e1;
    SR_HIP(hipEventCreate(&e0));
    SR_HIP(hipEventCreate(&e1));
    launch();                                      // warm-up
    SR_HIP(hipEventRecord(e0, st));
    for (int i = 0; i < iters; ++i) launch();
    SR_HIP(hipEventRecord(e1, st));
    SR_HIP(hipEventSynchronize(e1));
    float ms = 0.f;
    SR_HIP(hipEventElapsedTime(&ms, e0, e1));
    SR_HIP(hipGetLastError());
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    *ms_per_launch = ms / iters;
    return SR_OK;
}

}  // namespace
}  // namespace sr

using namespace sr;

extern "C" int sr_probe_hbm(const void *src, void *dst, size_t bytes, int mode, int iters, void *stream,
                            double *host_GBs) {
    if (!src || !host_GBs || iters < 1 || mode < 0 || mode > 2 || (mode == 2 && !dst)) return SR_E_ARG;
    // whole runs of 8 x 64 16-byte vectors per wavefront, 4096 wavefronts
    const size_t n_waves = 4096, unit = 8 * 64 * 16;
    const size_t per_wave = bytes / n_waves / unit * unit;
    if (per_wave == 0) return SR_E_ARG;
    hipStream_t st = (hipStream_t)stream;
    const size_t vec = per_wave / 16;
    double ms = 0;
    void *sink = nullptr;
    if (mode != 2) {
        if (!dst) return SR_E_ARG;                 // 16 bytes the read kernels may (never) write
        sink = dst;
    }
    SR_TRY(time_launches(st, iters, &ms, [&] {
        if (mode == 0) probe_read_kernel<true><<<dim3(n_waves / 4), dim3(256), 0, st>>>((const u32x4 *)src, vec, (u32x4 *)sink);
        else if (mode == 1) probe_read_kernel<false><<<dim3(n_waves / 4), dim3(256), 0, st>>>((const u32x4 *)src, vec, (u32x4 *)sink);
        else probe_copy_kernel<<<dim3(n_waves / 4), dim3(256), 0, st>>>((const u32x4 *)src, (u32x4 *)dst, vec);
    }));
    const double moved = (double)per_wave * n_waves * (mode == 2 ? 2.0 : 1.0);
    *host_GBs = moved / (ms * 1e-3) / 1e9;
    return SR_OK;
}

extern "C" int sr_probe_mfma_bf16(void *scratch, size_t scratch_bytes, int iters, void *stream, double *host_TFLOPs) {
    const int wgs = 1024;                          // four workgroups of four wavefronts per compute unit
    if (!scratch || !host_TFLOPs || iters < 1 || scratch_bytes < (size_t)wgs * 256 * 4) return SR_E_ARG;
    hipStream_t st = (hipStream_t)stream;
    const int inner = 20000;
    double ms = 0;
    SR_TRY(time_launches(st, iters, &ms,
                         [&] { probe_mfma_kernel<<<dim3(wgs), dim3(256), 0, st>>>((float *)scratch, inner); }));
    const double flop = (double)wgs * 4 * inner * 4 * 2.0 * 32 * 32 * 16;
    *host_TFLOPs = flop / (ms * 1e-3) / 1e12;
    return SR_OK;
}
