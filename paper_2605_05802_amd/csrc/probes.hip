// Measured ceilings of the chip this process runs on, for the roofline report: what a pure streaming
// read, a plain copy and a register-resident bf16 matrix-core loop achieve, next to the published peaks.
// Auxiliaries of the boundary (sr_probe_*); nothing on the rollout path calls them.
#include <functional>
#include <vector>

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

// The matrix-core loop with operand-sized loads beside it: every wavefront alternates sixteen register-resident
// 32x32x16 MFMAs with L wavefront-wide loads of 16 bytes per lane from a small buffer (a power of two of 16-byte
// vectors, so L2- or memory-side-cache resident), either into registers (PATH 1) or straight into LDS (PATH 2), and
// optionally twelve 16-byte LDS reads.  A 256 x 256 x 32 GEMM step with eight computing wavefronts is L = 4.
template <int PATH, int L, bool DS>
__global__ __launch_bounds__(512) void probe_mfma_loads_kernel(const u32x4 *__restrict__ src, size_t vec_mask, float *out,
                                                               int iters) {
    __shared__ u32x4 lds[8 * 8 * 64];     // 64 KiB: eight 1 KiB landing slots per wavefront
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    f32x16 acc[8];
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[i][v] = 0.f;
    bf16x8 a, b;
#pragma unroll
    for (int e = 0; e < 8; ++e) { a[e] = (__bf16)(0.001f * (lane + e)); b[e] = (__bf16)(0.002f * (lane - e)); }
    u32x4 sink = {0, 0, 0, 0};
    size_t pos = ((size_t)blockIdx.x * 8 + wave) * 4096 + lane;
    constexpr int NL = L > 0 ? L : 1;
    u32x4 r[2][NL];                        // the loads of one iteration are consumed two iterations later
#pragma unroll
    for (int p = 0; p < 2; ++p)
#pragma unroll
        for (int j = 0; j < NL; ++j) r[p][j] = sink;
    for (int it = 0; it < iters; ++it) {
        const int p = it & 1;
        if constexpr (PATH == 1) {
#pragma unroll
            for (int j = 0; j < L; ++j) { sink ^= r[p][j]; r[p][j] = src[(pos + j * 64) & vec_mask]; }
        } else if constexpr (PATH == 2) {
#pragma unroll
            for (int j = 0; j < L; ++j)
                __builtin_amdgcn_global_load_lds(
                    (const __attribute__((address_space(1))) void *)(src + ((pos + j * 64 - lane) & vec_mask) + lane),
                    (__attribute__((address_space(3))) void *)&lds[(wave * 8 + (j & 7)) * 64], 16, 0, 0);
        }
        if constexpr (DS) {
#pragma unroll
            for (int j = 0; j < 12; ++j) sink ^= lds[((wave * 8 + (j & 7)) * 64 + lane + it) & (8 * 8 * 64 - 1)];
        }
        pos += (size_t)L * 64;
#pragma unroll
        for (int q = 0; q < 2; ++q)
#pragma unroll
            for (int i = 0; i < 8; ++i) acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[i], 0, 0, 0);
    }
    __builtin_amdgcn_s_waitcnt(0x0F70);    // every load has landed before the wavefront (and its LDS) goes away
#pragma unroll
    for (int p = 0; p < 2; ++p)
#pragma unroll
        for (int j = 0; j < NL; ++j) sink ^= r[p][j];
    float t = 0.f;
#pragma unroll
    for (int i = 0; i < 8; ++i) t += acc[i][0];
    out[(size_t)blockIdx.x * 512 + threadIdx.x] = t + (float)((sink.x ^ sink.y ^ sink.z ^ sink.w) & 1u);
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

#define SR_PROBE_CASE(P, LL, D)                                                                                  \
    case P * 100 + LL * 2 + D:                                                                                   \
        probe_mfma_loads_kernel<P, LL, D != 0><<<dim3(wgs), dim3(512), 0, st>>>(src, mask, out, inner);          \
        break;

extern "C" int sr_probe_mfma_under_loads(const void *buf, size_t buf_bytes, void *scratch, size_t scratch_bytes, int path,
                                         int loads_per_16, int lds_reads, int iters, void *stream, double *host_TFLOPs,
                                         double *host_load_GBs) {
    const int wgs = 256;                           // one workgroup of eight wavefronts per compute unit
    if (!buf || !scratch || !host_TFLOPs || iters < 1 || path < 0 || path > 2 || scratch_bytes < (size_t)wgs * 512 * 4)
        return SR_E_ARG;
    if (buf_bytes < (1u << 16) || (buf_bytes & (buf_bytes - 1))) return SR_E_ARG;      // a power of two, >= 64 KiB
    if (path == 0 ? loads_per_16 != 0 : (loads_per_16 != 2 && loads_per_16 != 4 && loads_per_16 != 8)) return SR_E_ARG;
    if (lds_reads && path == 1) return SR_E_ARG;
    hipStream_t st = (hipStream_t)stream;
    const u32x4 *src = (const u32x4 *)buf;
    const size_t mask = buf_bytes / 16 - 1;
    float *out = (float *)scratch;
    const int inner = 4000;
    const int key = path * 100 + loads_per_16 * 2 + (lds_reads ? 1 : 0);
    double ms = 0;
    int bad = 0;
    auto launch = [&] {
        switch (key) {
            SR_PROBE_CASE(0, 0, 0) SR_PROBE_CASE(0, 0, 1)
            SR_PROBE_CASE(1, 2, 0) SR_PROBE_CASE(1, 4, 0) SR_PROBE_CASE(1, 8, 0)
            SR_PROBE_CASE(2, 2, 0) SR_PROBE_CASE(2, 4, 0) SR_PROBE_CASE(2, 8, 0)
            SR_PROBE_CASE(2, 2, 1) SR_PROBE_CASE(2, 4, 1) SR_PROBE_CASE(2, 8, 1)
            default: bad = 1;
        }
    };
    SR_TRY(time_launches(st, iters, &ms, launch));
    if (bad) return SR_E_ARG;
    const double flop = (double)wgs * 8 * inner * 16 * 2.0 * 32 * 32 * 16;
    *host_TFLOPs = flop / (ms * 1e-3) / 1e12;
    if (host_load_GBs) *host_load_GBs = (double)wgs * 8 * inner * loads_per_16 * 1024.0 / (ms * 1e-3) / 1e9;
    return SR_OK;
}

// The decode attention launch of one layer on synthetic pages, for studying its two phases apart: the shared-prompt
// phase (one unit per group, the members' query rows batched), the private phase (one unit per sequence), or both in
// one launch as the decode step does.  hot != 0 maps every page-table entry to the same few pages, so that all K/V
// loads hit in the caches and what is left is the kernel's own instruction and latency chain.
extern "C" int sr_probe_decode_attention(int n_groups, int G, int shared_tokens, int priv_tokens, int priv_splits,
                                         int phases, int hot, int iters, void *stream, double *host_us,
                                         double *host_kv_bytes) {
    const int n_q = 28, n_kv = 4, d = 128, page_tokens = 64, n_rep = n_q / n_kv, NL = 6;   // the 7B attention shape
    if (n_groups < 1 || G < 2 || G > 16 || shared_tokens < 0 || shared_tokens % page_tokens || priv_tokens < 1 ||
        priv_splits < 1 || priv_splits > 16 || phases < 1 || phases > 7 || !(phases & 3) || iters < 1 || !host_us)
        return SR_E_ARG;
    if ((phases & 1) && shared_tokens == 0) return SR_E_ARG;
    hipStream_t st = (hipStream_t)stream;
    const int M = n_groups * G;
    const int shared_pages = shared_tokens / page_tokens, priv_pages = ceil_div(priv_tokens, page_tokens);
    const int max_pages = shared_pages + priv_pages;
    const int n_pages = n_groups * shared_pages + M * priv_pages;
    const size_t layer_elems = (size_t)n_pages * n_kv * page_tokens * d;
    // NL layers' worth of pages are rotated through so that consecutive launches do not find their data in a cache
    uint16_t *kp = nullptr, *vp = nullptr, *q = nullptr;
    int32_t *dpt = nullptr;
    float *po = nullptr, *pml = nullptr;
    uint4 *merged = nullptr;
    const int mt_total = ceil_div(M, 16);
    std::vector<int32_t> pt((size_t)M * max_pages);
    for (int u = 0; u < M; ++u)
        for (int j = 0; j < max_pages; ++j) {
            int page = j < shared_pages ? (u / G) * shared_pages + j : n_groups * shared_pages + (j - shared_pages) * M + u;
            if (hot) page = j < shared_pages ? j % 4 : 4 + (j & 1);
            pt[(size_t)u * max_pages + j] = page;
        }
    AttnPhase x{}, y{};
    const int ctx = shared_tokens + priv_tokens;
    x.n_units = n_groups; x.q_per_unit = G; x.rt = 1;
    x.q_per_item = 16 / n_rep < G ? 16 / n_rep : G;
    x.items_per_unit = ceil_div(G, x.q_per_item);
    x.pt_row_stride = G; x.t_begin = 0; x.t_end = shared_tokens; x.causal_pos0 = ctx - 1;
    x.n_splits = shared_tokens ? ceil_div(shared_tokens, 256) : 1;
    if (x.n_splits > 16) x.n_splits = 16;
    x.split_tokens = shared_tokens ? round_up(ceil_div(shared_tokens, x.n_splits), 32) : 32;
    y.n_units = M; y.q_per_unit = 1; y.q_per_item = 1; y.items_per_unit = 1; y.rt = 1; y.pt_row_stride = 1;
    y.t_begin = shared_tokens; y.t_end = ctx; y.causal_pos0 = ctx - 1;
    y.n_splits = priv_splits; y.split_tokens = round_up(ceil_div(priv_tokens, priv_splits), 32);
    y.stream_loads = priv_tokens >= 512;
    const size_t items0 = (size_t)x.n_units * n_kv * x.items_per_unit * x.n_splits, items1 = (size_t)M * n_kv * y.n_splits;
    int rc = SR_OK;
    auto fail = [&](hipError_t e, const char *what) { note_hip_error(e, what); rc = SR_E_HIP; };
    hipError_t e;
    if ((e = hipMalloc(&kp, layer_elems * 2 * NL)) != hipSuccess) fail(e, "hipMalloc");
    if (rc == SR_OK && (e = hipMalloc(&vp, layer_elems * 2 * NL)) != hipSuccess) fail(e, "hipMalloc");
    if (rc == SR_OK && (e = hipMalloc(&q, (size_t)M * n_q * d * 2)) != hipSuccess) fail(e, "hipMalloc");
    if (rc == SR_OK && (e = hipMalloc(&dpt, pt.size() * 4)) != hipSuccess) fail(e, "hipMalloc");
    if (rc == SR_OK && (e = hipMalloc(&po, (items0 + items1) * 16 * d * 4)) != hipSuccess) fail(e, "hipMalloc");
    if (rc == SR_OK && (e = hipMalloc(&pml, (items0 + items1) * 16 * 2 * 4)) != hipSuccess) fail(e, "hipMalloc");
    if (rc == SR_OK && (phases & 4) && (e = hipMalloc(&merged, (size_t)mt_total * 16 * n_q * d * 2)) != hipSuccess)
        fail(e, "hipMalloc");
    if (rc == SR_OK) {
        (void)hipMemsetAsync(kp, 0x11, layer_elems * 2 * NL, st);      // small finite bf16 values
        (void)hipMemsetAsync(vp, 0x11, layer_elems * 2 * NL, st);
        (void)hipMemsetAsync(q, 0x11, (size_t)M * n_q * d * 2, st);
        if ((e = hipMemcpy(dpt, pt.data(), pt.size() * 4, hipMemcpyHostToDevice)) != hipSuccess) fail(e, "hipMemcpy");
    }
    if (rc == SR_OK) {
        x.part_o = po; x.part_ml = pml;
        y.part_o = po + items0 * 16 * d; y.part_ml = pml + items0 * 16 * 2;
        AttnArgs a{};
        a.q = q; a.page_table = dpt; a.pt_stride = max_pages; a.page_tokens = page_tokens;
        a.n_q = n_q; a.n_kv = n_kv; a.d = d; a.scale = 0.0883883f;
        AttnPhase ph[2] = {x, y};
        const AttnPhase *first = (phases & 3) == 2 ? ph + 1 : ph;
        const int n_ph = (phases & 3) == 3 ? 2 : 1;
        int layer = 0;
        double ms = 0;
        int lrc = SR_OK;
        rc = time_launches(st, iters, &ms, [&] {
            a.kpool = kp + (size_t)(layer % NL) * layer_elems;
            a.vpool = vp + (size_t)(layer % NL) * layer_elems;
            ++layer;
            int r = launch_attention(a, first, n_ph, st);
            if (r == SR_OK && (phases & 4)) r = launch_attn_merge(a, first, n_ph, M, merged, mt_total, nullptr, st);
            if (r != SR_OK) lrc = r;
        });
        if (rc == SR_OK) rc = lrc;
        *host_us = ms * 1e3;
        if (host_kv_bytes)
            *host_kv_bytes = 2.0 * n_kv * d * 2 * (((phases & 1) ? (double)n_groups * shared_tokens : 0.0) +
                                                    ((phases & 2) ? (double)M * priv_tokens : 0.0));
    }
    (void)hipStreamSynchronize(st);
    if (kp) (void)hipFree(kp);
    if (vp) (void)hipFree(vp);
    if (q) (void)hipFree(q);
    if (dpt) (void)hipFree(dpt);
    if (po) (void)hipFree(po);
    if (pml) (void)hipFree(pml);
    if (merged) (void)hipFree(merged);
    return rc;
}
