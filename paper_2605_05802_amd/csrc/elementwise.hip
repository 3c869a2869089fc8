// Row-wise kernels between the GEMMs: residual update + RMSNorm, QKV epilogue (bias, RoPE,
// KV page write), greedy argmax, and small utilities.  All reductions run in a fixed order
// that does not depend on the row index or on the batch size, so a sequence's numbers do not
// change when other rows enter or leave the batch.
#include "sr_internal.h"

namespace sr {
namespace {

// deterministic block-wide sums of ROWS values over 512 threads (the same order of additions for every row)
template <int ROWS>
__device__ __forceinline__ void block_sums_512(float (&v)[ROWS], float (*s_red)[8]) {
#pragma unroll
    for (int r = 0; r < ROWS; ++r)
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) v[r] += __shfl_xor(v[r], off, 64);
    const int wave = threadIdx.x >> 6;
    if ((threadIdx.x & 63) == 0) {
#pragma unroll
        for (int r = 0; r < ROWS; ++r) s_red[r][wave] = v[r];
    }
    __syncthreads();
#pragma unroll
    for (int r = 0; r < ROWS; ++r)
        v[r] = ((s_red[r][0] + s_red[r][1]) + (s_red[r][2] + s_red[r][3])) + ((s_red[r][4] + s_red[r][5]) + (s_red[r][6] + s_red[r][7]));
}

// x = resid (+ partials) or embedding row; resid <- x (if write_resid); out <- bf16(x * rsqrt(mean(x^2)+eps) * gain)
// H <= 8192: each thread keeps its (at most 2 x 8) values per row in registers between the two passes.
// A workgroup takes ROWS consecutive output rows and requests all of their data before the first reduction:
// one row at decode time (few rows, every compute unit should get one), four for prefill-sized batches, where
// a row's three dependent memory round trips would otherwise leave the memory system mostly idle.  The
// arithmetic of a row does not depend on ROWS.
template <bool F32OUT, int ROWS>
__global__ __launch_bounds__(512) void resid_norm_kernel(NormArgs a) {
    __shared__ float s_red[ROWS][8];
    const int nvec = a.H >> 3;                       // groups of 8 consecutive features
    float xv[ROWS][2][8];
    float ss[ROWS];
    // the gains do not depend on the reduction: fetch them first, so that the second pass starts from registers
    uint4 graw[2];
#pragma unroll
    for (int it = 0; it < 2; ++it) {
        const int v = threadIdx.x + it * 512;
        graw[it] = v < nvec ? *(const uint4 *)(a.gain + v * 8) : make_uint4(0, 0, 0, 0);
    }

#pragma unroll
    for (int r = 0; r < ROWS; ++r) {
        const int m = blockIdx.x * ROWS + r;
        ss[r] = 0.f;
        if (m >= a.rows_out) continue;               // uniform across the workgroup
        const size_t row = (size_t)(m / a.src_dup) * a.src_stride + a.src_off;
        float *x = a.resid + row * a.H;
        const uint16_t *e = nullptr;
        if (a.embed) {
            const int tok = a.tokens[(size_t)(m / a.tok_chunk) * a.tok_stride + a.tok_off + m % a.tok_chunk];
            e = a.embed + (size_t)tok * a.H;
        }
#pragma unroll
        for (int it = 0; it < 2; ++it) {
            const int v = threadIdx.x + it * 512;
            if (v < nvec) {
                float *f = xv[r][it];
                if (e) {
                    const uint4 raw = *(const uint4 *)(e + v * 8);
                    const uint32_t w[4] = {raw.x, raw.y, raw.z, raw.w};
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        f[2 * i] = __uint_as_float(w[i] << 16);
                        f[2 * i + 1] = __uint_as_float(w[i] & 0xFFFF0000u);
                    }
                } else {
                    f32x4 lo = *(const f32x4 *)(x + v * 8), hi = *(const f32x4 *)(x + v * 8 + 4);
                    const float *p0 = a.partials + row * a.H + v * 8;
                    int s = 0;
                    for (; s + 4 <= a.n_partials; s += 4) {          // four independent loads in flight,
                        f32x4 pl[4], ph[4];                          // added in split order
#pragma unroll
                        for (int u = 0; u < 4; ++u) {
                            const float *p = p0 + (size_t)(s + u) * a.partial_stride;
                            pl[u] = *(const f32x4 *)p;
                            ph[u] = *(const f32x4 *)(p + 4);
                        }
#pragma unroll
                        for (int u = 0; u < 4; ++u) { lo += pl[u]; hi += ph[u]; }
                    }
                    for (; s < a.n_partials; ++s) {
                        const float *p = p0 + (size_t)s * a.partial_stride;
                        lo += *(const f32x4 *)p;
                        hi += *(const f32x4 *)(p + 4);
                    }
#pragma unroll
                    for (int i = 0; i < 4; ++i) { f[i] = lo[i]; f[4 + i] = hi[i]; }
                }
#pragma unroll
                for (int i = 0; i < 8; ++i) ss[r] += f[i] * f[i];
                if (a.write_resid) {
                    *(f32x4 *)(x + v * 8) = f32x4{f[0], f[1], f[2], f[3]};
                    *(f32x4 *)(x + v * 8 + 4) = f32x4{f[4], f[5], f[6], f[7]};
                }
            }
        }
    }
    block_sums_512<ROWS>(ss, s_red);

#pragma unroll
    for (int r = 0; r < ROWS; ++r) {
        const int m = blockIdx.x * ROWS + r;
        if (m >= a.rows_out) continue;
        const float inv = 1.0f / sqrtf(ss[r] / (float)a.H + a.eps);
#pragma unroll
        for (int it = 0; it < 2; ++it) {
            const int v = threadIdx.x + it * 512;
            if (v < nvec) {
                const float *f = xv[r][it];
                const uint32_t gw[4] = {graw[it].x, graw[it].y, graw[it].z, graw[it].w};
                float y[8];
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    y[2 * i] = f[2 * i] * inv * __uint_as_float(gw[i] << 16);
                    y[2 * i + 1] = f[2 * i + 1] * inv * __uint_as_float(gw[i] & 0xFFFF0000u);
                }
                if constexpr (F32OUT) {
                    float *dst = a.out32 + (size_t)m * a.H + v * 8;
                    *(f32x4 *)dst = f32x4{y[0], y[1], y[2], y[3]};
                    *(f32x4 *)(dst + 4) = f32x4{y[4], y[5], y[6], y[7]};
                } else {
                    uint4 o = make_uint4(pack_bf16x2(y[0], y[1]), pack_bf16x2(y[2], y[3]), pack_bf16x2(y[4], y[5]),
                                         pack_bf16x2(y[6], y[7]));
                    *(uint4 *)((uint16_t *)a.out + frag_offset(m, v * 8, a.mt_total)) = o;
                }
            }
        }
    }
}

// One block per (row, group of heads): 64 threads at decode time, up to 640 (all heads of a row) for prefill-sized
// batches, where tens of thousands of one-wavefront blocks would cost more than they move.  A thread owns four
// consecutive dims i .. i+3 of the low half of a head and their rotation partners i + d/2 .. (16-byte loads of the
// fp32 partials); d/8 threads make a head.
__global__ __launch_bounds__(640) void qkv_post_kernel(QkvPostArgs a) {
    const int half = a.d >> 1, tph = half >> 2;               // threads per head
    const int m = blockIdx.x, head = blockIdx.y * (blockDim.x / tph) + threadIdx.x / tph, i = (threadIdx.x % tph) * 4;
    if (head >= a.n_q + 2 * a.n_kv) return;
    const int unit = m / a.chunk, ci = m - unit * a.chunk;
    const int pos = a.pos0 + ci;
    const int q_cols = a.n_q * a.d, kv_cols = a.n_kv * a.d;
    int col0;
    const uint16_t *bias;
    int kind, h;                                          // 0 q, 1 k, 2 v
    if (head < a.n_q) { kind = 0; h = head; col0 = h * a.d; bias = a.bq ? a.bq + h * a.d : nullptr; }
    else if (head < a.n_q + a.n_kv) { kind = 1; h = head - a.n_q; col0 = q_cols + h * a.d; bias = a.bk ? a.bk + h * a.d : nullptr; }
    else { kind = 2; h = head - a.n_q - a.n_kv; col0 = q_cols + kv_cols + h * a.d; bias = a.bv ? a.bv + h * a.d : nullptr; }

    f32x4 lo = {0.f, 0.f, 0.f, 0.f}, hi = {0.f, 0.f, 0.f, 0.f};
    {
        const float *p0 = a.partials + (size_t)m * a.ld + col0 + i;
        int s = 0;
        for (; s + 4 <= a.n_partials; s += 4) {                  // independent loads, adds in split order
            f32x4 pl[4], ph[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const float *p = p0 + (size_t)(s + u) * a.partial_stride;
                pl[u] = *(const f32x4 *)p;
                ph[u] = *(const f32x4 *)(p + half);
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) { lo += pl[u]; hi += ph[u]; }
        }
        for (; s < a.n_partials; ++s) {
            const float *p = p0 + (size_t)s * a.partial_stride;
            lo += *(const f32x4 *)p;
            hi += *(const f32x4 *)(p + half);
        }
    }
    if (bias) {
#pragma unroll
        for (int e = 0; e < 4; ++e) { lo[e] += bf16_to_f32(bias[i + e]); hi[e] += bf16_to_f32(bias[i + half + e]); }
    }
    if (kind != 2) {
        const f32x4 c = *(const f32x4 *)(a.rope_cos + (size_t)pos * half + i);
        const f32x4 sn = *(const f32x4 *)(a.rope_sin + (size_t)pos * half + i);
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const float rlo = lo[e] * c[e] - hi[e] * sn[e], rhi = hi[e] * c[e] + lo[e] * sn[e];
            lo[e] = rlo; hi[e] = rhi;
        }
    }
    const uint2 plo = make_uint2(pack_bf16x2(lo[0], lo[1]), pack_bf16x2(lo[2], lo[3]));
    const uint2 phi = make_uint2(pack_bf16x2(hi[0], hi[1]), pack_bf16x2(hi[2], hi[3]));
    if (kind == 0) {
        uint16_t *q = a.q_out + ((size_t)m * a.n_q + h) * a.d;
        *(uint2 *)(q + i) = plo;
        *(uint2 *)(q + i + half) = phi;
        return;
    }
    const int page = a.page_table[(size_t)unit * a.pt_row_stride * a.pt_stride + pos / a.page_tokens];
    const int tok = pos % a.page_tokens, blk = tok >> 5, t = tok & 31;
    const size_t base = ((((size_t)page * a.n_kv + h) * (a.page_tokens >> 5)) + blk) * (size_t)(32 * a.d);
    if (kind == 1) {
        // K block [d/32][32 tok][32]: four consecutive dims stay inside one 32-dim group
        uint16_t *k = a.kpool + base;
        *(uint2 *)(k + (((i >> 5) * 32 + t) << 5) + (i & 31)) = plo;
        const int i2 = i + half;
        *(uint2 *)(k + (((i2 >> 5) * 32 + t) << 5) + (i2 & 31)) = phi;
    } else {
        uint16_t *v = a.vpool + base;
        const int slot = 8 * ((t & 15) >> 2) + 4 * (t >> 4) + (t & 3);
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            v[(i + e) * 32 + slot] = f32_to_bf16(lo[e]);
            v[(i + half + e) * 32 + slot] = f32_to_bf16(hi[e]);
        }
    }
}

struct MaxIdx {
    float v;
    int i;
};
__device__ __forceinline__ MaxIdx better(MaxIdx a, MaxIdx b) {
    return (b.v > a.v || (b.v == a.v && b.i < a.i)) ? b : a;
}

__device__ __forceinline__ uint64_t smx_finalize(uint64_t z) {
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ULL;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBULL;
    return z ^ (z >> 31);
}

// One 1024-thread block per row: strided scan, wavefront shuffle reduction, then 16 wave results.
// With inv_temperature > 0 every logit is scaled and perturbed by a standard Gumbel variate drawn from a
// counter-based SplitMix64 stream keyed (seed, original sequence id, position), counter = vocabulary
// index: the argmax of the perturbed scores is a draw from softmax(logits / T).
__global__ __launch_bounds__(1024) void argmax_kernel(const float *__restrict__ logits, int vocab,
                                                      const int32_t *__restrict__ forced, int32_t *greedy_out,
                                                      int32_t *chosen, int32_t *actions, int max_turns,
                                                      int turn_idx, int action_mod, float inv_temperature,
                                                      uint64_t seed, const int32_t *__restrict__ orig_seq, int pos) {
    __shared__ MaxIdx s_best[16];
    const int r = blockIdx.x;
    const float *row = logits + (size_t)r * vocab;
    MaxIdx best{-INFINITY, 0x7FFFFFFF};
    const int nvec = vocab >> 2;
    if (inv_temperature > 0.f) {
        const uint64_t golden = 0x9E3779B97F4A7C15ULL;
        const uint64_t stream = ((uint64_t)(uint32_t)orig_seq[r] << 32) | (uint32_t)pos;
        const uint64_t key = smx_finalize(smx_finalize(seed + golden) ^ (stream * 0xD1342543DE82EF95ULL + 1ULL));
        for (int v = threadIdx.x; v < vocab; v += 1024) {
            const uint64_t rnd = smx_finalize(key + ((uint64_t)v + 1ULL) * golden);
            const float u = ((float)(uint32_t)(rnd >> 41) + 0.5f) * (1.0f / 8388608.0f);
            best = better(best, MaxIdx{row[v] * inv_temperature - logf(-logf(u)), v});
        }
    } else {
        for (int v = threadIdx.x; v < nvec; v += 1024) {
            const f32x4 x = *(const f32x4 *)(row + v * 4);
#pragma unroll
            for (int e = 0; e < 4; ++e) best = better(best, MaxIdx{x[e], v * 4 + e});
        }
        for (int v = nvec * 4 + threadIdx.x; v < vocab; v += 1024) best = better(best, MaxIdx{row[v], v});
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
        MaxIdx o{__shfl_xor(best.v, off, 64), __shfl_xor(best.i, off, 64)};
        best = better(best, o);
    }
    if ((threadIdx.x & 63) == 0) s_best[threadIdx.x >> 6] = best;
    __syncthreads();
    if (threadIdx.x == 0) {
        for (int w = 1; w < 16; ++w) best = better(best, s_best[w]);
        const int greedy = best.i;
        if (greedy_out) greedy_out[r] = greedy;
        const int tok = forced ? forced[r] : greedy;
        chosen[r] = tok;
        if (actions) actions[(size_t)r * max_turns + turn_idx] = tok % action_mod;
    }
}

__global__ void fill_i32_kernel(int32_t *dst, size_t n, int32_t value) {
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) dst[i] = value;
}

template <typename T>
__global__ void gather_rows_kernel(T *dst, const T *src, const int32_t *src_rows, size_t row_vec) {
    const int r = blockIdx.y;
    const size_t s = (size_t)src_rows[r];
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < row_vec; i += (size_t)gridDim.x * blockDim.x)
        dst[(size_t)r * row_vec + i] = src[s * row_vec + i];
}

__global__ void copy_page_kernel(uint4 *kpool, uint4 *vpool, size_t layer_vec, size_t page_vec, int src_page,
                                 int dst_page) {
    const int layer = blockIdx.y;
    uint4 *k = kpool + layer * layer_vec, *v = vpool + layer * layer_vec;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < page_vec; i += (size_t)gridDim.x * blockDim.x) {
        k[(size_t)dst_page * page_vec + i] = k[(size_t)src_page * page_vec + i];
        v[(size_t)dst_page * page_vec + i] = v[(size_t)src_page * page_vec + i];
    }
}

}  // namespace

int launch_resid_norm(const NormArgs &a, hipStream_t stream) {
    if (a.rows_out <= 0) return SR_OK;
    if (a.H % 8 || a.H > 8192) return SR_E_ARG;
    if (a.out32) resid_norm_kernel<true, 1><<<dim3(a.rows_out), dim3(512), 0, stream>>>(a);
    else if (a.rows_out >= 2048) resid_norm_kernel<false, 4><<<dim3(ceil_div(a.rows_out, 4)), dim3(512), 0, stream>>>(a);
    else resid_norm_kernel<false, 1><<<dim3(a.rows_out), dim3(512), 0, stream>>>(a);
    SR_HIP(hipGetLastError());
    return SR_OK;
}

int launch_qkv_post(const QkvPostArgs &a, hipStream_t stream) {
    if (a.rows <= 0) return SR_OK;
    if (a.d > 128 || a.d % 32 || a.rows > 0x7FFFFFF) return SR_E_ARG;
    const int heads_per_wave = 64 / (a.d / 8);                 // d/8 threads per head
    const int heads = a.n_q + 2 * a.n_kv;
    int waves = 1;                                             // wavefronts per block
    if (a.rows >= 2048) {
        waves = ceil_div(heads, heads_per_wave);
        if (waves > 10) waves = 10;
    }
    qkv_post_kernel<<<dim3(a.rows, ceil_div(heads, heads_per_wave * waves)), dim3(64 * waves), 0, stream>>>(a);
    SR_HIP(hipGetLastError());
    return SR_OK;
}

int launch_argmax(const float *logits, int rows, int vocab, const int32_t *forced, int32_t *greedy_out,
                  int32_t *chosen, int32_t *actions, int max_turns, int turn_idx, int action_mod,
                  float inv_temperature, uint64_t seed, const int32_t *orig_seq, int pos, hipStream_t stream) {
    if (rows <= 0) return SR_OK;
    argmax_kernel<<<dim3(rows), dim3(1024), 0, stream>>>(logits, vocab, forced, greedy_out, chosen, actions,
                                                         max_turns, turn_idx, action_mod, inv_temperature, seed,
                                                         orig_seq, pos);
    SR_HIP(hipGetLastError());
    return SR_OK;
}

int launch_fill_i32(int32_t *dst, size_t n, int32_t value, hipStream_t stream) {
    if (n == 0) return SR_OK;
    fill_i32_kernel<<<dim3((unsigned)((n + 255) / 256)), dim3(256), 0, stream>>>(dst, n, value);
    SR_HIP(hipGetLastError());
    return SR_OK;
}

int launch_gather_rows(void *dst, const void *src, const int32_t *src_rows, int n_out, size_t row_bytes,
                       hipStream_t stream) {
    if (n_out <= 0 || row_bytes == 0) return SR_OK;
    if (row_bytes % 4) return SR_E_ARG;
    const bool wide = row_bytes % 16 == 0;
    const size_t row_vec = row_bytes / (wide ? 16 : 4);
    unsigned bx = (unsigned)((row_vec + 255) / 256);
    if (bx > 256) bx = 256;
    if (wide)
        gather_rows_kernel<uint4><<<dim3(bx, n_out), dim3(256), 0, stream>>>((uint4 *)dst, (const uint4 *)src, src_rows, row_vec);
    else
        gather_rows_kernel<uint32_t><<<dim3(bx, n_out), dim3(256), 0, stream>>>((uint32_t *)dst, (const uint32_t *)src, src_rows, row_vec);
    SR_HIP(hipGetLastError());
    return SR_OK;
}

int launch_copy_page(uint16_t *kpool, uint16_t *vpool, size_t layer_stride, int n_layers, size_t page_elems,
                     int src_page, int dst_page, hipStream_t stream) {
    const size_t page_vec = page_elems / 8;
    unsigned bx = (unsigned)((page_vec + 255) / 256);
    if (bx > 64) bx = 64;
    copy_page_kernel<<<dim3(bx, n_layers), dim3(256), 0, stream>>>((uint4 *)kpool, (uint4 *)vpool, layer_stride / 8,
                                                                   page_vec, src_page, dst_page);
    SR_HIP(hipGetLastError());
    return SR_OK;
}

}  // namespace sr
