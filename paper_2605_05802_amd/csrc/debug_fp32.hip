// Single-precision debugging path (sr_options.fp32_debug).
//
// The same decoder with every activation, the stored keys and values and the attention probabilities in
// fp32 and every contraction as plain fused multiply-adds -- no bf16 rounding of operands, no matrix
// cores.  What is NOT different is everything that could hide an indexing mistake behind rounding noise:
// the page tables and copy-on-write, the (unit, kv head, split, query tile) decomposition of attention and
// its partial-result format and merge, the k-step ranges of the projections' K splits and the order in
// which the consumers add the partial sums, the packed weight layout (read here element by element),
// token selection, gate and compaction.  Against an exact evaluation this path differs by single-precision
// rounding only.  Speed is not a goal: tiles are small and go through LDS once.
#include "sr_internal.h"

namespace sr {
namespace {

constexpr float kNegBig = -1.0e30f;
constexpr int kTile = 64;            // output tile of the debugging GEMM: 64 rows x 64 packed columns

// One 256-thread workgroup per (64 packed columns, 64 rows, K split); thread (ty, tx) owns a 4 x 4 patch.
// Products are added in ascending k within the split, in fp32.
template <int EPI>
__global__ __launch_bounds__(256) void dbg_gemm_kernel(DbgGemmArgs a) {
    __shared__ float xs[32][kTile + 1];       // [k][row]
    __shared__ float ws[32][kTile + 1];       // [k][column]
    __shared__ float cs[EPI == EPI_SWIGLU ? kTile : 1][kTile + 1];
    const int tid = threadIdx.x, tx = tid & 15, ty = tid >> 4;
    const int n0 = blockIdx.x * kTile, m0 = blockIdx.y * kTile, sp = blockIdx.z;
    int ks0, ks1;
    split_range(a.ks_total, 8, a.splits, sp, &ks0, &ks1);

    float acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = 0.f;

    for (int ks = ks0; ks < ks1; ++ks) {
        // X tile: 64 rows x 32 k, coalesced along k
#pragma unroll
        for (int r = 0; r < 8; ++r) {
            const int idx = tid + 256 * r, row = idx >> 5, kk = idx & 31;
            const int m = m0 + row, k = ks * 32 + kk;
            xs[kk][row] = (m < a.M && k < a.ldx) ? a.X[(size_t)m * a.ldx + k] : 0.f;
        }
        // W tile: four 16-column tiles of the packed matrix; lane slot (n % 16) + 16 * (k % 32 / 8), 8 bf16 each
        {
            const int j = tid >> 6, lane = tid & 63;
            const int nt = (n0 >> 4) + j;
            const uint16_t *src = a.W + (((size_t)nt * a.ks_total + ks) * 64 + lane) * 8;
            const uint4 raw = *(const uint4 *)src;
            const uint32_t w[4] = {raw.x, raw.y, raw.z, raw.w};
            const int n = j * 16 + (lane & 15), kb = (lane >> 4) * 8;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                ws[kb + 2 * e][n] = __uint_as_float(w[e] << 16);
                ws[kb + 2 * e + 1][n] = __uint_as_float(w[e] & 0xFFFF0000u);
            }
        }
        __syncthreads();
#pragma unroll 8
        for (int k = 0; k < 32; ++k) {
            float xv[4], wv[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) { xv[i] = xs[k][ty * 4 + i]; wv[i] = ws[k][tx * 4 + i]; }
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(xv[i], wv[j], acc[i][j]);
        }
        __syncthreads();
    }

    if constexpr (EPI == EPI_F32) {
        float *out = a.out + (size_t)sp * a.split_stride;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int m = m0 + ty * 4 + i;
            if (m >= a.M) continue;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int n = n0 + tx * 4 + j;
                if (n < a.N) out[(size_t)m * a.ld_out + n] = acc[i][j];
            }
        }
    } else {
        // packed columns come in groups of 32: 16 gate features, then the 16 matching up features
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j) cs[ty * 4 + i][tx * 4 + j] = acc[i][j];
        __syncthreads();
#pragma unroll
        for (int r = 0; r < 8; ++r) {
            const int idx = tid + 256 * r, row = idx >> 5, f = idx & 31;
            const int m = m0 + row, feat = (n0 >> 1) + f;
            if (m < a.M && feat < a.ld_out) {
                const float g = cs[row][(f >> 4) * 32 + (f & 15)], u = cs[row][(f >> 4) * 32 + 16 + (f & 15)];
                a.out[(size_t)m * a.ld_out + feat] = g / (1.0f + expf(-g)) * u;
            }
        }
    }
}

// One 64-thread workgroup per (row, head); thread i owns the rotation pair (i, i + d/2).
__global__ __launch_bounds__(64) void dbg_qkv_post_kernel(DbgQkvPostArgs x) {
    const QkvPostArgs &a = x.base;
    const int half = a.d >> 1;
    const int m = blockIdx.x, head = blockIdx.y, i = threadIdx.x;
    if (i >= half) return;
    const int unit = m / a.chunk, ci = m - unit * a.chunk;
    const int pos = a.pos0 + ci;
    const int q_cols = a.n_q * a.d, kv_cols = a.n_kv * a.d;
    int col0, kind, h;
    const uint16_t *bias;
    if (head < a.n_q) { kind = 0; h = head; col0 = h * a.d; bias = a.bq ? a.bq + h * a.d : nullptr; }
    else if (head < a.n_q + a.n_kv) { kind = 1; h = head - a.n_q; col0 = q_cols + h * a.d; bias = a.bk ? a.bk + h * a.d : nullptr; }
    else { kind = 2; h = head - a.n_q - a.n_kv; col0 = q_cols + kv_cols + h * a.d; bias = a.bv ? a.bv + h * a.d : nullptr; }

    float lo = 0.f, hi = 0.f;
    const float *p0 = a.partials + (size_t)m * a.ld + col0 + i;
    for (int s = 0; s < a.n_partials; ++s) {              // split order, as the normal path
        lo += p0[(size_t)s * a.partial_stride];
        hi += p0[(size_t)s * a.partial_stride + half];
    }
    if (bias) { lo += bf16_to_f32(bias[i]); hi += bf16_to_f32(bias[i + half]); }
    if (kind != 2) {
        const float c = a.rope_cos[(size_t)pos * half + i], sn = a.rope_sin[(size_t)pos * half + i];
        const float rlo = lo * c - hi * sn, rhi = hi * c + lo * sn;
        lo = rlo; hi = rhi;
    }
    if (kind == 0) {
        float *q = x.q32 + ((size_t)m * a.n_q + h) * a.d;
        q[i] = lo;
        q[i + half] = hi;
        return;
    }
    const int page = a.page_table[(size_t)unit * a.pt_row_stride * a.pt_stride + pos / a.page_tokens];
    const int tok = pos % a.page_tokens;
    float *dst = (kind == 1 ? x.kpool32 : x.vpool32) + (((size_t)page * a.n_kv + h) * a.page_tokens + tok) * a.d;
    dst[i] = lo;
    dst[i + half] = hi;
}

// One wavefront per (work item, query row of the item); lane l owns head dimensions l and l + 64.
// Tokens are visited one by one with a running maximum and sum (base-2 exponentials of the scaled scores, the
// convention of the partial-result format), so a split leaves exactly what the normal path's split leaves.
__global__ __launch_bounds__(256) void dbg_attn_kernel(DbgAttnArgs x, AttnPhase p0, AttnPhase p1, int n0, int rows_per_item) {
    const AttnArgs &a = x.base;
    const int lane = threadIdx.x & 63;
    const int row = blockIdx.y * 4 + (threadIdx.x >> 6);
    if (row >= rows_per_item) return;
    const int gitem = blockIdx.x;
    const bool second = gitem >= n0;
    const AttnPhase &p = second ? p1 : p0;
    const int item = second ? gitem - n0 : gitem;

    int rest = item;
    const int qtile = rest % p.items_per_unit; rest /= p.items_per_unit;
    const int split = rest % p.n_splits; rest /= p.n_splits;
    const int kvh = rest % a.n_kv;
    const int unit = rest / a.n_kv;
    const int n_rep = a.n_q / a.n_kv;
    const int D = a.d;

    const int u_row0 = p.unit_row0 ? p.unit_row0[unit] : unit * p.q_per_unit;
    const int u_count = p.unit_count ? p.unit_count[unit] : p.q_per_unit;
    const int32_t *pt = a.page_table + (size_t)(p.unit_row0 ? u_row0 : unit * p.pt_row_stride) * a.pt_stride;

    const int qi = qtile * p.q_per_item + row / n_rep, hr = row % n_rep;
    const bool used = (row < p.q_per_item * n_rep) && (qi < u_count);
    if (!used) return;
    const int limit = p.causal_pos0 + qi * p.causal_stride;
    const int t_lo = p.t_begin + split * p.split_tokens;
    const int t_hi = min(min(p.t_end, t_lo + p.split_tokens), limit + 1);

    const size_t qtok = (size_t)u_row0 + qi;
    const float *q = x.q32 + (qtok * a.n_q + kvh * n_rep + hr) * D;
    const bool two = D > 64;
    const float q0 = lane < D ? q[lane] : 0.f, q1 = two ? q[lane + 64] : 0.f;
    const float scale_log2 = a.scale * 1.4426950408889634f;

    float m = kNegBig, l = 0.f, o0 = 0.f, o1 = 0.f;
    for (int t = t_lo; t < t_hi; ++t) {
        const int page = pt[t / a.page_tokens];
        const size_t base = (((size_t)page * a.n_kv + kvh) * a.page_tokens + t % a.page_tokens) * D;
        const float *k = x.kpool32 + base, *v = x.vpool32 + base;
        float dot = lane < D ? q0 * k[lane] : 0.f;
        if (two) dot = fmaf(q1, k[lane + 64], dot);
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) dot += __shfl_xor(dot, off, 64);
        const float s = dot * scale_log2;
        const float mnew = fmaxf(m, s);
        const float alpha = exp2f(m - mnew), pe = exp2f(s - mnew);
        m = mnew;
        l = l * alpha + pe;
        o0 = o0 * alpha + (lane < D ? pe * v[lane] : 0.f);
        if (two) o1 = o1 * alpha + pe * v[lane + 64];
    }

    if (x.direct_out32) {
        float *dst = x.direct_out32 + (qtok * a.n_q + kvh * n_rep + hr) * D;
        if (lane < D) dst[lane] = l > 0.f ? o0 / l : 0.f;
        if (two) dst[lane + 64] = l > 0.f ? o1 / l : 0.f;
        return;
    }
    const size_t prow = (size_t)item * rows_per_item + row;
    float *po = p.part_o + prow * D;
    if (lane < D) po[lane] = o0;
    if (two) po[lane + 64] = o1;
    if (lane == 0) {
        p.part_ml[prow * 2] = m;
        p.part_ml[prow * 2 + 1] = l;
    }
}

}  // namespace

int launch_dbg_gemm(const DbgGemmArgs &a, GemmEpilogue epi, hipStream_t stream) {
    if (a.M <= 0) return SR_OK;
    if (a.splits < 1 || a.splits > 65535 || a.ks_total % 8 || a.ldx > a.ks_total * 32) return SR_E_ARG;
    if (epi == EPI_SWIGLU && a.splits != 1) return SR_E_ARG;
    dim3 grid(ceil_div(a.N, kTile), ceil_div(a.M, kTile), a.splits), block(256);
    if (grid.y > 65535) return SR_E_ARG;
    if (epi == EPI_F32) dbg_gemm_kernel<EPI_F32><<<grid, block, 0, stream>>>(a);
    else dbg_gemm_kernel<EPI_SWIGLU><<<grid, block, 0, stream>>>(a);
    SR_HIP(hipGetLastError());
    return SR_OK;
}

int launch_dbg_qkv_post(const DbgQkvPostArgs &a, hipStream_t stream) {
    if (a.base.rows <= 0) return SR_OK;
    if (a.base.d > 128 || a.base.d % 2 || a.base.rows > 0x7FFFFFF) return SR_E_ARG;
    dbg_qkv_post_kernel<<<dim3(a.base.rows, a.base.n_q + 2 * a.base.n_kv), dim3(64), 0, stream>>>(a);
    SR_HIP(hipGetLastError());
    return SR_OK;
}

int launch_dbg_attention(const DbgAttnArgs &a, const AttnPhase *phases, int n_phases, hipStream_t stream) {
    if (n_phases < 1 || n_phases > 2 || a.base.d > 128) return SR_E_ARG;
    long long n[2] = {0, 0};
    const int n_rep = a.base.n_q / a.base.n_kv;
    for (int i = 0; i < n_phases; ++i) {
        const AttnPhase &p = phases[i];
        n[i] = (long long)p.n_units * a.base.n_kv * p.items_per_unit * p.n_splits;
        if (p.t_end <= p.t_begin) n[i] = 0;
        if (p.split_tokens <= 0 || p.q_per_item * n_rep > 16 * p.rt || p.rt != phases[0].rt) return SR_E_ARG;
    }
    if (a.direct_out32 && (n_phases != 1 || phases[0].n_splits != 1)) return SR_E_ARG;
    const long long n_items = n[0] + n[1];
    if (n_items <= 0) return SR_OK;
    if (n_items > 0x7FFFFFFF) return SR_E_ARG;
    const int rows_per_item = 16 * phases[0].rt;
    dbg_attn_kernel<<<dim3((unsigned)n_items, rows_per_item / 4), dim3(256), 0, stream>>>(
        a, phases[0], phases[n_phases - 1], (int)n[0], rows_per_item);
    SR_HIP(hipGetLastError());
    return SR_OK;
}

}  // namespace sr
