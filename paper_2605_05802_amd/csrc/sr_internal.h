// Internal declarations shared by the translation units of libsr.so (not part of the C boundary).
//
// Data layouts used throughout (all chosen for 64-wide wavefronts and the 16x16x32 bf16 MFMA):
//
//  * "fragment-major" bf16 matrices.  A matrix A[rows][K] that feeds an MFMA is stored as
//    [K/32][rows/16][64 lanes][8 bf16]: element (r, k) lives in k-step k/32, row tile r/16,
//    lane (r%16) + 16*((k%32)/8), slot k%8.  One lane's 16 bytes are exactly its MFMA operand,
//    so a wavefront fetches an operand tile with one fully coalesced 1 KiB load and an LDS copy
//    of a tile is read back conflict-free.  Activations use this layout with rows = batch rows;
//    weights W[N][K] use it with the roles [N/16][K/32][64][8] (k-steps contiguous per row tile,
//    so a wavefront streams its rows of W as one long contiguous run).
//
//  * KV pages.  A page holds page_tokens tokens of one sequence for every layer and kv head,
//    in 32-token blocks.  K block: [d/32][32 tokens][32] (operand tiles of K for S^T = K Q^T
//    are contiguous 1 KiB runs); V block: [d][32 slots], token t of the block stored in slot
//    8*((t%16)/4) + 4*(t/16) + t%4, which is the order in which the S^T accumulator of two
//    16-token tiles hands probabilities to the P^T operand of O^T = V^T P^T.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "sr.h"

namespace sr {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

// Remember the text of the last failing HIP call for sr_strerror(SR_E_HIP).
void note_hip_error(hipError_t e, const char *what);

#define SR_HIP(call)                                   \
    do {                                               \
        hipError_t e__ = (call);                       \
        if (e__ != hipSuccess) {                       \
            ::sr::note_hip_error(e__, #call);          \
            return SR_E_HIP;                           \
        }                                              \
    } while (0)

#define SR_TRY(call)                                   \
    do {                                               \
        int rc__ = (call);                             \
        if (rc__ != SR_OK) return rc__;                \
    } while (0)

__host__ __device__ inline int ceil_div(int a, int b) { return (a + b - 1) / b; }
__host__ __device__ inline int round_up(int a, int b) { return ceil_div(a, b) * b; }

__device__ __forceinline__ float bf16_to_f32(uint16_t b) { return __uint_as_float((uint32_t)b << 16); }
// round to nearest even; inputs are finite
__device__ __forceinline__ uint16_t f32_to_bf16(float f) {
    uint32_t u = __float_as_uint(f);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
    return (uint32_t)f32_to_bf16(lo) | ((uint32_t)f32_to_bf16(hi) << 16);
}

// element offset of (row r, column k) in a fragment-major activation matrix with mt_total row tiles
__host__ __device__ inline size_t frag_offset(int r, int k, int mt_total) {
    return ((((size_t)(k >> 5) * mt_total + (r >> 4)) * 64) + (r & 15) + 16 * ((k & 31) >> 3)) * 8 + (k & 7);
}

// ---------------------------------------------------------------------------------------------
// gate
// ---------------------------------------------------------------------------------------------
// Integer form of the gate rule (Eq. 2): retire iff S_K < gate_bound.
int64_t gate_bound(double d_L, int G, int K);

struct GateLens {
    int n;
    int len[8];
    int bound[8];
};

int launch_gate(const int32_t *actions, int n_groups, int G, int stride, const GateLens &lens,
                int32_t *sums, uint8_t *retire, hipStream_t stream);
// the same result by the other decomposition (one workgroup per group, anti-diagonals in LDS)
int launch_gate_antidiag(const int32_t *actions, int n_groups, int G, int stride, const GateLens &lens,
                         int32_t *sums, uint8_t *retire, hipStream_t stream);

// Gate input of groups with finished members: slot s (group-major, G per group) takes the action row
// src[s] of live_actions when src[s] >= 0, else row -1 - src[s] of fin_actions.
int launch_assemble_gate(const int32_t *src, const int32_t *live_actions, const int32_t *fin_actions, int n_slots,
                         int max_turns, int32_t *out, hipStream_t stream);
// sums[g] = sig[g].lev_sum; retire[g] = use_or ? sig[g].cut_or : sig[g].cut_d
int launch_extract_gate(const sr_signals_t *sig, int n_groups, int use_or, int32_t *sums, uint8_t *retire,
                        hipStream_t stream);

// ---------------------------------------------------------------------------------------------
// weights
// ---------------------------------------------------------------------------------------------
// Pack rows [row0, row0+n_rows) of a row-major bf16 matrix src[*][K] into the weight layout of
// dst (ks_total k-steps per row tile), placing source row row0+i at packed row dst_row0 + f(i):
// f(i) = i (interleave16 == 0) or, for the gate|up pair, 32*(i/16) + 16*which + i%16.
int launch_pack_rows(const uint16_t *src, int n_rows, int K, uint16_t *dst, int ks_total, int dst_row0,
                     int interleave16, int which, hipStream_t stream);

// ---------------------------------------------------------------------------------------------
// GEMM  Y[M][N] = X[M][K] * W[N][K]^T, X fragment-major bf16, W packed bf16, fp32 accumulate
// ---------------------------------------------------------------------------------------------
enum GemmEpilogue {
    EPI_F32 = 0,    // out fp32 [split][M][ld_out] row-major (split-K partials, or the result if splits == 1)
    EPI_SWIGLU = 1  // packed rows alternate 16 gate / 16 up features; out = silu(gate)*up, bf16 fragment-major
};

// k-steps [*k0, *k1) of split sp when `units` groups of `unit` k-steps are dealt out evenly
__device__ __forceinline__ void split_range(int ks_total, int unit, int splits, int sp, int *k0, int *k1) {
    const int units = ks_total / unit, q = units / splits, r = units % splits;
    const int u0 = sp * q + min(sp, r);
    *k0 = u0 * unit;
    *k1 = (u0 + q + (sp < r ? 1 : 0)) * unit;
}


struct GemmArgs {
    const uint4 *X;
    const uint4 *W;
    int M, N;            // valid rows / valid output columns (packed columns for EPI_SWIGLU)
    int mt_total;        // row tiles in X (and in a fragment-major output)
    int ks_total;        // k-steps (K padded to 32) in X and W
    int splits;          // split-K factor (EPI_F32 only)
    int wide;            // M <= 128 only: 2, 4, 5, 8 or 10 = computing wavefronts per workgroup (32 features each) of the
                         // kernel with a loader wavefront; 0 = the 4-wavefront, 128-feature kernel
    int ring;            // with `wide`: k-steps of weights in flight per wavefront, 8 (default) or 16
    void *out;
    int ld_out;          // EPI_F32: row stride (elements); EPI_SWIGLU: k-steps*32 of the output matrix
    size_t split_stride; // EPI_F32: elements between consecutive splits
};

// The decode-time kernel with a loader wavefront (a.wide != 0, M <= 128); launch_gemm dispatches to it.
int launch_gemm_stream(const GemmArgs &a, GemmEpilogue epi, hipStream_t stream);
int launch_gemm(const GemmArgs &a, GemmEpilogue epi, hipStream_t stream);

// ---------------------------------------------------------------------------------------------
// element-wise kernels
// ---------------------------------------------------------------------------------------------
struct NormArgs {
    float *resid;            // [rows][H] fp32 residual stream (updated in place)
    const float *partials;   // [n_partials][rows][H] fp32 to be added first, or null
    int n_partials;
    size_t partial_stride;
    const int32_t *tokens;   // embedding mode (embed != null): resid[m] = embed[tokens[index(m)]], with
    int tok_chunk, tok_stride, tok_off;  //   index(m) = (m / tok_chunk) * tok_stride + tok_off + m % tok_chunk
    const uint16_t *embed;
    const uint16_t *gain;    // [H] bf16
    uint4 *out;              // fragment-major bf16 [rows_out][H]
    float *out32;            // non-null (single-precision debugging path): row-major fp32 [rows_out][H] instead of `out`
    int rows_out;            // rows normalised (grid size)
    int src_dup, src_stride, src_off;  // source row of output row m: (m / src_dup) * src_stride + src_off
    int write_resid;         // 0: leave resid untouched (several output rows may share one source row)
    int H, mt_total;
    float eps;
};
int launch_resid_norm(const NormArgs &a, hipStream_t stream);

struct QkvPostArgs {
    const float *partials;   // [n_partials][rows][ld] fp32: columns [q | k | v]
    int n_partials;
    size_t partial_stride;
    int ld;
    const uint16_t *bq, *bk, *bv;  // may be null
    const float *rope_cos, *rope_sin;  // [max_pos][d/2]
    uint16_t *q_out;         // [rows][n_q][d] bf16
    uint16_t *kpool, *vpool; // layer base
    const int32_t *page_table;
    int pt_stride;           // entries per page-table row
    int pt_row_stride;       // page-table row of unit u = u * pt_row_stride
    int rows, chunk;         // row m = unit (m / chunk), token (m % chunk) of the chunk
    int pos0;                // absolute position of the chunk's first token
    int n_q, n_kv, d, page_tokens;
};
int launch_qkv_post(const QkvPostArgs &a, hipStream_t stream);

// greedy[r] = lowest index of the largest logit of row r; tok = forced ? forced[r] : greedy[r];
// chosen[r] = tok; if actions != null: actions[r*max_turns + turn_idx] = tok % action_mod.
// inv_temperature > 0: sample instead (Gumbel-max over logits * inv_temperature, uniforms keyed by
// (seed, orig_seq[r], pos)).
int launch_argmax(const float *logits, int rows, int vocab, const int32_t *forced, int32_t *greedy_out,
                  int32_t *chosen, int32_t *actions, int max_turns, int turn_idx, int action_mod,
                  float inv_temperature, uint64_t seed, const int32_t *orig_seq, int pos, hipStream_t stream);

// ---------------------------------------------------------------------------------------------
// attention
// ---------------------------------------------------------------------------------------------
// One launch covers one token range of the context for a set of "units" (a sequence, or a group
// when the range is the prompt shared by its members).  A work item (one wavefront) owns up to
// 16*RT query rows = q_per_item consecutive query tokens of a unit x the n_rep query heads of
// one kv head, and one split of the token range.
struct AttnPhase {
    int n_units;
    int q_per_unit;      // query tokens per unit (prefill: chunk; decode private: 1; decode shared: G)
    int q_per_item;      // query tokens per work item
    int items_per_unit;  // ceil(q_per_unit / q_per_item)
    int pt_row_stride;   // page-table row of unit u = u * pt_row_stride
    int t_begin, t_end;  // token range [t_begin, t_end)
    int causal_pos0, causal_stride;  // query token i of a unit sees tokens t <= causal_pos0 + i*causal_stride
    int n_splits, split_tokens;      // split s covers [t_begin + s*split_tokens, ...) (multiples of 32)
    int rt;              // row tiles per item (1 or 2)
    int stream_loads;    // 1: no other work item of the launch reads this phase's tokens; fetch them with the
                         // non-temporal hint
    // Units of unequal size (a group some of whose members have left the batch): unit u owns query tokens
    // unit_row0[u] .. unit_row0[u] + unit_count[u] - 1 (count <= q_per_unit) and its pages are those of row
    // unit_row0[u]; row_unit[token] is the unit of a query token.  All three null: unit u owns tokens
    // u * q_per_unit .. and page-table row u * pt_row_stride.
    const int32_t *unit_row0, *unit_count, *row_unit;
    float *part_o;       // [items][16*rt][d] fp32 un-normalised outputs
    float *part_ml;      // [items][16*rt][2] running max (scaled logits) and sum
};

struct AttnArgs {
    const uint16_t *q;   // [query tokens][n_q][d] bf16
    const uint16_t *kpool, *vpool;   // layer base
    const int32_t *page_table;
    int pt_stride, page_tokens, n_q, n_kv, d;
    float scale;
    // Non-null only when every query row gets exactly one partial result (one phase, one split): the attention
    // kernel then normalises and writes the fragment-major bf16 output [query tokens][n_q*d] itself, with the
    // arithmetic of the merge, and no merge is launched.
    uint16_t *direct_out;
    int out_mt_total;
};
// One launch over one or two phases (same rt); phases whose token range is empty contribute no work.
int launch_attention(const AttnArgs &a, const AttnPhase *phases, int n_phases, hipStream_t stream);

// Merge the partial results of up to two phases into out (fragment-major bf16 [query tokens][n_q*d]) or, when
// out32 is non-null (single-precision debugging path), into out32 (row-major fp32, same shape).
// Query token qt belongs to unit qt / q_per_unit of each phase.
int launch_attn_merge(const AttnArgs &a, const AttnPhase *phases, int n_phases, int n_qtok, uint4 *out,
                      int mt_total, float *out32, hipStream_t stream);

// ---------------------------------------------------------------------------------------------
// single-precision debugging path (sr_options.fp32_debug): same work decomposition, plain fp32 arithmetic
// ---------------------------------------------------------------------------------------------
// Y = X W^T with X row-major fp32 [M][K] and W the packed bf16 matrix of the normal path (widened exactly).
// K splits cover the same k-step ranges as the normal path's split-K; EPI_F32 writes [split][M][ld_out] fp32,
// EPI_SWIGLU writes silu(gate) * up as row-major fp32 [M][ld_out] (ld_out = ffn; splits must be 1).
struct DbgGemmArgs {
    const float *X;
    int ldx;                 // = K, the valid inner dimension
    const uint16_t *W;
    int M, N, ks_total, splits;
    float *out;
    int ld_out;
    size_t split_stride;
};
int launch_dbg_gemm(const DbgGemmArgs &a, GemmEpilogue epi, hipStream_t stream);

// qkv_post with fp32 outputs: q_out [rows][n_q][d] fp32; K and V pages [page][kv head][page_tokens][d] fp32.
struct DbgQkvPostArgs {
    QkvPostArgs base;        // q_out, kpool, vpool of `base` are unused
    float *q32, *kpool32, *vpool32;
};
int launch_dbg_qkv_post(const DbgQkvPostArgs &a, hipStream_t stream);

// Attention over fp32 pages with the phases, work items and partial-result format of launch_attention.
// direct_out32 (row-major fp32 [query tokens][n_q*d]) plays the role of AttnArgs::direct_out.
struct DbgAttnArgs {
    AttnArgs base;           // q, kpool, vpool, direct_out of `base` are unused
    const float *q32, *kpool32, *vpool32;
    float *direct_out32;
};
int launch_dbg_attention(const DbgAttnArgs &a, const AttnPhase *phases, int n_phases, hipStream_t stream);

// ---------------------------------------------------------------------------------------------
// teacher-forced scoring
// ---------------------------------------------------------------------------------------------
// Row r of `logits` is row row0 + r of a pass whose units hold rows_per_unit consecutive rows each: it
// belongs to unit (row0 + r) / rows_per_unit and gives the distribution of chunk token
// tok0 + (row0 + r) % rows_per_unit of that unit; out[unit][token] = log softmax(row)[tokens[unit][token]],
// or 0 where mask[unit][token] == 0.  Rows whose token index is >= chunk_len are skipped.
struct LogprobArgs {
    const float *logits;     // [rows][vocab]
    int vocab;
    const int32_t *tokens;   // [units][chunk_len]
    const uint8_t *mask;     // [units][chunk_len] or null
    int chunk_len;
    int row0, rows_per_unit, tok0;
    float *out;              // [units][chunk_len]
};
int launch_logprob_rows(const LogprobArgs &a, int rows, hipStream_t stream);
// logprob[u] += sum over t of tok_lp[u][t], in token order
int launch_accumulate_logprob(const float *tok_lp, int n_seq, int chunk_len, double *logprob, hipStream_t stream);

// ---------------------------------------------------------------------------------------------
// misc
// ---------------------------------------------------------------------------------------------
int launch_fill_i32(int32_t *dst, size_t n, int32_t value, hipStream_t stream);
// dst row r (r < n_out) = src row src_rows[r], row_bytes each (multiples of 4)
int launch_gather_rows(void *dst, const void *src, const int32_t *src_rows, int n_out, size_t row_bytes,
                       hipStream_t stream);
// copy `tokens` leading tokens of page src to page dst for every layer and kv head
int launch_copy_page(uint16_t *kpool, uint16_t *vpool, size_t layer_stride, int n_layers, size_t page_elems,
                     int src_page, int dst_page, hipStream_t stream);

}  // namespace sr
