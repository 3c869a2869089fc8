// Grouped-query attention over the paged KV cache, for decode and for chunked prefill.
//
// A work item is one wavefront.  It owns up to 16*RT query rows -- consecutive query tokens of
// one unit times the n_rep query heads that share one kv head -- and one split of a token
// range.  K and V tiles go from HBM straight into MFMA operand registers (the page layout is
// the operand layout, so each 16-byte lane load is part of a contiguous 1 KiB run); nothing is
// staged in LDS because a KV byte is used by exactly one wavefront.
//
// Per 32-token block:   S^T = K Q^T   (tokens x rows; the accumulator leaves each lane holding
// four consecutive tokens of one query row), online softmax with the row maximum reduced by
// two cross-lane shuffles, then  O^T += V^T P^T  where the probabilities of the two 16-token
// tiles are packed, in-lane, into the P^T operand (the V block's slot order matches).
// Splits leave (un-normalised O, running max, running sum); a merge kernel combines the splits
// of the shared-prompt phase and of the private phase in fixed order.
//
// Group batching: during decode the prompt pages shared by the G members of a group are read
// once per group (the members' G*n_rep query rows form the row tiles of the work item)
// instead of once per member.
#include <type_traits>

#include "sr_internal.h"

namespace sr {
namespace {

constexpr float kNegBig = -1.0e30f;
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// A 16-byte K/V fragment.  STREAM: with the non-temporal hint, for tokens that exactly one work item reads in
// this launch (a sequence's private context): the caches do not retain the line and a long stream gains 8 %.
// Blocks that sibling work items re-read (the shared prompt, prefill) keep the default policy.
template <bool STREAM>
__device__ __forceinline__ bf16x8 load_frag(const uint16_t *p) {
    if constexpr (STREAM) return __builtin_bit_cast(bf16x8, __builtin_nontemporal_load((const u32x4 *)p));
    else return __builtin_bit_cast(bf16x8, *(const u32x4 *)p);
}

// One launch may cover two phases (decode: the shared-prompt phase followed by the private phase), so
// that the short, narrow shared phase overlaps the private one instead of running alone.
template <int D, int RT>
__global__ __launch_bounds__(256, RT == 1 ? 3 : 2) void attn_kernel(AttnArgs a, AttnPhase p0, AttnPhase p1, int n0, int n_items) {
    constexpr int KS = D / 32;     // k-steps of the QK^T contraction
    constexpr int DT = D / 16;     // 16-wide tiles of the head dimension
    const int lane = threadIdx.x & 63;
    // the wavefront index is uniform: tell the compiler, so that everything derived from the work item
    // (phase, token range, page-table reads) lives in scalar registers
    const int gitem = blockIdx.x * 4 + __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    if (gitem >= n_items) return;
    const bool second = gitem >= n0;
    const AttnPhase &p = second ? p1 : p0;
    const int item = second ? gitem - n0 : gitem;

    // item -> (unit, kv head, split, q tile): the q tiles of one split are neighbours
    int rest = item;
    const int qtile = rest % p.items_per_unit; rest /= p.items_per_unit;
    const int split = rest % p.n_splits; rest /= p.n_splits;
    const int kvh = rest % a.n_kv;
    const int unit = rest / a.n_kv;
    const int n_rep = a.n_q / a.n_kv;

    const int c = lane & 15, g = lane >> 4;
    const int u_row0 = p.unit_row0 ? p.unit_row0[unit] : unit * p.q_per_unit;   // first query token of the unit
    const int u_count = p.unit_count ? p.unit_count[unit] : p.q_per_unit;       // its query tokens
    const int32_t *pt = a.page_table + (size_t)(p.unit_row0 ? u_row0 : unit * p.pt_row_stride) * a.pt_stride;
    const int blocks_per_page = a.page_tokens >> 5;
    const size_t block_elems = (size_t)32 * D;
    auto block_base = [&](int t0) -> size_t {
        const int page = pt[t0 / a.page_tokens];
        const int blk = (t0 % a.page_tokens) >> 5;
        return (((size_t)page * a.n_kv + kvh) * blocks_per_page + blk) * block_elems;
    };
    const int t_lo = p.t_begin + split * p.split_tokens;

    // query rows of this lane's column c in each row tile
    bf16x8 qf[RT][KS];
    int limit[RT];                  // last visible token of row (rt, c); -1 = row unused
#pragma unroll
    for (int rt = 0; rt < RT; ++rt) {
        const int row = rt * 16 + c;
        const int qi = qtile * p.q_per_item + row / n_rep;       // query token within the unit
        const int hr = row % n_rep;
        const bool used = (row < p.q_per_item * n_rep) && (qi < u_count);
        limit[rt] = used ? p.causal_pos0 + qi * p.causal_stride : -1;
        const size_t qtok = (size_t)u_row0 + qi;
        const uint16_t *qp = a.q + (qtok * a.n_q + kvh * n_rep + hr) * D + 8 * g;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            uint4 raw = make_uint4(0, 0, 0, 0);
            if (used) raw = *(const uint4 *)(qp + ks * 32);
            qf[rt][ks] = __builtin_bit_cast(bf16x8, raw);
        }
    }

    // token range of this split, clipped to what any row of the item can see
    int max_limit = -1;
#pragma unroll
    for (int rt = 0; rt < RT; ++rt) max_limit = max(max_limit, limit[rt]);
#pragma unroll
    for (int off = 1; off < 16; off <<= 1) max_limit = max(max_limit, __shfl_xor(max_limit, off, 64));
    // the same in every lane after the reduction; kept in a scalar register so that the block loop, the
    // page-table lookups and the block addresses stay on the scalar unit
    const int t_hi = __builtin_amdgcn_readfirstlane(min(min(p.t_end, t_lo + p.split_tokens), max_limit + 1));

    f32x4 o[DT][RT];
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
        for (int rt = 0; rt < RT; ++rt) o[dt][rt] = f32x4{0.f, 0.f, 0.f, 0.f};
    float mrun[RT], lrun[RT];
#pragma unroll
    for (int rt = 0; rt < RT; ++rt) { mrun[rt] = kNegBig; lrun[rt] = 0.f; }
    const float scale_log2 = a.scale * 1.4426950408889634f;

    bf16x8 kf[2][KS], vf[DT];
    auto load_k = [&](auto stream, const uint16_t *kb) {
#pragma unroll
        for (int tt = 0; tt < 2; ++tt)
#pragma unroll
            for (int ks = 0; ks < KS; ++ks)
                kf[tt][ks] = load_frag<decltype(stream)::value>(kb + ((ks * 32 + tt * 16 + c) * 32 + 8 * g));
    };
    auto load_v = [&](auto stream, const uint16_t *vb) {
#pragma unroll
        for (int dt = 0; dt < DT; ++dt)
            vf[dt] = load_frag<decltype(stream)::value>(vb + ((dt * 16 + c) * 32 + 8 * g));
    };
    // S^T = K Q^T for all row tiles
    auto scores = [&](f32x4 (&s)[RT][2]) {
#pragma unroll
        for (int rt = 0; rt < RT; ++rt)
#pragma unroll
            for (int tt = 0; tt < 2; ++tt) {
                s[rt][tt] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int ks = 0; ks < KS; ++ks)
                    s[rt][tt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf[tt][ks], qf[rt][ks], s[rt][tt], 0, 0, 0);
            }
    };
    // online softmax of one block; leaves the packed probabilities and the rescale factor per row tile
    auto softmax = [&](f32x4 (&s)[RT][2], int t0, bf16x8 (&pf)[RT], float (&alpha)[RT]) {
#pragma unroll
        for (int rt = 0; rt < RT; ++rt) {
            // lane holds tokens t0 + tt*16 + 4g + e of query row (rt, c)
            const int lim = min(limit[rt], t_hi - 1);
            float bmax = kNegBig;
            bool ok[2][4];
#pragma unroll
            for (int tt = 0; tt < 2; ++tt)
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    ok[tt][e] = (t0 + tt * 16 + 4 * g + e) <= lim;
                    s[rt][tt][e] = ok[tt][e] ? s[rt][tt][e] * scale_log2 : kNegBig;
                    bmax = fmaxf(bmax, s[rt][tt][e]);
                }
            bmax = fmaxf(bmax, __shfl_xor(bmax, 16, 64));
            bmax = fmaxf(bmax, __shfl_xor(bmax, 32, 64));
            const float mnew = fmaxf(mrun[rt], bmax);
            alpha[rt] = exp2f(mrun[rt] - mnew);
            mrun[rt] = mnew;
            float psum = 0.f;
            float pv[8];
#pragma unroll
            for (int tt = 0; tt < 2; ++tt)
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const float pe = ok[tt][e] ? exp2f(s[rt][tt][e] - mnew) : 0.f;
                    pv[tt * 4 + e] = pe;
                    psum += pe;
                }
            lrun[rt] = lrun[rt] * alpha[rt] + psum;
            const uint4 praw = make_uint4(pack_bf16x2(pv[0], pv[1]), pack_bf16x2(pv[2], pv[3]),
                                          pack_bf16x2(pv[4], pv[5]), pack_bf16x2(pv[6], pv[7]));
            pf[rt] = __builtin_bit_cast(bf16x8, praw);
        }
    };
    // O^T = alpha O^T + V^T P^T
    auto accumulate = [&](const bf16x8 (&pf)[RT], const float (&alpha)[RT]) {
#pragma unroll
        for (int rt = 0; rt < RT; ++rt)
#pragma unroll
            for (int dt = 0; dt < DT; ++dt) {
                o[dt][rt] *= alpha[rt];
                o[dt][rt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf[dt], pf[rt], o[dt][rt], 0, 0, 0);
            }
    };

    // Software pipeline without spare registers: the K fragments of the next block are requested
    // into the registers of the current ones as soon as the score MFMAs have consumed them, and
    // the V fragments likewise after the P.V MFMAs, so 8 KiB per wavefront (d = 128) are in
    // flight behind the softmax and behind the next block's scores.  With one row tile (decode) the register
    // budget stays low enough for three wavefronts per SIMD, so every item of a decode step is resident at once.
    auto block_loop = [&](auto stream) {
        if (t_lo < t_hi) {
            const size_t base = block_base(t_lo);
            load_k(stream, a.kpool + base);
            load_v(stream, a.vpool + base);
        }
        for (int t0 = t_lo; t0 < t_hi; t0 += 32) {          // t_lo is a multiple of 32
            const int tn = t0 + 32 < t_hi ? t0 + 32 : t0;   // after the last block: harmless re-read
            const size_t base_n = block_base(tn);
            f32x4 s[RT][2];
            scores(s);
            // the scheduling fences keep each refill where it is written: right behind the last use
            // of the registers it overwrites, a whole softmax (or score pass) ahead of its first use
            __builtin_amdgcn_sched_barrier(0);
            load_k(stream, a.kpool + base_n);
            __builtin_amdgcn_sched_barrier(0);
            bf16x8 pf[RT];
            float alpha[RT];
            softmax(s, t0, pf, alpha);
            accumulate(pf, alpha);
            __builtin_amdgcn_sched_barrier(0);
            load_v(stream, a.vpool + base_n);
            __builtin_amdgcn_sched_barrier(0);
        }
    };
    if (p.stream_loads) block_loop(std::true_type{});       // uniform: one of two copies of the loop runs
    else block_loop(std::false_type{});

    // results: O^T tile lane (c, g) holds head dims dt*16 + 4g..4g+3 of row (rt, c)
#pragma unroll
    for (int rt = 0; rt < RT; ++rt) {
        float l = lrun[rt];
        l += __shfl_xor(l, 16, 64);
        l += __shfl_xor(l, 32, 64);
        if (a.direct_out) {
            // the only partial result of its rows: what the merge of one item computes, o / l (0 for an empty row)
            if (limit[rt] < 0) continue;
            const int row = rt * 16 + c;
            const size_t qtok = (size_t)u_row0 + qtile * p.q_per_item + row / n_rep;
            const int col = (kvh * n_rep + row % n_rep) * D + 4 * g;
#pragma unroll
            for (int dt = 0; dt < DT; ++dt) {
                float r[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) r[e] = l > 0.f ? o[dt][rt][e] / l : 0.f;
                *(uint2 *)(a.direct_out + frag_offset((int)qtok, col + dt * 16, a.out_mt_total)) =
                    make_uint2(pack_bf16x2(r[0], r[1]), pack_bf16x2(r[2], r[3]));
            }
            continue;
        }
        const size_t prow = (size_t)item * (16 * RT) + rt * 16 + c;
        float *po = p.part_o + prow * D;
        if (limit[rt] < 0) continue;        // padding row of the tile: the merge never reads it
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) *(f32x4 *)(po + dt * 16 + 4 * g) = o[dt][rt];
        if (g == 0) {
            p.part_ml[prow * 2] = mrun[rt];
            p.part_ml[prow * 2 + 1] = l;
        }
    }
}

// ---------------------------------------------------------------------------------------------
// Prefill attention: the four work items of a workgroup are four consecutive query tiles of one
// (unit, kv head) and need the same K/V blocks, so a block goes from global memory to LDS once per
// workgroup (each thread copies its 16-byte slots, one block ahead, through registers) and every
// wavefront takes its MFMA operands from LDS: a quarter of the vector-memory traffic of the kernel
// above, which at a context of thousands of tokens is bound by what L2 can deliver.  Two LDS buffers,
// one workgroup barrier per block.  One split, one phase: the normalised output is written directly.
// ---------------------------------------------------------------------------------------------
template <int D, int RT>
__global__ __launch_bounds__(256, 2) void attn_prefill_shared_kernel(AttnArgs a, AttnPhase p) {
    constexpr int KS = D / 32, DT = D / 16;
    constexpr int SLOTS = 32 * D / 8;              // 16-byte slots of one K (or V) block
    constexpr int NS = SLOTS / 256;                // slots per thread
    __shared__ u32x4 lds[2][2][SLOTS];             // [buffer][K, V][slot]
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);

    const int groups_per_unit = (p.items_per_unit + 3) >> 2;
    int rest = blockIdx.x;
    const int qg = rest % groups_per_unit; rest /= groups_per_unit;
    const int kvh = rest % a.n_kv;
    const int unit = rest / a.n_kv;
    const int qtile = qg * 4 + wave;               // beyond items_per_unit: this wavefront only helps with the copies
    const int n_rep = a.n_q / a.n_kv;

    const int c = lane & 15, g = lane >> 4;
    const int u_row0 = p.unit_row0 ? p.unit_row0[unit] : unit * p.q_per_unit;
    const int u_count = p.unit_count ? p.unit_count[unit] : p.q_per_unit;
    const int32_t *pt = a.page_table + (size_t)(p.unit_row0 ? u_row0 : unit * p.pt_row_stride) * a.pt_stride;
    const int blocks_per_page = a.page_tokens >> 5;
    auto block_base = [&](int t0) -> size_t {
        const int page = pt[t0 / a.page_tokens];
        const int blk = (t0 % a.page_tokens) >> 5;
        return (((size_t)page * a.n_kv + kvh) * blocks_per_page + blk) * (size_t)(32 * D);
    };

    bf16x8 qf[RT][KS];
    int limit[RT];
#pragma unroll
    for (int rt = 0; rt < RT; ++rt) {
        const int row = rt * 16 + c;
        const int qi = qtile * p.q_per_item + row / n_rep;
        const int hr = row % n_rep;
        const bool used = qtile < p.items_per_unit && (row < p.q_per_item * n_rep) && (qi < u_count);
        limit[rt] = used ? p.causal_pos0 + qi * p.causal_stride : -1;
        const uint16_t *qp = a.q + (((size_t)u_row0 + qi) * a.n_q + kvh * n_rep + hr) * D + 8 * g;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            uint4 raw = make_uint4(0, 0, 0, 0);
            if (used) raw = *(const uint4 *)(qp + ks * 32);
            qf[rt][ks] = __builtin_bit_cast(bf16x8, raw);
        }
    }
    int max_limit = -1, min_limit = 0x7FFFFFFF;      // over the used rows of this wavefront
#pragma unroll
    for (int rt = 0; rt < RT; ++rt) {
        max_limit = max(max_limit, limit[rt]);
        min_limit = min(min_limit, limit[rt] < 0 ? 0x7FFFFFFF : limit[rt]);
    }
#pragma unroll
    for (int off = 1; off < 16; off <<= 1) {
        max_limit = max(max_limit, __shfl_xor(max_limit, off, 64));
        min_limit = min(min_limit, __shfl_xor(min_limit, off, 64));
    }
    // tokens below t_vis are visible to every used row (unused rows hold zero queries and are never written out)
    const int t_vis = __builtin_amdgcn_readfirstlane(min_limit == 0x7FFFFFFF ? 0 : min_limit + 1);
    // this wavefront's range, and the workgroup's: its last query token sees the most
    const int t_hi = __builtin_amdgcn_readfirstlane(min(p.t_end, max_limit + 1));
    const int last_q = min((qg * 4 + 4) * p.q_per_item, u_count) - 1;
    const int t_hi_wg = min(p.t_end, p.causal_pos0 + last_q * p.causal_stride + 1);
    const int n_blocks = (t_hi_wg - p.t_begin + 31) >> 5;          // t_begin is a multiple of 32

    f32x4 o[DT][RT];
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
        for (int rt = 0; rt < RT; ++rt) o[dt][rt] = f32x4{0.f, 0.f, 0.f, 0.f};
    float mrun[RT], lrun[RT];
#pragma unroll
    for (int rt = 0; rt < RT; ++rt) { mrun[rt] = kNegBig; lrun[rt] = 0.f; }
    const float scale_log2 = a.scale * 1.4426950408889634f;

    u32x4 sk[NS], sv[NS];                           // this thread's slots of the block being brought in
    auto fetch = [&](int blk) {
        const size_t base = block_base(p.t_begin + 32 * blk);
        const u32x4 *ksrc = (const u32x4 *)(a.kpool + base), *vsrc = (const u32x4 *)(a.vpool + base);
#pragma unroll
        for (int i = 0; i < NS; ++i) { sk[i] = ksrc[tid + 256 * i]; sv[i] = vsrc[tid + 256 * i]; }
    };
    auto stash = [&](int buf) {
#pragma unroll
        for (int i = 0; i < NS; ++i) { lds[buf][0][tid + 256 * i] = sk[i]; lds[buf][1][tid + 256 * i] = sv[i]; }
    };

    if (n_blocks > 0) {
        fetch(0);
        stash(0);
        __syncthreads();
        if (n_blocks > 1) fetch(1);
    }
    for (int blk = 0; blk < n_blocks; ++blk) {
        const int buf = blk & 1;
        const int t0 = p.t_begin + 32 * blk;
        if (t0 < t_hi) {                            // uniform per wavefront: later blocks are invisible to all its rows
            const u32x4 *kb = lds[buf][0], *vb = lds[buf][1];
            f32x4 s[RT][2];
#pragma unroll
            for (int rt = 0; rt < RT; ++rt)
#pragma unroll
                for (int tt = 0; tt < 2; ++tt) s[rt][tt] = f32x4{0.f, 0.f, 0.f, 0.f};
            // k-steps outermost: 2 x RT independent accumulators take turns, so an MFMA never waits for the one before it
#pragma unroll
            for (int ks = 0; ks < KS; ++ks)
#pragma unroll
                for (int tt = 0; tt < 2; ++tt) {
                    const bf16x8 kf = __builtin_bit_cast(bf16x8, kb[(ks * 32 + tt * 16 + c) * 4 + g]);
#pragma unroll
                    for (int rt = 0; rt < RT; ++rt)
                        s[rt][tt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf, qf[rt][ks], s[rt][tt], 0, 0, 0);
                }
            bf16x8 pf[RT];
            float alpha[RT];
            // Online softmax.  A block that every used row sees entirely (all but the last one or two of a range)
            // skips the per-token visibility tests; the exponentials are the hardware's base-2 exponential as it is
            // (arguments <= 0; results below 2^-126 of the row maximum may flush to zero).
            auto softmax = [&](auto masked) __attribute__((always_inline)) {
                constexpr bool MASKED = decltype(masked)::value;
#pragma unroll
                for (int rt = 0; rt < RT; ++rt) {
                    const int lim = min(limit[rt], t_hi - 1);
                    float bmax = kNegBig;
                    bool ok[2][4];
#pragma unroll
                    for (int tt = 0; tt < 2; ++tt)
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            ok[tt][e] = !MASKED || (t0 + tt * 16 + 4 * g + e) <= lim;
                            s[rt][tt][e] = ok[tt][e] ? s[rt][tt][e] * scale_log2 : kNegBig;
                            bmax = fmaxf(bmax, s[rt][tt][e]);
                        }
                    bmax = fmaxf(bmax, __shfl_xor(bmax, 16, 64));
                    bmax = fmaxf(bmax, __shfl_xor(bmax, 32, 64));
                    const float mnew = fmaxf(mrun[rt], bmax);
                    alpha[rt] = __builtin_amdgcn_exp2f(mrun[rt] - mnew);
                    mrun[rt] = mnew;
                    float psum = 0.f;
                    float pv[8];
#pragma unroll
                    for (int tt = 0; tt < 2; ++tt)
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            const float pe = ok[tt][e] ? __builtin_amdgcn_exp2f(s[rt][tt][e] - mnew) : 0.f;
                            pv[tt * 4 + e] = pe;
                            psum += pe;
                        }
                    lrun[rt] = lrun[rt] * alpha[rt] + psum;
                    const uint4 praw = make_uint4(pack_bf16x2(pv[0], pv[1]), pack_bf16x2(pv[2], pv[3]),
                                                  pack_bf16x2(pv[4], pv[5]), pack_bf16x2(pv[6], pv[7]));
                    pf[rt] = __builtin_bit_cast(bf16x8, praw);
                }
            };
            if (t0 + 32 <= t_vis && t0 + 32 <= t_hi) softmax(std::false_type{});
            else softmax(std::true_type{});
            // the accumulators are rescaled only when some row's maximum moved (after the first blocks it rarely does)
            bool moved = false;
#pragma unroll
            for (int rt = 0; rt < RT; ++rt) moved |= alpha[rt] != 1.0f;
            const bool rescale = __any(moved);
#pragma unroll
            for (int dt = 0; dt < DT; ++dt) {
                const bf16x8 vf = __builtin_bit_cast(bf16x8, vb[(dt * 16 + c) * 4 + g]);
#pragma unroll
                for (int rt = 0; rt < RT; ++rt) {
                    if (rescale) o[dt][rt] *= alpha[rt];
                    o[dt][rt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf, pf[rt], o[dt][rt], 0, 0, 0);
                }
            }
        }
        if (blk + 1 < n_blocks) stash(buf ^ 1);     // the other buffer was last read before the previous barrier
        __syncthreads();
        if (blk + 2 < n_blocks) fetch(blk + 2);
    }

#pragma unroll
    for (int rt = 0; rt < RT; ++rt) {
        float l = lrun[rt];
        l += __shfl_xor(l, 16, 64);
        l += __shfl_xor(l, 32, 64);
        if (limit[rt] < 0) continue;
        const int row = rt * 16 + c;
        const size_t qtok = (size_t)u_row0 + qtile * p.q_per_item + row / n_rep;
        const int col = (kvh * n_rep + row % n_rep) * D + 4 * g;
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) {
            float r[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) r[e] = l > 0.f ? o[dt][rt][e] / l : 0.f;
            *(uint2 *)(a.direct_out + frag_offset((int)qtok, col + dt * 16, a.out_mt_total)) =
                make_uint2(pack_bf16x2(r[0], r[1]), pack_bf16x2(r[2], r[3]));
        }
    }
}

struct MergeArgs {
    AttnPhase ph[2];
    int n_phases;
    int n_q, n_kv, d, mt_total;
    uint16_t *out;
    float *out32;       // non-null: row-major fp32 output instead of `out`
};

// One block per (query token, query head); thread = head dimension.  The rows of all partial results are
// worked out first; then the (max, sum) pairs, one per thread, and the first four partial outputs of every
// thread are fetched in the same round trip, the pairs are turned into weights, and the weighted sum runs
// over the items in a fixed order.
constexpr int kMaxMergeItems = 64;

__global__ __launch_bounds__(128) void attn_merge_kernel(MergeArgs a) {
    __shared__ float s_m[kMaxMergeItems], s_l[kMaxMergeItems], s_w[kMaxMergeItems];
    __shared__ unsigned s_row[kMaxMergeItems];      // partial-result row of each item
    __shared__ const float *s_ml[kMaxMergeItems];   // its (max, sum) pair
    const int qt = blockIdx.x, h = blockIdx.y, dd = threadIdx.x;
    const int n_rep = a.n_q / a.n_kv;
    const int kvh = h / n_rep, hr = h % n_rep;

    int n_items = 0;
    for (int ph = 0; ph < a.n_phases; ++ph) {
        const AttnPhase &p = a.ph[ph];
        const int unit = p.row_unit ? p.row_unit[qt] : qt / p.q_per_unit;
        const int qi = p.row_unit ? qt - p.unit_row0[unit] : qt % p.q_per_unit;
        const int qtile = qi / p.q_per_item, row = (qi % p.q_per_item) * n_rep + hr;
        const size_t item0 = ((size_t)unit * a.n_kv + kvh) * p.n_splits;
        if (dd < p.n_splits) {
            const size_t prow = ((item0 + dd) * p.items_per_unit + qtile) * (16 * p.rt) + row;
            const size_t base = (size_t)(p.part_o - a.ph[0].part_o) / a.d;   // phases share one buffer
            s_row[n_items + dd] = (unsigned)(base + prow);
            s_ml[n_items + dd] = p.part_ml + prow * 2;
        }
        n_items += p.n_splits;
    }
    __syncthreads();
    const float *po = a.ph[0].part_o + (dd < a.d ? dd : 0);
    float v[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) v[u] = u < n_items ? po[(size_t)s_row[u] * a.d] : 0.f;
    if (dd < n_items) {
        const float2 ml = *(const float2 *)s_ml[dd];
        s_m[dd] = ml.x;
        s_l[dd] = ml.y;
    }
    __syncthreads();
    float mbest = kNegBig;
    for (int i = 0; i < n_items; ++i)
        if (s_l[i] > 0.f) mbest = fmaxf(mbest, s_m[i]);
    float den = 0.f;
    for (int i = 0; i < n_items; ++i) {
        const float w = s_l[i] > 0.f ? exp2f(s_m[i] - mbest) : 0.f;
        den += s_l[i] * w;
        if (dd == 0) s_w[i] = w;
    }
    __syncthreads();
    if (dd >= a.d) return;
    float num = 0.f;
#pragma unroll
    for (int u = 0; u < 4; ++u)
        if (u < n_items) num += v[u] * s_w[u];
    int i = 4;
    for (; i + 4 <= n_items; i += 4) {
#pragma unroll
        for (int u = 0; u < 4; ++u) v[u] = po[(size_t)s_row[i + u] * a.d];
#pragma unroll
        for (int u = 0; u < 4; ++u) num += v[u] * s_w[i + u];
    }
    for (; i < n_items; ++i) num += po[(size_t)s_row[i] * a.d] * s_w[i];
    const float r = den > 0.f ? num / den : 0.f;
    if (a.out32) a.out32[((size_t)qt * a.n_q + h) * a.d + dd] = r;
    else a.out[frag_offset(qt, h * a.d + dd, a.mt_total)] = f32_to_bf16(r);
}

}  // namespace

int launch_attention(const AttnArgs &a, const AttnPhase *phases, int n_phases, hipStream_t stream) {
    if (n_phases < 1 || n_phases > 2) return SR_E_ARG;
    long long n[2] = {0, 0};
    const int n_rep = a.n_q / a.n_kv;
    for (int i = 0; i < n_phases; ++i) {
        const AttnPhase &p = phases[i];
        n[i] = (long long)p.n_units * a.n_kv * p.items_per_unit * p.n_splits;
        if (p.t_end <= p.t_begin) n[i] = 0;
        if ((p.t_begin & 31) || (p.split_tokens & 31) || p.split_tokens <= 0 || p.q_per_item * n_rep > 16 * p.rt ||
            p.rt != phases[0].rt)
            return SR_E_ARG;
    }
    if (a.direct_out && (n_phases != 1 || phases[0].n_splits != 1)) return SR_E_ARG;
    const long long n_items = n[0] + n[1];
    if (n_items <= 0) return SR_OK;
    if (n_items > 0x7FFFFFFF) return SR_E_ARG;
    const AttnPhase &p0 = phases[0], &p1 = phases[n_phases - 1];
    const int rt = p0.rt, n0 = (int)n[0], nt = (int)n_items;
    if (a.direct_out && p0.items_per_unit >= 2) {
        // prefill: the query tiles of a (unit, kv head) share their K/V blocks through LDS, four to a workgroup
        const long long wgs = (long long)p0.n_units * a.n_kv * ((p0.items_per_unit + 3) / 4);
        if (wgs > 0x7FFFFFFF) return SR_E_ARG;
        dim3 sgrid((unsigned)wgs);
        if (a.d == 128 && rt == 1) attn_prefill_shared_kernel<128, 1><<<sgrid, dim3(256), 0, stream>>>(a, p0);
        else if (a.d == 128 && rt == 2) attn_prefill_shared_kernel<128, 2><<<sgrid, dim3(256), 0, stream>>>(a, p0);
        else if (a.d == 64 && rt == 1) attn_prefill_shared_kernel<64, 1><<<sgrid, dim3(256), 0, stream>>>(a, p0);
        else if (a.d == 64 && rt == 2) attn_prefill_shared_kernel<64, 2><<<sgrid, dim3(256), 0, stream>>>(a, p0);
        else return SR_E_ARG;
        SR_HIP(hipGetLastError());
        return SR_OK;
    }
    dim3 grid((unsigned)((n_items + 3) / 4)), block(256);
    if (a.d == 128 && rt == 1) attn_kernel<128, 1><<<grid, block, 0, stream>>>(a, p0, p1, n0, nt);
    else if (a.d == 128 && rt == 2) attn_kernel<128, 2><<<grid, block, 0, stream>>>(a, p0, p1, n0, nt);
    else if (a.d == 64 && rt == 1) attn_kernel<64, 1><<<grid, block, 0, stream>>>(a, p0, p1, n0, nt);
    else if (a.d == 64 && rt == 2) attn_kernel<64, 2><<<grid, block, 0, stream>>>(a, p0, p1, n0, nt);
    else return SR_E_ARG;
    SR_HIP(hipGetLastError());
    return SR_OK;
}

int launch_attn_merge(const AttnArgs &a, const AttnPhase *phases, int n_phases, int n_qtok, uint4 *out,
                      int mt_total, float *out32, hipStream_t stream) {
    if (n_qtok <= 0) return SR_OK;
    if (n_phases < 1 || n_phases > 2) return SR_E_ARG;
    int total = 0;
    for (int i = 0; i < n_phases; ++i) total += phases[i].n_splits;
    if (total > kMaxMergeItems) return SR_E_ARG;
    MergeArgs m{};
    for (int i = 0; i < n_phases; ++i) m.ph[i] = phases[i];
    m.n_phases = n_phases;
    m.n_q = a.n_q; m.n_kv = a.n_kv; m.d = a.d; m.mt_total = mt_total;
    m.out = (uint16_t *)out;
    m.out32 = out32;
    attn_merge_kernel<<<dim3(n_qtok, a.n_q), dim3(128), 0, stream>>>(m);
    SR_HIP(hipGetLastError());
    return SR_OK;
}

}  // namespace sr
