// In-group divergence signals at step K (paper Appendix B) and the two-clause gate (Appendix E,
// Eq. 3), for groups whose members may have finished before step K.
//
// Member i finished after end_step[i] environment steps, so at step K it contributes the prefix
// a_i[0 : len_i], len_i = min(K, end_step[i]).  Per group and per requested K the kernel produces
//   - d_K: the mean over pairs of the prefix edit distance divided by the longer of the two prefix
//     lengths (Section 3.2), as a double and exactly, in units of 1 / lcm(1..32);
//   - the action-bigram Jaccard distance, the distinct-prefix count, the distinct step-K action and
//     observation counts, the step-K action entropy and the number of finished members;
//   - the decisions  d_K < d_L  (Eq. 2) and  d_K < d_L or tau_K >= tau_H  (Eq. 3) in integers.
//
// Work decomposition, as for the equal-length gate: one lane owns one pair and keeps both
// sequences and the current table row in registers.  Cell (r, c) of the table of two sequences
// is the distance of their prefixes of lengths r and c, so one table serves every requested K:
// the lane picks cell (len_i, len_j) when row len_i is complete.  Bigram sets need no second pass
// per K either: a bigram position is the first occurrence of its bigram in every prefix that
// contains it, so the lane computes once a bit mask of first occurrences per sequence and, per
// position of a, the mask of positions of b holding the same bigram; each K is then a few mask
// operations.  Lanes leave five small integers per (K, pair) in LDS; one thread per (K, group)
// turns them into the outputs, adding the pair terms in pair order (i, j), i < j, so that the
// floating-point results do not depend on scheduling.
#include "sr_internal.h"

static_assert(sizeof(sr_signals_t) == 64, "sr_signals_t is part of the C boundary");

namespace sr {
namespace {

constexpr int kSigThreads = 256;
constexpr int kSigLdsInts = 4096;
constexpr int kSigMaxLens = 8;
constexpr long long kLcm32 = 144403552893600LL;      // lcm(1..32)

struct SigLens {
    int n;
    int len[kSigMaxLens];
    long long d_bound;                // d_K < d_L  <=>  lev_scaled < d_bound
    long long tau_num;                // tau_K >= tau_H  <=>  n_done * 1e6 >= tau_num * G
};

struct PairRec {                       // what a pair lane leaves for one K
    uint8_t lev, longer, inter, uni, same;
};

template <int KMAX>
__global__ __launch_bounds__(kSigThreads) void signals_kernel(
    const int32_t *__restrict__ actions, const int32_t *__restrict__ obs, const int32_t *__restrict__ end_step,
    int n_groups, int G, int stride, int pairs, int groups_per_block, SigLens lens, sr_signals_t *__restrict__ out) {
    __shared__ int32_t s_act[kSigLdsInts];                    // [groups_per_block][G][KMAX]
    __shared__ int32_t s_obs[kSigMaxLens][kSigThreads];       // [K index][group in block * G + member]: o_{i,K}
    __shared__ int32_t s_end[kSigThreads];                    // [group in block * G + member]
    __shared__ PairRec s_pair[kSigMaxLens][kSigThreads];      // [K index][group in block * pairs + pair]

    const int tid = threadIdx.x;
    const int g0 = blockIdx.x * groups_per_block;
    const int n_here = min(groups_per_block, n_groups - g0);
    const int rows = n_here * G;

    // stage the first KMAX actions of every member (columns past the stride are never part of a prefix)
    for (int i = tid; i < rows * KMAX; i += kSigThreads) {
        const int r = i / KMAX, c = i - r * KMAX;
        s_act[i] = (c < stride) ? actions[((size_t)g0 * G + r) * stride + c] : -1 - c;
    }
    for (int i = tid; i < rows; i += kSigThreads) {
        s_end[i] = end_step ? max(end_step[(size_t)g0 * G + i], 0) : 0x7FFFFFFF;
        for (int l = 0; l < lens.n; ++l)
            s_obs[l][i] = obs ? obs[((size_t)g0 * G + i) * stride + lens.len[l] - 1] : 0;
    }
    __syncthreads();

    const int gl = tid / pairs;                       // group within the block
    if (gl < n_here) {
        int p = tid - gl * pairs, i = 0;              // pair index -> (i, j), i < j
        while (p >= G - 1 - i) { p -= G - 1 - i; ++i; }
        const int j = i + 1 + p;
        int32_t a[KMAX], b[KMAX];
        const int32_t *sa = s_act + (gl * G + i) * KMAX, *sb = s_act + (gl * G + j) * KMAX;
#pragma unroll
        for (int c = 0; c < KMAX; ++c) { a[c] = sa[c]; b[c] = sb[c]; }
        const int ei = s_end[gl * G + i], ej = s_end[gl * G + j];

        int li[kSigMaxLens], lj[kSigMaxLens];
        unsigned res[kSigMaxLens];
        int maxlen = 0;
#pragma unroll
        for (int l = 0; l < kSigMaxLens; ++l) {
            const int K = l < lens.n ? lens.len[l] : 0;
            li[l] = min(K, ei);
            lj[l] = min(K, ej);
            res[l] = (unsigned)lj[l];                 // row 0 of the table: distance from the empty prefix
            maxlen = max(maxlen, K);
        }

        // edit-distance table, one row at a time; cell (len_i, len_j) is picked when row len_i is complete
        unsigned row[KMAX + 1];
#pragma unroll
        for (int c = 0; c <= KMAX; ++c) row[c] = c;
#pragma unroll
        for (int r = 1; r <= KMAX; ++r) {
            if (r <= maxlen) {                        // uniform across the workgroup
                unsigned diag = row[0];
                row[0] = r;
#pragma unroll
                for (int c = 1; c <= KMAX; ++c) {
                    const unsigned up = row[c];
                    row[c] = min(min(diag + (a[r - 1] != b[c - 1] ? 1u : 0u), up + 1u), row[c - 1] + 1u);
                    diag = up;
                }
#pragma unroll
                for (int l = 0; l < kSigMaxLens; ++l)
                    if (li[l] == r) {
                        unsigned v = row[0];
#pragma unroll
                        for (int c = 1; c <= KMAX; ++c) v = (lj[l] == c) ? row[c] : v;
                        res[l] = v;
                    }
            }
        }

        // bigram t = (x[t], x[t+1]), t = 0 .. KMAX-2.  first_x: positions holding the first occurrence of
        // their bigram in x; in_b[t]: positions of b whose bigram equals bigram t of a.
        unsigned first_a = 0, first_b = 0, in_b[KMAX - 1];
#pragma unroll
        for (int t = 0; t < KMAX - 1; ++t) {
            bool seen_a = false, seen_b = false;
            unsigned m = 0;
#pragma unroll
            for (int u = 0; u < KMAX - 1; ++u) {
                if (u < t) {
                    seen_a |= (a[u] == a[t]) & (a[u + 1] == a[t + 1]);
                    seen_b |= (b[u] == b[t]) & (b[u + 1] == b[t + 1]);
                }
                m |= ((b[u] == a[t]) & (b[u + 1] == a[t + 1])) ? (1u << u) : 0u;
            }
            first_a |= seen_a ? 0u : (1u << t);
            first_b |= seen_b ? 0u : (1u << t);
            in_b[t] = m;
        }

        for (int l = 0; l < lens.n; ++l) {
            // a prefix of length n holds bigram positions 0 .. n-2
            const unsigned ma = li[l] >= 2 ? (0xFFFFFFFFu >> (33 - li[l])) : 0u;
            const unsigned mb = lj[l] >= 2 ? (0xFFFFFFFFu >> (33 - lj[l])) : 0u;
            const int na = __popc(first_a & ma), nb = __popc(first_b & mb);
            int inter = 0;
#pragma unroll
            for (int t = 0; t < KMAX - 1; ++t) inter += (((first_a & ma) >> t) & 1u) & ((in_b[t] & mb) != 0u ? 1u : 0u);
            PairRec rec;
            rec.lev = (uint8_t)res[l];
            rec.longer = (uint8_t)max(li[l], lj[l]);
            rec.inter = (uint8_t)inter;
            rec.uni = (uint8_t)(na + nb - inter);
            rec.same = (uint8_t)(li[l] == lj[l] && res[l] == 0u);
            s_pair[l][tid] = rec;
        }
    }
    __syncthreads();

    // one thread per (K, group): pair terms in pair order, then the per-member counts
    for (int w = tid; w < lens.n * n_here; w += kSigThreads) {
        const int l = w / n_here, g = w - l * n_here;
        const int K = lens.len[l];
        const PairRec *pr = &s_pair[l][g * pairs];
        double dsum = 0.0, jsum = 0.0;
        long long scaled = 0;
        int lev_sum = 0;
        for (int q = 0; q < pairs; ++q) {
            const PairRec r = pr[q];
            lev_sum += r.lev;
            if (r.longer > 0) {
                dsum += (double)r.lev / (double)r.longer;
                scaled += (long long)r.lev * (kLcm32 / r.longer);
            }
            jsum += r.uni > 0 ? 1.0 - (double)r.inter / (double)r.uni : 0.0;
        }
        // member j repeats an earlier prefix iff some pair (i, j), i < j, is marked `same`
        int uniq = 0, n_at = 0, ua = 0, uo = 0, n_done = 0;
        double H = 0.0;
        const int32_t *acts = s_act + g * G * KMAX;
        const int32_t *ends = s_end + g * G;
        const int32_t *ob = &s_obs[l][g * G];
        for (int j = 0; j < G; ++j) n_at += min(K, ends[j]) == K ? 1 : 0;
        for (int j = 0; j < G; ++j) {
            bool dup = false;
            for (int i = 0; i < j; ++i) {
                const int q = i * G - i * (i + 1) / 2 + (j - i - 1);     // index of pair (i, j)
                dup |= pr[q].same != 0;
            }
            uniq += dup ? 0 : 1;
            n_done += ends[j] <= K ? 1 : 0;
            if (min(K, ends[j]) != K) continue;
            const int32_t aj = acts[j * KMAX + K - 1];
            bool first_act = true, first_obs = true;
            int count = 0;
            for (int i = 0; i < G; ++i) {
                if (min(K, ends[i]) != K) continue;
                const bool same_a = acts[i * KMAX + K - 1] == aj;
                count += same_a ? 1 : 0;
                if (i < j && same_a) first_act = false;
                if (i < j && ob[i] == ob[j]) first_obs = false;
            }
            if (first_act) {
                ++ua;
                const double pj = (double)count / (double)n_at;
                H -= pj * log(pj);
            }
            if (first_obs) ++uo;
        }
        sr_signals_t o;
        const double P = (double)pairs;
        o.d_K = dsum / P;
        o.lev_scaled = scaled;
        o.bigram_jaccard = jsum / P;
        o.action_entropy = H;
        o.unique_prefix = uniq;
        o.n_at_step = n_at;
        o.unique_action = ua;
        o.unique_obs = obs ? uo : 0;
        o.n_done = n_done;
        o.lev_sum = lev_sum;
        o.cut_d = (uint8_t)(scaled < lens.d_bound);
        o.cut_or = (uint8_t)(o.cut_d || (long long)n_done * 1000000LL >= lens.tau_num * G);
        for (int i = 0; i < 6; ++i) o.reserved[i] = 0;
        out[(size_t)l * n_groups + g0 + g] = o;
    }
}

__global__ void assemble_gate_kernel(const int32_t *__restrict__ src, const int32_t *__restrict__ live_actions,
                                     const int32_t *__restrict__ fin_actions, int n_slots, int max_turns,
                                     int32_t *__restrict__ out) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n_slots * max_turns) return;
    const int s = i / max_turns, t = i - s * max_turns;
    const int r = src[s];
    out[i] = r >= 0 ? live_actions[(size_t)r * max_turns + t] : fin_actions[(size_t)(-1 - r) * max_turns + t];
}

__global__ void extract_gate_kernel(const sr_signals_t *__restrict__ sig, int n_groups, int use_or,
                                    int32_t *__restrict__ sums, uint8_t *__restrict__ retire) {
    const int g = blockIdx.x * blockDim.x + threadIdx.x;
    if (g >= n_groups) return;
    sums[g] = sig[g].lev_sum;
    retire[g] = use_or ? sig[g].cut_or : sig[g].cut_d;
}

}  // namespace

int launch_assemble_gate(const int32_t *src, const int32_t *live_actions, const int32_t *fin_actions, int n_slots,
                         int max_turns, int32_t *out, hipStream_t stream) {
    const int n = n_slots * max_turns;
    if (n <= 0) return SR_OK;
    assemble_gate_kernel<<<dim3((n + 255) / 256), dim3(256), 0, stream>>>(src, live_actions, fin_actions, n_slots,
                                                                         max_turns, out);
    SR_HIP(hipGetLastError());
    return SR_OK;
}

int launch_extract_gate(const sr_signals_t *sig, int n_groups, int use_or, int32_t *sums, uint8_t *retire,
                        hipStream_t stream) {
    if (n_groups <= 0) return SR_OK;
    extract_gate_kernel<<<dim3((n_groups + 255) / 256), dim3(256), 0, stream>>>(sig, n_groups, use_or, sums, retire);
    SR_HIP(hipGetLastError());
    return SR_OK;
}

}  // namespace sr

extern "C" int sr_signals_batch(const int32_t *actions, const int32_t *obs, const int32_t *end_step, int n_groups,
                                int G, int stride, const int *prefix_lens, int n_lens, double d_L, double tau_H,
                                sr_signals_t *out, void *stream) {
    using namespace sr;
    if (!prefix_lens || n_groups < 0 || G < 2 || G > 16 || stride < 1 || n_lens < 1 || n_lens > kSigMaxLens ||
        !(d_L >= 0.0) || d_L > 1.0 || !(tau_H >= 0.0) || tau_H > 4.0)
        return SR_E_ARG;
    if (n_groups > 0 && (!actions || !out)) return SR_E_ARG;
    SigLens lens{};
    lens.n = n_lens;
    int maxlen = 0;
    for (int l = 0; l < n_lens; ++l) {
        const int K = prefix_lens[l];
        if (K < 1 || K > 32 || K > stride) return SR_E_ARG;
        lens.len[l] = K;
        maxlen = K > maxlen ? K : maxlen;
    }
    // d_K < d_L  <=>  lev_scaled * 1e6 < num * P * lcm  <=>  lev_scaled < ceil(num * P * lcm / 1e6)
    const __int128 num = (__int128)__builtin_llround(d_L * 1e6), P = (__int128)G * (G - 1) / 2;
    lens.d_bound = (long long)((num * P * (__int128)kLcm32 + 999999) / 1000000);
    lens.tau_num = (long long)__builtin_llround(tau_H * 1e6);
    if (n_groups == 0) return SR_OK;
    const int pairs = G * (G - 1) / 2;
    const int kmax = maxlen <= 8 ? 8 : maxlen <= 16 ? 16 : maxlen <= 24 ? 24 : 32;
    int gpb = kSigThreads / pairs;
    if (gpb > kSigLdsInts / (G * kmax)) gpb = kSigLdsInts / (G * kmax);
    if (gpb > kSigThreads / G) gpb = kSigThreads / G;         // per-member staging arrays hold 256 entries
    if (gpb < 1) return SR_E_ARG;
    dim3 grid((n_groups + gpb - 1) / gpb), block(kSigThreads);
    hipStream_t st = (hipStream_t)stream;
    switch (kmax) {
        case 8:  signals_kernel<8><<<grid, block, 0, st>>>(actions, obs, end_step, n_groups, G, stride, pairs, gpb, lens, out); break;
        case 16: signals_kernel<16><<<grid, block, 0, st>>>(actions, obs, end_step, n_groups, G, stride, pairs, gpb, lens, out); break;
        case 24: signals_kernel<24><<<grid, block, 0, st>>>(actions, obs, end_step, n_groups, G, stride, pairs, gpb, lens, out); break;
        default: signals_kernel<32><<<grid, block, 0, st>>>(actions, obs, end_step, n_groups, G, stride, pairs, gpb, lens, out); break;
    }
    SR_HIP(hipGetLastError());
    return SR_OK;
}
