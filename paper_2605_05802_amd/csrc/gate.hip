// Selective-Rollout gate: mean pairwise prefix edit distance of a group's action sequences
// (paper Section 3.2) compared with the threshold d_L (Eq. 2), in exact integer arithmetic.
//
// Work decomposition.  The work is G(G-1)/2 independent Levenshtein tables per group and is
// bound by integer ALU throughput, not by memory (a group is G*K*4 bytes in, 5 bytes out).
// One lane owns one pair and runs the whole dynamic programme for it, row by row, with the
// current table row and both sequences held in registers; all loops are unrolled, so there
// is no cross-lane traffic and every active lane does useful work on every instruction.
// (Spreading one table over the lanes of an anti-diagonal leaves half of the lanes idle in
// the triangular ramp-up and ramp-down and pays an LDS round trip per diagonal.)
// A 256-thread workgroup serves floor(256 / pairs) whole groups; their sequences are staged
// once through LDS and the per-group sums are accumulated with LDS integer atomics, which
// are order-independent and therefore deterministic.
//
// Prefix nesting: cell (k,k) of the table of two length-Kmax sequences is the distance of
// their length-k prefixes, so one table serves every requested prefix length.
#include "sr_internal.h"

namespace sr {

int64_t gate_bound(double d_L, int G, int K) {
    const int64_t den = 1000000;
    const int64_t num = (int64_t)__builtin_llround(d_L * 1e6);
    const int64_t pairs = (int64_t)G * (G - 1) / 2;
    return (num * pairs * (int64_t)K + den - 1) / den;
}

namespace {

constexpr int kGateThreads = 256;
constexpr int kGateLdsInts = 4096;

__device__ __forceinline__ unsigned min3u(unsigned a, unsigned b, unsigned c) {
    return min(a, min(b, c));
}

template <int KMAX>
__global__ __launch_bounds__(kGateThreads) void gate_kernel(
    const int32_t *__restrict__ actions, int n_groups, int G, int stride, int pairs,
    int groups_per_block, GateLens lens, int32_t *__restrict__ sums, uint8_t *__restrict__ retire) {
    __shared__ int32_t s_act[kGateLdsInts];          // [groups_per_block][G][KMAX]
    __shared__ int s_sum[8][kGateThreads];           // [len index][group in block]

    const int tid = threadIdx.x;
    const int g0 = blockIdx.x * groups_per_block;
    const int n_here = min(groups_per_block, n_groups - g0);

    for (int i = tid; i < 8 * kGateThreads; i += kGateThreads) (&s_sum[0][0])[i] = 0;
    // stage the first KMAX actions of every member (pad with distinct negative ids: never compared,
    // because no requested prefix reaches a padded column)
    const int rows = n_here * G;
    for (int i = tid; i < rows * KMAX; i += kGateThreads) {
        const int r = i / KMAX, c = i - r * KMAX;
        s_act[i] = (c < stride) ? actions[((size_t)g0 * G + r) * stride + c] : -1 - c;
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

        int maxlen = 0;
        for (int l = 0; l < lens.n; ++l) maxlen = max(maxlen, lens.len[l]);

        unsigned row[KMAX + 1];
        unsigned res[8];
#pragma unroll
        for (int l = 0; l < 8; ++l) res[l] = 0;
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
                    row[c] = min3u(diag + (a[r - 1] != b[c - 1] ? 1u : 0u), up + 1u, row[c - 1] + 1u);
                    diag = up;
                }
#pragma unroll
                for (int l = 0; l < 8; ++l)
                    if (l < lens.n && lens.len[l] == r) res[l] = row[r];
            }
        }
        for (int l = 0; l < lens.n; ++l) atomicAdd(&s_sum[l][gl], (int)res[l]);
    }
    __syncthreads();

    for (int i = tid; i < lens.n * n_here; i += kGateThreads) {
        const int l = i / n_here, g = i - l * n_here;
        const int s = s_sum[l][g];
        if (sums) sums[(size_t)l * n_groups + g0 + g] = s;
        if (retire) retire[(size_t)l * n_groups + g0 + g] = (uint8_t)(s < lens.bound[l]);
    }
}

// ---------------------------------------------------------------------------------------------
// The other decomposition, kept for comparison: one workgroup per group, every pair's table advanced
// one anti-diagonal at a time by a segment of SEG lanes (lane i owns row i of the table), the last
// three anti-diagonals of every pair in LDS.  256 / SEG pairs advance together; with G = 8 the 28
// pairs take two passes at SEG = 16 and four at SEG = 32.  Cell (k, k), the distance of the two
// length-k prefixes, appears on anti-diagonal 2k in lane k.  A segment never straddles a wavefront,
// and a wavefront's LDS accesses complete in program order, so no workgroup barrier is needed
// between anti-diagonals.  Half of a segment's lanes are idle in the triangular ramp-up and
// ramp-down and every step is an LDS round trip, which is why the lane-per-pair kernel above is the
// one the library uses; sr_gate_batch_antidiag exposes this one so that the two can be measured
// side by side and checked against each other.
// ---------------------------------------------------------------------------------------------
template <int SEG>
__global__ __launch_bounds__(kGateThreads) void gate_antidiag_kernel(
    const int32_t *__restrict__ actions, int n_groups, int G, int stride, int pairs, int maxlen, GateLens lens,
    int32_t *__restrict__ sums, uint8_t *__restrict__ retire) {
    constexpr int kSlots = kGateThreads / SEG;             // pairs that advance together
    __shared__ int32_t s_act[16 * SEG];                      // [member][step], the first SEG steps
    __shared__ unsigned s_d[3][kSlots][SEG + 1];             // anti-diagonals d-2, d-1, d of every slot, by table row
    __shared__ int s_sum[8];

    const int tid = threadIdx.x, g = blockIdx.x;
    if (tid < 8) s_sum[tid] = 0;
    for (int i = tid; i < G * SEG; i += kGateThreads) {
        const int r = i / SEG, c = i - r * SEG;
        s_act[i] = (c < stride) ? actions[((size_t)g * G + r) * stride + c] : -1 - c;
    }
    __syncthreads();

    const int slot = tid / SEG, row = tid % SEG + 1;         // this lane owns table row `row` (1-based)
    for (int p0 = 0; p0 < pairs; p0 += kSlots) {
        int p = p0 + slot;
        const bool live = p < pairs;
        int mi = 0;
        if (live) while (p >= G - 1 - mi) { p -= G - 1 - mi; ++mi; }
        const int mj = live ? mi + 1 + p : 1;
        const int32_t a_row = s_act[mi * SEG + row - 1];     // a[row - 1]
        const int32_t *b = s_act + mj * SEG;
        // anti-diagonal 0: D[0][0] = 0; anti-diagonal 1: D[0][1] = D[1][0] = 1
        if (row == 1) { s_d[0][slot][0] = 0; s_d[1][slot][0] = 1; s_d[1][slot][1] = 1; }
        __builtin_amdgcn_wave_barrier();
        for (int d = 2; d <= 2 * maxlen; ++d) {
            const unsigned *prev2 = s_d[(d - 2) % 3][slot], *prev = s_d[(d - 1) % 3][slot];
            unsigned *cur = s_d[d % 3][slot];
            const int col = d - row;                         // this lane's cell is (row, col)
            if (row <= maxlen) {
                if (col == 0) {
                    cur[row] = (unsigned)row;                // first column of the table
                } else if (col >= 1 && col <= maxlen) {
                    const unsigned v = min3u(prev2[row - 1] + (a_row != b[col - 1] ? 1u : 0u), prev[row - 1] + 1u,
                                             prev[row] + 1u);
                    cur[row] = v;
                    if (live && col == row) {                // cell (k, k): the answer for prefix length k
#pragma unroll
                        for (int l = 0; l < 8; ++l)
                            if (l < lens.n && lens.len[l] == row) atomicAdd(&s_sum[l], (int)v);
                    }
                }
            }
            if (row == 1 && d <= maxlen) cur[0] = (unsigned)d;   // first row of the table
            __builtin_amdgcn_wave_barrier();
        }
    }
    __syncthreads();
    if (tid < lens.n) {
        const int sum = s_sum[tid];
        if (sums) sums[(size_t)tid * n_groups + g] = sum;
        if (retire) retire[(size_t)tid * n_groups + g] = (uint8_t)(sum < lens.bound[tid]);
    }
}

}  // namespace

int launch_gate_antidiag(const int32_t *actions, int n_groups, int G, int stride, const GateLens &lens,
                         int32_t *sums, uint8_t *retire, hipStream_t stream) {
    if (n_groups <= 0) return SR_OK;
    int maxlen = 0;
    for (int l = 0; l < lens.n; ++l) maxlen = lens.len[l] > maxlen ? lens.len[l] : maxlen;
    const int pairs = G * (G - 1) / 2;
    dim3 grid(n_groups), block(kGateThreads);
    if (maxlen <= 16)
        gate_antidiag_kernel<16><<<grid, block, 0, stream>>>(actions, n_groups, G, stride, pairs, maxlen, lens, sums, retire);
    else
        gate_antidiag_kernel<32><<<grid, block, 0, stream>>>(actions, n_groups, G, stride, pairs, maxlen, lens, sums, retire);
    SR_HIP(hipGetLastError());
    return SR_OK;
}

int launch_gate(const int32_t *actions, int n_groups, int G, int stride, const GateLens &lens,
                int32_t *sums, uint8_t *retire, hipStream_t stream) {
    if (n_groups <= 0) return SR_OK;
    int maxlen = 0;
    for (int l = 0; l < lens.n; ++l) maxlen = lens.len[l] > maxlen ? lens.len[l] : maxlen;
    const int pairs = G * (G - 1) / 2;
    const int kmax = maxlen <= 8 ? 8 : maxlen <= 16 ? 16 : maxlen <= 24 ? 24 : 32;
    int gpb = kGateThreads / pairs;
    const int lds_cap = kGateLdsInts / (G * kmax);
    if (gpb > lds_cap) gpb = lds_cap;
    if (gpb < 1) return SR_E_ARG;
    const int blocks = (n_groups + gpb - 1) / gpb;
    dim3 grid(blocks), block(kGateThreads);
    switch (kmax) {
        case 8:  gate_kernel<8><<<grid, block, 0, stream>>>(actions, n_groups, G, stride, pairs, gpb, lens, sums, retire); break;
        case 16: gate_kernel<16><<<grid, block, 0, stream>>>(actions, n_groups, G, stride, pairs, gpb, lens, sums, retire); break;
        case 24: gate_kernel<24><<<grid, block, 0, stream>>>(actions, n_groups, G, stride, pairs, gpb, lens, sums, retire); break;
        default: gate_kernel<32><<<grid, block, 0, stream>>>(actions, n_groups, G, stride, pairs, gpb, lens, sums, retire); break;
    }
    SR_HIP(hipGetLastError());
    return SR_OK;
}

}  // namespace sr

extern "C" int sr_gate_batch(const int32_t *actions, int n_groups, int G, int stride,
                             const int *prefix_lens, int n_lens, double threshold, int32_t *sums,
                             uint8_t *retire, void *stream) {
    if (!actions || !prefix_lens || n_groups < 0 || G < 2 || G > 16 || stride < 1 || n_lens < 1 ||
        n_lens > 8 || !(threshold >= 0.0) || threshold > 1.0)
        return SR_E_ARG;
    sr::GateLens lens{};
    lens.n = n_lens;
    for (int l = 0; l < n_lens; ++l) {
        const int K = prefix_lens[l];
        if (K < 1 || K > 32 || K > stride) return SR_E_ARG;
        lens.len[l] = K;
        lens.bound[l] = (int)sr::gate_bound(threshold, G, K);
    }
    return sr::launch_gate(actions, n_groups, G, stride, lens, sums, retire, (hipStream_t)stream);
}

extern "C" int sr_gate_batch_antidiag(const int32_t *actions, int n_groups, int G, int stride,
                                      const int *prefix_lens, int n_lens, double threshold, int32_t *sums,
                                      uint8_t *retire, void *stream) {
    if (!actions || !prefix_lens || n_groups < 0 || G < 2 || G > 16 || stride < 1 || n_lens < 1 ||
        n_lens > 8 || !(threshold >= 0.0) || threshold > 1.0)
        return SR_E_ARG;
    sr::GateLens lens{};
    lens.n = n_lens;
    for (int l = 0; l < n_lens; ++l) {
        const int K = prefix_lens[l];
        if (K < 1 || K > 32 || K > stride) return SR_E_ARG;
        lens.len[l] = K;
        lens.bound[l] = (int)sr::gate_bound(threshold, G, K);
    }
    return sr::launch_gate_antidiag(actions, n_groups, G, stride, lens, sums, retire, (hipStream_t)stream);
}
