// Teacher-forced log-likelihood (paper Appendix C.2) and the policy-gradient loss (Section 2.1).
//
// logprob_rows_kernel: one workgroup per logits row.  log softmax(row)[target] needs the row's
// maximum and the sum of exponentials; every thread keeps a running (max, sum) pair over its
// strided part of the row, so the row (vocab x 4 bytes, 608 KiB at the 7B shape) is read once, and
// the pairs are combined through LDS.  Rows whose next token is not an action token are skipped.
//
// accumulate_logprob_kernel: one thread per sequence adds the per-token values of a chunk to the
// sequence's running log-likelihood in token order (double), so the sum does not depend on scheduling.
//
// grpo_loss_kernel: one thread per group computes the advantages of Eq. 1 (population standard
// deviation; exactly zero when all rewards of the group are equal) and the group's share of
// sum_i A_i log p(tau_i); thread 0 adds the shares in group order.
#include <mutex>

#include "sr_internal.h"

namespace sr {
namespace {

constexpr int kLpThreads = 512;

__device__ __forceinline__ void lse_merge(float &m, float &s, float m2, float s2) {
    const float mn = fmaxf(m, m2);
    s = s * expf(m - mn) + s2 * expf(m2 - mn);
    m = mn;
}

__global__ __launch_bounds__(kLpThreads) void logprob_rows_kernel(LogprobArgs a) {
    __shared__ float s_m[kLpThreads / 64], s_s[kLpThreads / 64];
    const int row = blockIdx.x, tid = threadIdx.x;
    // row -> (unit, token index in the chunk whose probability this row's logits give)
    const int u = (a.row0 + row) / a.rows_per_unit;
    const int t = a.tok0 + (a.row0 + row) % a.rows_per_unit;
    if (t >= a.chunk_len) return;                             // the chunk's last row predicts nothing here
    float *dst = a.out + (size_t)u * a.chunk_len + t;
    if (a.mask && !a.mask[(size_t)u * a.chunk_len + t]) {
        if (tid == 0) *dst = 0.f;
        return;
    }
    const float *lg = a.logits + (size_t)row * a.vocab;
    float m = -3.0e38f, s = 0.f;
    const int v4 = a.vocab & ~3;
    for (int v = tid * 4; v < v4; v += kLpThreads * 4) {
        const float4 x = *(const float4 *)(lg + v);
        const float mx = fmaxf(fmaxf(x.x, x.y), fmaxf(x.z, x.w));
        const float mn = fmaxf(m, mx);
        s = s * expf(m - mn) + expf(x.x - mn) + expf(x.y - mn) + expf(x.z - mn) + expf(x.w - mn);
        m = mn;
    }
    for (int v = v4 + tid; v < a.vocab; v += kLpThreads) lse_merge(m, s, lg[v], 1.f);
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) lse_merge(m, s, __shfl_xor(m, off, 64), __shfl_xor(s, off, 64));
    if ((tid & 63) == 0) { s_m[tid >> 6] = m; s_s[tid >> 6] = s; }
    __syncthreads();
    if (tid == 0) {
        for (int w = 1; w < kLpThreads / 64; ++w) lse_merge(m, s, s_m[w], s_s[w]);
        const int target = a.tokens[(size_t)u * a.chunk_len + t];
        *dst = (lg[target] - m) - logf(s);
    }
}

__global__ void accumulate_logprob_kernel(const float *__restrict__ tok_lp, int n_seq, int chunk_len,
                                          double *__restrict__ logprob) {
    const int u = blockIdx.x * blockDim.x + threadIdx.x;
    if (u >= n_seq) return;
    double acc = logprob[u];
    for (int t = 0; t < chunk_len; ++t) acc += (double)tok_lp[(size_t)u * chunk_len + t];
    logprob[u] = acc;
}

__global__ __launch_bounds__(256) void grpo_loss_kernel(const double *__restrict__ logprob,
                                                        const float *__restrict__ rewards, int n_groups, int G,
                                                        double eps, float *__restrict__ adv, double *__restrict__ share,
                                                        double *__restrict__ loss) {
    for (int g = threadIdx.x; g < n_groups; g += blockDim.x) {
        const float *r = rewards + (size_t)g * G;
        bool all_equal = true;
        double mean = 0.0;
        for (int i = 0; i < G; ++i) {
            all_equal &= r[i] == r[0];
            mean += (double)r[i];
        }
        mean /= G;
        double var = 0.0;
        for (int i = 0; i < G; ++i) var += ((double)r[i] - mean) * ((double)r[i] - mean);
        const double sigma = sqrt(var / G);
        double acc = 0.0;
        for (int i = 0; i < G; ++i) {
            const double A = all_equal ? 0.0 : ((double)r[i] - mean) / (sigma + eps);
            if (adv) adv[(size_t)g * G + i] = (float)A;
            acc += A * logprob[(size_t)g * G + i];
        }
        share[g] = acc;
    }
    __syncthreads();          // one workgroup: the shares written above are visible to thread 0
    if (threadIdx.x == 0) {
        double acc = 0.0;
        for (int g = 0; g < n_groups; ++g) acc += share[g];
        *loss = -acc / ((double)n_groups * G);
    }
}

}  // namespace

int launch_logprob_rows(const LogprobArgs &a, int rows, hipStream_t stream) {
    if (rows <= 0) return SR_OK;
    if (a.rows_per_unit < 1 || a.vocab < 1 || a.chunk_len < 1) return SR_E_ARG;
    logprob_rows_kernel<<<dim3(rows), dim3(kLpThreads), 0, stream>>>(a);
    SR_HIP(hipGetLastError());
    return SR_OK;
}

int launch_accumulate_logprob(const float *tok_lp, int n_seq, int chunk_len, double *logprob, hipStream_t stream) {
    if (n_seq <= 0) return SR_OK;
    accumulate_logprob_kernel<<<dim3((n_seq + 63) / 64), dim3(64), 0, stream>>>(tok_lp, n_seq, chunk_len, logprob);
    SR_HIP(hipGetLastError());
    return SR_OK;
}

}  // namespace sr

extern "C" int sr_grpo_loss(const double *logprob, const float *rewards, int n_groups, int G, double eps,
                            float *advantages, double *group_scratch, double *loss, void *stream) {
    if (!logprob || !rewards || !group_scratch || !loss || n_groups < 1 || G < 1 || !(eps >= 0.0)) return SR_E_ARG;
    sr::grpo_loss_kernel<<<dim3(1), dim3(256), 0, (hipStream_t)stream>>>(logprob, rewards, n_groups, G, eps, advantages,
                                                                         group_scratch, loss);
    SR_HIP(hipGetLastError());
    return SR_OK;
}

// ---------------------------------------------------------------------------------------------
// The same loss for callers that cannot allocate: the per-group shares live in a file-scope device
// array instead of a buffer the caller brings.
// ---------------------------------------------------------------------------------------------
namespace {

constexpr int kStaticMaxGroups = SR_GRPO_STATIC_MAX_GROUPS;
static __device__ __align__(256) double scratch[kStaticMaxGroups];   // every GPU holds its own copy

constexpr int kMaxDevices = 64;
double *g_scratch_ptr[kMaxDevices];        // device address of `scratch` on each GPU, looked up once
bool g_scratch_known[kMaxDevices];
std::mutex g_scratch_mutex;

// Device address of this GPU's copy of `scratch` (the array's name is only a host-side stand-in).
int static_scratch(double **out) {
    int dev = -1;
    SR_HIP(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return SR_E_ARG;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_known[dev]) {
        void *p = nullptr;
        SR_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        g_scratch_ptr[dev] = (double *)p;
        g_scratch_known[dev] = true;
    }
    *out = g_scratch_ptr[dev];
    return SR_OK;
}

}  // namespace

extern "C" int sr_grpo_loss_static(const double *logprob, const float *rewards, int n_groups, int G, double eps,
                                   float *advantages, double *loss, void *stream) {
    if (!logprob || !rewards || !loss || n_groups < 1 || G < 1 || !(eps >= 0.0)) return SR_E_ARG;
    if (n_groups > kStaticMaxGroups) return SR_E_LIMIT;
    double *share = nullptr;
    SR_TRY(static_scratch(&share));
    // every share[g], g < n_groups, is written before it is read: nothing of an earlier call is used
    sr::grpo_loss_kernel<<<dim3(1), dim3(256), 0, (hipStream_t)stream>>>(logprob, rewards, n_groups, G, eps, advantages,
                                                                         share, loss);
    SR_HIP(hipGetLastError());
    return SR_OK;
}
