// Projection GEMMs  Y[M][N] = X[M][K] * W[N][K]^T  on the bf16 matrix cores.
//
// During decode the batch M is the number of live sequences (128 at the headline shape), so
// every projection is a weight-streaming problem: W is read exactly once per step from HBM
// and each byte of it is used for M multiply-adds.  The kernel is organised around that
// stream:
//   - W is stored pre-tiled in MFMA operand order, so each wavefront reads its 32 output
//     features as two contiguous runs with 16-byte loads per lane straight into registers
//     (no LDS hop for the operand that is used once);
//   - the activations X (small, re-used by every workgroup, L2 resident) are staged through
//     LDS in the same operand order and shared by the four wavefronts of a workgroup;
//   - one workgroup owns all rows of a 128-row block for its 128 output features, so no
//     weight byte is fetched twice; thin matrices are split along K across workgroups and the
//     fp32 partial results are summed, in fixed order, by the kernel that consumes them.
// The same kernel serves prefill, where M is thousands of rows: grid.y walks 128-row blocks.
#include "sr_internal.h"

namespace sr {
namespace {

constexpr int kThreads = 256;
constexpr int kKC = 4;                    // k-steps (of 32) per LDS chunk
constexpr int kChunkVec = kKC * 512;      // uint4 per chunk: 8 row tiles x 64 lanes per k-step

// SKINNY = the whole batch fits one 128-row block (decode): a distinct instantiation, so that the
// weight-streaming launches and the compute-bound prefill launches are told apart in profiles.
template <int EPI, bool SKINNY>
__global__ __launch_bounds__(kThreads, 2) void gemm_kernel(GemmArgs a) {
    __shared__ uint4 lds[2][kChunkVec];   // 2 x 32 KiB

    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int nb = blockIdx.x, mb = SKINNY ? 0 : blockIdx.y, sp = blockIdx.z;
    const int ks_per_split = ceil_div(a.ks_total, a.splits);
    const int ks0 = sp * ks_per_split;
    const int ks1 = min(ks0 + ks_per_split, a.ks_total);
    const int nt0 = nb * 8 + wave * 2;    // first of this wavefront's two 16-feature tiles
    const int m_valid = min(128, a.M - mb * 128);
    const int mt_valid = ceil_div(m_valid, 16);

    f32x4 acc[8][2];
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int t = 0; t < 2; ++t) acc[i][t] = f32x4{0.f, 0.f, 0.f, 0.f};

    const uint4 *wp0 = a.W + ((size_t)nt0 * a.ks_total) * 64 + lane;
    const uint4 *wp1 = wp0 + (size_t)a.ks_total * 64;
    const uint4 *xp = a.X + (size_t)mb * 8 * 64;        // + (ks*mt_total)*64 + i

    uint4 wcur[kKC][2], wnext[kKC][2], xnext[8];
    const uint4 zero4 = make_uint4(0, 0, 0, 0);

    auto load_w = [&](int ks, uint4 (&w)[kKC][2]) {
#pragma unroll
        for (int kk = 0; kk < kKC; ++kk) {
            if (ks + kk < ks1) {
                w[kk][0] = wp0[(size_t)(ks + kk) * 64];
                w[kk][1] = wp1[(size_t)(ks + kk) * 64];
            } else {
                w[kk][0] = zero4;
                w[kk][1] = zero4;
            }
        }
    };
    auto load_x = [&](int ks) {
#pragma unroll
        for (int r = 0; r < 8; ++r) {
            const int i = tid + kThreads * r;           // uint4 index within the chunk
            const int kk = i >> 9, within = i & 511;
            xnext[r] = (ks + kk < ks1) ? xp[((size_t)(ks + kk) * a.mt_total) * 64 + within] : zero4;
        }
    };
    auto store_x = [&](int buf) {
#pragma unroll
        for (int r = 0; r < 8; ++r) lds[buf][tid + kThreads * r] = xnext[r];
    };

    if (ks0 < ks1) {
        load_x(ks0);
        load_w(ks0, wcur);
        store_x(0);
        __syncthreads();
        int buf = 0;
        for (int ks = ks0; ks < ks1; ks += kKC) {
            const bool more = ks + kKC < ks1;
            if (more) {
                load_x(ks + kKC);
                load_w(ks + kKC, wnext);
            }
#pragma unroll
            for (int kk = 0; kk < kKC; ++kk) {
                if (ks + kk < ks1) {
                    const bf16x8 w0 = __builtin_bit_cast(bf16x8, wcur[kk][0]);
                    const bf16x8 w1 = __builtin_bit_cast(bf16x8, wcur[kk][1]);
#pragma unroll
                    for (int mt = 0; mt < 8; ++mt) {
                        if (mt < mt_valid) {
                            const bf16x8 x = __builtin_bit_cast(bf16x8, lds[buf][kk * 512 + mt * 64 + lane]);
                            acc[mt][0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(w0, x, acc[mt][0], 0, 0, 0);
                            acc[mt][1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(w1, x, acc[mt][1], 0, 0, 0);
                        }
                    }
                }
            }
            if (more) {
                store_x(buf ^ 1);
#pragma unroll
                for (int kk = 0; kk < kKC; ++kk) {
                    wcur[kk][0] = wnext[kk][0];
                    wcur[kk][1] = wnext[kk][1];
                }
            }
            __syncthreads();
            buf ^= 1;
        }
    }

    // accumulator tile: lane (j = lane%16, g = lane/16) holds output features 4g..4g+3 of batch row j
    const int j = lane & 15, g = lane >> 4;
    if constexpr (EPI == EPI_F32) {
        float *out = (float *)a.out + (size_t)sp * a.split_stride;
#pragma unroll
        for (int mt = 0; mt < 8; ++mt) {
            const int m = mb * 128 + mt * 16 + j;
            if (mt < mt_valid && m < a.M) {
#pragma unroll
                for (int t = 0; t < 2; ++t) {
                    const int n = (nt0 + t) * 16 + 4 * g;
                    if (n < a.N) *(f32x4 *)(out + (size_t)m * a.ld_out + n) = acc[mt][t];
                }
            }
        }
    } else {
        // tile 0 = gate, tile 1 = up, for features f0..f0+15
        uint16_t *out = (uint16_t *)a.out;
        const int f = (nt0 >> 1) * 16 + 4 * g;
        if (f < a.ld_out) {
#pragma unroll
            for (int mt = 0; mt < 8; ++mt) {
                const int m = mb * 128 + mt * 16 + j;
                if (mt < mt_valid && m < a.M) {
                    float r[4];
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const float gt = acc[mt][0][e];
                        r[e] = gt / (1.0f + __expf(-gt)) * acc[mt][1][e];
                    }
                    uint2 v = make_uint2(pack_bf16x2(r[0], r[1]), pack_bf16x2(r[2], r[3]));
                    *(uint2 *)(out + frag_offset(m, f, a.mt_total)) = v;
                }
            }
        }
    }
}

// One thread per 16-byte lane slot of the packed matrix.
__global__ void pack_rows_kernel(const uint16_t *__restrict__ src, int n_rows, int K, uint16_t *__restrict__ dst,
                                 int ks_total, int dst_row0, int interleave16, int which) {
    const size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;   // (row i, k-step, k-group)
    const size_t per_row = (size_t)ks_total * 4;
    if (idx >= (size_t)n_rows * per_row) return;
    const int i = (int)(idx / per_row);
    const int rem = (int)(idx - (size_t)i * per_row);
    const int ks = rem >> 2, kg = rem & 3;
    const int prow = dst_row0 + (interleave16 ? 32 * (i / 16) + 16 * which + (i % 16) : i);
    const int k0 = ks * 32 + kg * 8;
    uint16_t v[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) v[e] = (k0 + e < K) ? src[(size_t)i * K + k0 + e] : (uint16_t)0;
    uint16_t *d = dst + ((((size_t)(prow >> 4) * ks_total + ks) * 64) + (prow & 15) + 16 * kg) * 8;
    *(uint4 *)d = *(const uint4 *)v;
}

}  // namespace

int launch_pack_rows(const uint16_t *src, int n_rows, int K, uint16_t *dst, int ks_total, int dst_row0,
                     int interleave16, int which, hipStream_t stream) {
    const size_t n = (size_t)n_rows * ks_total * 4;
    if (n == 0) return SR_OK;
    pack_rows_kernel<<<dim3((unsigned)((n + 255) / 256)), dim3(256), 0, stream>>>(src, n_rows, K, dst, ks_total,
                                                                                  dst_row0, interleave16, which);
    SR_HIP(hipGetLastError());
    return SR_OK;
}

int launch_gemm(const GemmArgs &a, GemmEpilogue epi, hipStream_t stream) {
    if (a.M <= 0) return SR_OK;
    const int n_blocks = ceil_div(a.N, 128);
    const int m_blocks = ceil_div(a.M, 128);
    if (m_blocks * 8 > a.mt_total || a.splits < 1 || m_blocks > 65535 || a.splits > 65535) return SR_E_ARG;
    dim3 grid(n_blocks, m_blocks, epi == EPI_F32 ? a.splits : 1), block(kThreads);
    const bool skinny = m_blocks == 1;
    if (epi == EPI_F32) {
        if (skinny) gemm_kernel<EPI_F32, true><<<grid, block, 0, stream>>>(a);
        else gemm_kernel<EPI_F32, false><<<grid, block, 0, stream>>>(a);
    } else {
        if (skinny) gemm_kernel<EPI_SWIGLU, true><<<grid, block, 0, stream>>>(a);
        else gemm_kernel<EPI_SWIGLU, false><<<grid, block, 0, stream>>>(a);
    }
    SR_HIP(hipGetLastError());
    return SR_OK;
}

}  // namespace sr
