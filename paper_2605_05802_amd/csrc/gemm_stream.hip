// Decode-time projection GEMM  Y[M][N] = X[M][K] * W[N][K]^T  for M <= 128 on the bf16 matrix cores:
// the weight-streaming kernel that carries most of a decode step's HBM traffic.
#include "sr_internal.h"

namespace sr {
namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int kKC = 4;                    // k-steps (of 32) per LDS chunk of X
constexpr int kChunkVec = kKC * 512;      // uint4 per chunk: 8 row tiles x 64 lanes per k-step

// Every weight byte is used once per launch, so the load carries the non-temporal hint: the caches do
// not retain the line, and a pure streaming read measures 13 % faster with it (6.97 against 6.15 TB/s).
__device__ __forceinline__ u32x4 load_w_stream(const u32x4 *p) { return __builtin_nontemporal_load(p); }

// ---------------------------------------------------------------------------------------------
// Decode-time (M <= 128) weight-streaming kernel with a loader wavefront.
//
// A workgroup owns 32 * WAVES output features and all rows; each of its WAVES computing wavefronts
// owns 32 features and streams their weights through a register ring of RING k-steps (2 KiB each),
// refilling a slot as soon as its MFMAs are issued, so RING * 2 KiB per wavefront stay in flight
// across the workgroup barriers.  The loop body has no branch: the compiler counts outstanding
// loads exactly, and prefetches past the end re-read the last valid k-step.
//
// The activations are brought in by one extra wavefront that does nothing else: it copies X chunks
// (kKC k-steps, 32 KiB) from global memory straight into LDS with lane-linear 16-byte direct-to-LDS
// loads, two chunks ahead of the MFMAs, through three buffers.  Vector-memory loads return in order
// within a wavefront, so an activation load inside a computing wavefront would make its wait drain
// the older weight loads too; with the loader the computing wavefronts carry only weight loads,
// never wait for an activation and keep no staging registers, and the loader's wait for its own
// copies stalls nobody.
//
// The MFMA is the 32x32x16 form: with one workgroup per CU all wavefronts stall at the same
// barriers, and a single wavefront keeps the matrix pipe far busier with 32x32 tiles than with
// 16x16 ones.  Its operands (32 rows x 16 k) are assembled from the 16-row fragment layout by
// addressing: lane (r = lane % 32, g = lane / 32) of k-half h takes the 16 bytes of row tile r / 16,
// lane slot (r % 16) + 16 * (2h + g).
//
// MT32 = number of 32-row tiles computed (M <= 32 * MT32): smaller batches skip the idle rows'
// copies, LDS reads and MFMAs.  Workgroup width matters because with one workgroup per CU a matrix
// should break into about 256 equal workgroups: 37 888 packed gate|up rows give 148 workgroups of
// 256 features (108 CUs idle) but 237 of 160.
// ---------------------------------------------------------------------------------------------
constexpr int kStBufs = 3;                 // LDS chunk buffers: the loader runs two chunks ahead
constexpr int kStLdsBytes = kStBufs * kChunkVec * 16;

// RING = k-steps of W each computing wavefront keeps in flight (8 or 16; 2 KiB per k-step)
template <int EPI, int WAVES, int MT32, int RING>
__global__ __launch_bounds__(64 * (WAVES + 1)) void gemm_stream_kernel(GemmArgs a) {
    extern __shared__ u32x4 lds_dyn[];     // [kStBufs][k-step in chunk][16-row tile 0..7][lane]

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int nb = blockIdx.x, sp = blockIdx.z;
    int ks0, ks1;
    split_range(a.ks_total, RING, a.splits, sp, &ks0, &ks1);
    const int last = ks1 - 1;

    if (wave == WAVES) {
        // ---- loader.  Chunk c lives in buffer c % 3.  Barrier c (c = 0, 1, ...) is passed by the
        // computing wavefronts once they are done with chunk c - 1, and by the loader once chunk c has
        // landed; after it the loader may overwrite the buffer of chunk c - 1 with chunk c + 2.
        if (ks0 >= ks1) return;
        const u32x4 *xp = (const u32x4 *)a.X + lane;
        const size_t x_ks_stride = (size_t)a.mt_total * 64;
        constexpr int kCopies = kKC * 2 * MT32;         // direct-to-LDS loads per chunk (<= 32)
        auto copy_chunk = [&](int kc, int buf) {
#pragma unroll
            for (int kk = 0; kk < kKC; ++kk) {
                const u32x4 *src = xp + (size_t)min(kc + kk, last) * x_ks_stride;
#pragma unroll
                for (int b = 0; b < 2 * MT32; ++b)
                    __builtin_amdgcn_global_load_lds(
                        (const __attribute__((address_space(1))) void *)(src + b * 64),
                        (__attribute__((address_space(3))) void *)&lds_dyn[buf * kChunkVec + kk * 512 + b * 64], 16,
                        0, 0);
            }
        };
        // wait until at most one chunk of copies is outstanding: vmcnt(kCopies), other counters untouched
        constexpr int kWaitOlder = 0x0F70 | (kCopies & 15) | ((kCopies >> 4) << 14);
        copy_chunk(ks0, 0);
        copy_chunk(ks0 + kKC, 1);
        int buf = 2;
        for (int kc = ks0; kc < ks1; kc += kKC) {
            __builtin_amdgcn_s_waitcnt(kWaitOlder);
            asm volatile("" ::: "memory");
            __builtin_amdgcn_s_barrier();
            asm volatile("" ::: "memory");
            copy_chunk(kc + 2 * kKC, buf);               // past the end: re-copies the last k-step, never read
            buf = buf == kStBufs - 1 ? 0 : buf + 1;
        }
        __builtin_amdgcn_s_waitcnt(kWaitOlder);
        asm volatile("" ::: "memory");
        __builtin_amdgcn_s_barrier();
        __builtin_amdgcn_s_waitcnt(0x0F70);              // nothing may still be writing LDS at exit
        return;
    }

    const int nt32 = nb * WAVES + wave;             // this wavefront's 32 output features
    const int r32 = lane & 31, g2 = lane >> 5;
    const int sub = r32 >> 4;                       // which 16-row tile of the pair
    const int slot0 = (r32 & 15) + 16 * g2;         // lane slot for k-half 0; k-half 1 is +32

    f32x16 acc[MT32];
#pragma unroll
    for (int i = 0; i < MT32; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[i][v] = 0.f;

    if (ks0 < ks1) {
        const u32x4 *wp0 = (const u32x4 *)a.W + ((size_t)(nt32 * 2 + sub) * a.ks_total) * 64 + slot0;
        const u32x4 *wp1 = wp0 + 32;
        const int xoff = sub * 64 + slot0;          // + mt32 * 128 + h * 32 inside a k-step of a buffer
        constexpr int NF = 2 * MT32;                // X fragments per k-step

        u32x4 w0[RING], w1[RING];
#pragma unroll
        for (int i = 0; i < RING; ++i) {
            w0[i] = load_w_stream(wp0 + (size_t)(ks0 + i) * 64);
            w1[i] = load_w_stream(wp1 + (size_t)(ks0 + i) * 64);
        }
        __syncthreads();                                         // barrier 0: chunk 0 is in LDS

        int buf = 0;
        for (int ks = ks0; ks < ks1; ks += RING) {
#pragma unroll
            for (int q = 0; q < RING / kKC; ++q) {
                const int kc0 = ks + q * kKC;
                bf16x8 xf[2][NF];                                // [parity][mt32 * 2 + k-half]
                const u32x4 *xb = &lds_dyn[buf * kChunkVec + xoff];
                buf = buf == kStBufs - 1 ? 0 : buf + 1;
#pragma unroll
                for (int f = 0; f < NF; ++f)
                    xf[0][f] = __builtin_bit_cast(bf16x8, xb[(f >> 1) * 128 + (f & 1) * 32]);
#pragma unroll
                for (int kk = 0; kk < kKC; ++kk) {
                    const int i = q * kKC + kk;
                    __builtin_amdgcn_sched_barrier(0);
                    const bf16x8 wa = __builtin_bit_cast(bf16x8, w0[i]);
                    const bf16x8 wb = __builtin_bit_cast(bf16x8, w1[i]);
                    if (kk + 1 < kKC) {
#pragma unroll
                        for (int f = 0; f < NF; ++f)
                            xf[(kk + 1) & 1][f] =
                                __builtin_bit_cast(bf16x8, xb[(kk + 1) * 512 + (f >> 1) * 128 + (f & 1) * 32]);
                    }
#pragma unroll
                    for (int mt = 0; mt < MT32; ++mt) {
                        acc[mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wa, xf[kk & 1][mt * 2], acc[mt], 0, 0, 0);
                        acc[mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wb, xf[kk & 1][mt * 2 + 1], acc[mt], 0, 0, 0);
                    }
                    const int kn = min(kc0 + kk + RING, last);  // refill the slot just consumed
                    w0[i] = load_w_stream(wp0 + (size_t)kn * 64);
                    w1[i] = load_w_stream(wp1 + (size_t)kn * 64);
                    if (kk + 1 < kKC) {
#pragma unroll
                        for (int f = 0; f < NF; ++f) {
                            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);   // 1 MFMA
                            __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);   // 1 LDS read
                        }
                    } else {
                        __builtin_amdgcn_sched_group_barrier(0x008, NF, 0);
                    }
                    __builtin_amdgcn_sched_group_barrier(0x020, 2, 0);           // W refills
                }
                __builtin_amdgcn_sched_barrier(0);
                __syncthreads();
            }
        }
    }

    // accumulator of row tile mt: lane (r32 = batch row within the tile, g2) holds, in register v,
    // output feature 8 * (v / 4) + 4 * g2 + v % 4 of the wavefront's 32
    if constexpr (EPI == EPI_F32) {
        float *out = (float *)a.out + (size_t)sp * a.split_stride;
#pragma unroll
        for (int mt = 0; mt < MT32; ++mt) {
            const int m = mt * 32 + r32;
            if (m < a.M) {
#pragma unroll
                for (int vq = 0; vq < 4; ++vq) {
                    const int n = nt32 * 32 + 8 * vq + 4 * g2;
                    if (n < a.N)
                        *(f32x4 *)(out + (size_t)m * a.ld_out + n) =
                            f32x4{acc[mt][4 * vq], acc[mt][4 * vq + 1], acc[mt][4 * vq + 2], acc[mt][4 * vq + 3]};
                }
            }
        }
    } else {
        // packed rows 0..15 of the 32 are gate features, 16..31 the matching up features
        uint16_t *out = (uint16_t *)a.out;
#pragma unroll
        for (int mt = 0; mt < MT32; ++mt) {
            const int m = mt * 32 + r32;
            if (m < a.M) {
#pragma unroll
                for (int vq = 0; vq < 2; ++vq) {
                    const int f = nt32 * 16 + 8 * vq + 4 * g2;
                    if (f < a.ld_out) {
                        float r[4];
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            const float gt = acc[mt][4 * vq + e];
                            r[e] = gt / (1.0f + __expf(-gt)) * acc[mt][4 * (vq + 2) + e];
                        }
                        uint2 v = make_uint2(pack_bf16x2(r[0], r[1]), pack_bf16x2(r[2], r[3]));
                        *(uint2 *)(out + frag_offset(m, f, a.mt_total)) = v;
                    }
                }
            }
        }
    }
}

}  // namespace

int launch_gemm_stream(const GemmArgs &a, GemmEpilogue epi, hipStream_t stream) {
    if (a.M <= 0) return SR_OK;
    if (a.M > 128 || a.mt_total < 8 || a.splits < 1 || a.splits > 65535) return SR_E_ARG;
    const int ring = a.ring == 16 ? 16 : 8;
    if (a.ks_total % ring || (a.wide != 2 && a.wide != 4 && a.wide != 5 && a.wide != 8 && a.wide != 10)) return SR_E_ARG;
    dim3 sgrid(ceil_div(a.N, 32 * a.wide), 1, epi == EPI_F32 ? a.splits : 1), lblock(64 * (a.wide + 1));
    const int mt32 = ceil_div(a.M, 32);
    hipError_t attr = hipSuccess;
#define SR_STREAM_CASE(E, W, T, R)                                                                          \
    (attr = hipFuncSetAttribute((const void *)gemm_stream_kernel<E, W, T, R>,                                \
                        hipFuncAttributeMaxDynamicSharedMemorySize, kStLdsBytes),                   \
     gemm_stream_kernel<E, W, T, R><<<sgrid, lblock, kStLdsBytes, stream>>>(a))
#define SR_STREAM_MT(E, W, R)                                                                               \
    (mt32 == 1 ? SR_STREAM_CASE(E, W, 1, R) : mt32 == 2 ? SR_STREAM_CASE(E, W, 2, R)                         \
     : mt32 == 3 ? SR_STREAM_CASE(E, W, 3, R) : SR_STREAM_CASE(E, W, 4, R))
#define SR_STREAM_W(E, R)                                                                                   \
    (a.wide == 2 ? SR_STREAM_MT(E, 2, R) : a.wide == 4 ? SR_STREAM_MT(E, 4, R)                               \
     : a.wide == 5 ? SR_STREAM_MT(E, 5, R) : a.wide == 8 ? SR_STREAM_MT(E, 8, R) : SR_STREAM_MT(E, 10, R))
    // nine wavefronts put three on one SIMD, which leaves too few registers for the deep ring
#define SR_STREAM_W16(E)                                                                                    \
    (a.wide == 2 ? SR_STREAM_MT(E, 2, 16) : a.wide == 4 ? SR_STREAM_MT(E, 4, 16) : SR_STREAM_MT(E, 5, 16))
    if (ring == 16 && a.wide >= 8) return SR_E_ARG;
    if (epi == EPI_F32) { if (ring == 16) SR_STREAM_W16(EPI_F32); else SR_STREAM_W(EPI_F32, 8); }
    else { if (ring == 16) SR_STREAM_W16(EPI_SWIGLU); else SR_STREAM_W(EPI_SWIGLU, 8); }
    SR_HIP(attr);
    SR_HIP(hipGetLastError());
    return SR_OK;
}

}  // namespace sr
