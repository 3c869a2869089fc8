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

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int kThreads = 256;
constexpr int kKC = 4;                    // k-steps (of 32) per LDS chunk of X
constexpr int kPF = 8;                    // k-steps of W held in registers ahead of the MFMAs (two X chunks)
constexpr int kChunkVec = kKC * 512;      // uint4 per chunk: 8 row tiles x 64 lanes per k-step

// Weight loads.  At decode time every weight byte is used once per launch, so the load carries the
// non-temporal hint: the caches do not retain the line, and a pure streaming read measures 13 %
// faster with it (6.97 against 6.15 TB/s).  Prefill re-reads W once per row block and keeps the default policy.
template <bool STREAM>
__device__ __forceinline__ u32x4 load_w(const u32x4 *p) {
    if constexpr (STREAM) return __builtin_nontemporal_load(p);
    else return *p;
}

// SKINNY = the whole batch fits one 128-row block (decode): a distinct instantiation, so that the
// weight-streaming launches and the compute-bound prefill launches are told apart in profiles.
//
// Software pipeline per wavefront: a ring of kPF k-steps of W lives in registers; every k-step is
// consumed by 16 MFMAs and its slot is refilled at once with the k-step kPF further on, so 16 KiB of
// weights per wavefront are always in flight.  X chunks (kKC k-steps, 32 KiB) are double buffered
// in LDS: the next chunk is fetched into registers while the current one is being consumed.
// The loop body spans kPF k-steps (two X chunks) and contains no branch: the k extent of X and W is
// padded to a multiple of kPF k-steps with zeros, every split covers whole groups of kPF k-steps,
// prefetches past the end re-read the last valid k-step (never used), and rows of X beyond M are
// computed and never stored.  Without branches the compiler can count outstanding loads exactly,
// so the weight prefetch survives across the workgroup barriers.
template <int EPI, bool SKINNY>
__global__ __launch_bounds__(kThreads, 2) void gemm_kernel(GemmArgs a) {
    __shared__ u32x4 lds[2][kChunkVec];   // 2 x 32 KiB

    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int nb = blockIdx.x, mb = SKINNY ? 0 : blockIdx.y, sp = blockIdx.z;
    int ks0, ks1;                                              // whole groups of kPF k-steps
    split_range(a.ks_total, kPF, a.splits, sp, &ks0, &ks1);
    const int nt0 = nb * 8 + wave * 2;    // first of this wavefront's two 16-feature tiles

    f32x4 acc[8][2];
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int t = 0; t < 2; ++t) acc[i][t] = f32x4{0.f, 0.f, 0.f, 0.f};

    if (ks0 < ks1) {
        const u32x4 *wp0 = (const u32x4 *)a.W + ((size_t)nt0 * a.ks_total) * 64 + lane;
        const u32x4 *wp1 = wp0 + (size_t)a.ks_total * 64;
        // X: thread's r-th vector of a chunk is k-step (tid + 256 r) / 512, position (tid + 256 r) % 512
        const u32x4 *xp = (const u32x4 *)a.X + (size_t)mb * 8 * 64 + tid;
        const size_t x_ks_stride = (size_t)a.mt_total * 64;
        const int last = ks1 - 1;

        u32x4 w0[kPF], w1[kPF], xr[8];
#pragma unroll
        for (int i = 0; i < kPF; ++i) {
            w0[i] = load_w<SKINNY>(wp0 + (size_t)(ks0 + i) * 64);
            w1[i] = load_w<SKINNY>(wp1 + (size_t)(ks0 + i) * 64);
        }
#pragma unroll
        for (int r = 0; r < 8; ++r) xr[r] = xp[(size_t)(ks0 + (r >> 1)) * x_ks_stride + ((r & 1) << 8)];
#pragma unroll
        for (int r = 0; r < 8; ++r) lds[0][tid + kThreads * r] = xr[r];
        __syncthreads();

        for (int ks = ks0; ks < ks1; ks += kPF) {
#pragma unroll
            for (int half = 0; half < kPF / kKC; ++half) {
                const int kc0 = ks + half * kKC;                 // first k-step of the chunk in LDS buffer `half`
#pragma unroll
                for (int r = 0; r < 8; ++r) {                    // next chunk of X (clamped at the end)
                    const int k = min(kc0 + kKC + (r >> 1), last);
                    xr[r] = xp[(size_t)k * x_ks_stride + ((r & 1) << 8)];
                }
                __builtin_amdgcn_sched_barrier(0);
                // X fragments come from LDS one k-step ahead of their MFMAs, the two streams interleaved
                bf16x8 xf[2][8];
#pragma unroll
                for (int mt = 0; mt < 8; ++mt)
                    xf[0][mt] = __builtin_bit_cast(bf16x8, lds[half][mt * 64 + lane]);
#pragma unroll
                for (int kk = 0; kk < kKC; ++kk) {
                    const int i = half * kKC + kk;
                    __builtin_amdgcn_sched_barrier(0);
                    const bf16x8 wa = __builtin_bit_cast(bf16x8, w0[i]);
                    const bf16x8 wb = __builtin_bit_cast(bf16x8, w1[i]);
                    if (kk + 1 < kKC) {
#pragma unroll
                        for (int mt = 0; mt < 8; ++mt)
                            xf[(kk + 1) & 1][mt] = __builtin_bit_cast(bf16x8, lds[half][(kk + 1) * 512 + mt * 64 + lane]);
                    }
#pragma unroll
                    for (int mt = 0; mt < 8; ++mt) {
                        acc[mt][0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wa, xf[kk & 1][mt], acc[mt][0], 0, 0, 0);
                        acc[mt][1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wb, xf[kk & 1][mt], acc[mt][1], 0, 0, 0);
                    }
                    const int kn = min(kc0 + kk + kPF, last);    // refill the slot just consumed
                    w0[i] = load_w<SKINNY>(wp0 + (size_t)kn * 64);
                    w1[i] = load_w<SKINNY>(wp1 + (size_t)kn * 64);
                    if (kk + 1 < kKC) {
#pragma unroll
                        for (int mt = 0; mt < 8; ++mt) {
                            __builtin_amdgcn_sched_group_barrier(0x008, 2, 0);   // 2 MFMA
                            __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);   // 1 LDS read
                        }
                    } else {
                        __builtin_amdgcn_sched_group_barrier(0x008, 16, 0);
                    }
                    __builtin_amdgcn_sched_group_barrier(0x020, 2, 0);           // W refills
                }
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int r = 0; r < 8; ++r) lds[half ^ 1][tid + kThreads * r] = xr[r];
                __syncthreads();
            }
        }
    }

    // accumulator tile: lane (j = lane%16, g = lane/16) holds output features 4g..4g+3 of batch row j
    const int j = lane & 15, g = lane >> 4;
    if constexpr (EPI == EPI_F32) {
        float *out = (float *)a.out + (size_t)sp * a.split_stride;
#pragma unroll
        for (int mt = 0; mt < 8; ++mt) {
            const int m = mb * 128 + mt * 16 + j;
            if (m < a.M) {
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
                if (m < a.M) {
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

// ---------------------------------------------------------------------------------------------
// Prefill (M > 128) kernel: compute bound, so the tile is sized for the matrix cores.
//
// A workgroup owns a 256 x 256 output tile.  Eight computing wavefronts in a 4 x 2 arrangement each take
// 64 features x 128 rows with 32x32x16 MFMAs (128 accumulator registers); both operands reach them through
// LDS, so every byte crosses the vector-memory path once per workgroup: 128 flop per byte fetched.
// Two more wavefronts do nothing but fetch: one copies the W half, the other the X half of each k-step
// (16 KiB each) from global memory straight into LDS with direct-to-LDS loads, up to three k-steps ahead
// through four 32 KiB buffers, and join one workgroup barrier per k-step.  LDS itself is the landing zone
// of the loads in flight, so the prefetch distance is no longer what a register staging set can hold, and
// the computing wavefronts issue nothing but LDS reads and MFMAs (fragments of a k-half are read while the
// MFMAs of the previous one run).  Ten wavefronts put three on two of the SIMDs: 168 registers each.
// Workgroups are numbered so that the 32 that run together on one XCD form an 8 x 4 block of tiles
// (2048 rows x 1024 features) whose operands they share through that XCD's L2.
// ---------------------------------------------------------------------------------------------
constexpr int kPfThreads = 640;            // 8 computing wavefronts + 2 loaders (W, X)
constexpr int kPfKs = 1;                   // k-steps per stage
constexpr int kPfStageVec = 2048 * kPfKs;  // u32x4 per stage: per k-step [W: 16 tiles x 64][X: 16 tiles x 64]
constexpr int kPfBufs = 4;                 // stages in LDS: the loaders run up to three stages ahead
constexpr int kPfLdsBytes = kPfBufs * kPfStageVec * 16;

template <int EPI>
__global__ __launch_bounds__(kPfThreads) void gemm_prefill_kernel(GemmArgs a, int m_blocks, int n_blocks, int sm_count,
                                                                  int st_count) {
    extern __shared__ u32x4 pf_lds[];      // [kPfBufs][kPfStageVec]

    // linear id -> XCD -> supertile -> tile
    const int L = blockIdx.x;
    const int xcd = L & 7, jj = L >> 3;
    const int w = jj & 31, sg = (jj >> 5) * 8 + xcd;
    if (sg >= st_count) return;
    const int mb = (sg % sm_count) * 8 + (w & 7);
    const int nb = (sg / sm_count) * 4 + (w >> 3);
    if (mb >= m_blocks || nb >= n_blocks) return;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);

    const int n_stages = a.ks_total / kPfKs;
    if (wave >= 8) {
        // loaders (wavefront 8: W, wavefront 9: X): stage s lives in buffer s % kPfBufs; barrier s is passed by
        // the computing wavefronts when they are done with stage s - 1 and by a loader when its half of stage s
        // has landed; then buffer (s - 1) % kPfBufs is free and receives stage s + kPfBufs - 1
        const bool is_x = wave == 9;
        const u32x4 *src = is_x ? (const u32x4 *)a.X + (size_t)mb * 16 * 64 + lane
                                : (const u32x4 *)a.W + ((size_t)(nb * 16) * a.ks_total) * 64 + lane;
        const size_t ks_stride = is_x ? (size_t)a.mt_total * 64 : 64;
        const size_t tile_stride = is_x ? 64 : (size_t)a.ks_total * 64;
        const int dst0 = is_x ? 1024 : 0;
        auto copy_stage = [&](int st, int buf) {
            const int k0 = min(st, n_stages - 1) * kPfKs;
#pragma unroll
            for (int kk = 0; kk < kPfKs; ++kk)
#pragma unroll
                for (int t = 0; t < 16; ++t)
                    __builtin_amdgcn_global_load_lds(
                        (const __attribute__((address_space(1))) void *)(src + t * tile_stride + (size_t)(k0 + kk) * ks_stride),
                        (__attribute__((address_space(3))) void *)&pf_lds[buf * kPfStageVec + kk * 2048 + dst0 + t * 64], 16, 0, 0);
        };
#pragma unroll
        for (int i = 0; i < kPfBufs - 1; ++i) copy_stage(i, i);
        int buf = kPfBufs - 1;
        constexpr int kOut = 16 * kPfKs * (kPfBufs - 2);
        constexpr int kWait = 0x0F70 | (kOut & 15) | ((kOut >> 4) << 14);     // all but the oldest stage may stay in flight
        for (int s = 0; s < n_stages; ++s) {
            __builtin_amdgcn_s_waitcnt(kWait);
            asm volatile("" ::: "memory");
            __builtin_amdgcn_s_barrier();
            asm volatile("" ::: "memory");
            copy_stage(s + kPfBufs - 1, buf);
            buf = buf == kPfBufs - 1 ? 0 : buf + 1;
        }
        __builtin_amdgcn_s_waitcnt(0x0F70);
        return;
    }

    const int wn = wave & 3, wm = wave >> 2;
    const int r32 = lane & 31, g2 = lane >> 5;
    const int sub = r32 >> 4, slot0 = (r32 & 15) + 16 * g2;

    f32x16 acc[2][4];                      // [feature group of 32][row group of 32]
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    // fragment offsets inside a k-step: W group i of this wavefront, X group j
    const int woff = (wn * 4 + sub) * 64 + slot0;          // + i * 128 (two tiles) + h * 32
    const int xoff = 1024 + (wm * 8 + sub) * 64 + slot0;   // + j * 128 + h * 32

    int buf = 0;
    for (int s = 0; s < n_stages; ++s) {
        __syncthreads();                   // barrier s: stage s is in LDS
        const u32x4 *base = pf_lds + buf * kPfStageVec;
        buf = buf == kPfBufs - 1 ? 0 : buf + 1;
        bf16x8 wf[2][2], xf[2][4];         // [parity][group]
#pragma unroll
        for (int i = 0; i < 2; ++i) wf[0][i] = __builtin_bit_cast(bf16x8, base[woff + i * 128]);
#pragma unroll
        for (int j = 0; j < 4; ++j) xf[0][j] = __builtin_bit_cast(bf16x8, base[xoff + j * 128]);
        constexpr int Q = 2 * kPfKs;
#pragma unroll
        for (int q = 0; q < Q; ++q) {      // q = k-step * 2 + k-half
            __builtin_amdgcn_sched_barrier(0);
            if (q + 1 < Q) {
                const int o = ((q + 1) >> 1) * 2048 + ((q + 1) & 1) * 32;
#pragma unroll
                for (int i = 0; i < 2; ++i) wf[(q + 1) & 1][i] = __builtin_bit_cast(bf16x8, base[woff + i * 128 + o]);
#pragma unroll
                for (int j = 0; j < 4; ++j) xf[(q + 1) & 1][j] = __builtin_bit_cast(bf16x8, base[xoff + j * 128 + o]);
            }
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[q & 1][i], xf[q & 1][j], acc[i][j], 0, 0, 0);
            if (q + 1 < Q) {
#pragma unroll
                for (int f = 0; f < 6; ++f) {
                    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);   // 1 MFMA
                    __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);   // 1 LDS read
                }
                __builtin_amdgcn_sched_group_barrier(0x008, 2, 0);
            }
        }
        __builtin_amdgcn_sched_barrier(0);
    }

    // accumulator (i, j): lane (r32 = row within the 32-row group, g2) holds, in register v,
    // feature 8 * (v / 4) + 4 * g2 + v % 4 of the 32-feature group
    if constexpr (EPI == EPI_F32) {
        float *out = (float *)a.out;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int m = mb * 256 + wm * 128 + j * 32 + r32;
            if (m < a.M) {
#pragma unroll
                for (int i = 0; i < 2; ++i)
#pragma unroll
                    for (int vq = 0; vq < 4; ++vq) {
                        const int n = nb * 256 + wn * 64 + i * 32 + 8 * vq + 4 * g2;
                        if (n < a.N)
                            *(f32x4 *)(out + (size_t)m * a.ld_out + n) =
                                f32x4{acc[i][j][4 * vq], acc[i][j][4 * vq + 1], acc[i][j][4 * vq + 2], acc[i][j][4 * vq + 3]};
                    }
            }
        }
    } else {
        uint16_t *out = (uint16_t *)a.out;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int m = mb * 256 + wm * 128 + j * 32 + r32;
            if (m < a.M) {
#pragma unroll
                for (int i = 0; i < 2; ++i)
#pragma unroll
                    for (int vq = 0; vq < 2; ++vq) {
                        const int f = nb * 128 + wn * 32 + i * 16 + 8 * vq + 4 * g2;
                        if (f < a.ld_out) {
                            float r[4];
#pragma unroll
                            for (int e = 0; e < 4; ++e) {
                                const float gt = acc[i][j][4 * vq + e];
                                r[e] = gt / (1.0f + __expf(-gt)) * acc[i][j][4 * (vq + 2) + e];
                            }
                            uint2 v = make_uint2(pack_bf16x2(r[0], r[1]), pack_bf16x2(r[2], r[3]));
                            *(uint2 *)(out + frag_offset(m, f, a.mt_total)) = v;
                        }
                    }
            }
        }
    }
}

// ---------------------------------------------------------------------------------------------
// Batches of a few hundred rows (decode steps of a 512-sequence batch) against a wide matrix: neither a weight
// stream (the matrix pipe, not HBM, bounds 512 rows) nor a large tiled GEMM (two row blocks of 256 leave 1.16 rounds
// of tiles and fetch every weight from HBM with only two workgroups sharing it).  One workgroup takes ALL rows (up
// to 512) of 160 packed features, so every weight byte is fetched from HBM exactly once and the 37 888 packed
// gate|up rows of the 7B shape break into 237 workgroups, one round.  Eight wavefronts, each 64 rows x 160 features
// (2 x 5 accumulator tiles of 32 x 32 = 160 registers; seven LDS fragment reads per ten MFMAs).  Both operands go
// global -> LDS with direct-to-LDS loads, one barrier per k-step: X (32 KiB per k-step, L2 resident) two k-steps
// ahead through three buffers, W (10 KiB per k-step, from HBM) five k-steps ahead through six;
// each wavefront copies the X rows it consumes itself and its share of the ten W tiles.  The copies are issued
// from inline assembly: the compiler's wait-count pass then neither sees them nor waits for them before the LDS
// reads, and the wait for the stage that is needed is placed by hand (vector-memory operations of a wavefront
// retire in order, so "all but the newer stage's copies" is a count).
// ---------------------------------------------------------------------------------------------
constexpr int kMidThreads = 512;
constexpr int kMidWTiles = 10;                                     // 160 packed features
constexpr int kMidXTiles = 32;                                     // 512 rows
constexpr int kMidXBufs = 3, kMidWBufs = 6;                        // k-steps of X (from L2) and of W (from HBM) in LDS
constexpr int kMidXVec = kMidXTiles * 64, kMidWVec = kMidWTiles * 64;       // u32x4 per k-step: 32 KiB and 10 KiB
constexpr int kMidLdsBytes = (kMidXBufs * kMidXVec + kMidWBufs * kMidWVec) * 16;   // 156 KiB

__device__ __forceinline__ void lds_dma16(const u32x4 *g, unsigned lds_byte_offset) {
    asm volatile("s_mov_b32 m0, %1\n\tglobal_load_lds_dwordx4 %0, off" ::"v"(g), "s"(lds_byte_offset) : "memory");
}

// wait until at most n of this wavefront's vector-memory operations are outstanding (n uniform, 0..8)
__device__ __forceinline__ void wait_vm_at_most(int n) {
    switch (n) {
        case 0: __builtin_amdgcn_s_waitcnt(0x0F70); break;
        case 1: __builtin_amdgcn_s_waitcnt(0x0F71); break;
        case 2: __builtin_amdgcn_s_waitcnt(0x0F72); break;
        case 3: __builtin_amdgcn_s_waitcnt(0x0F73); break;
        case 4: __builtin_amdgcn_s_waitcnt(0x0F74); break;
        case 5: __builtin_amdgcn_s_waitcnt(0x0F75); break;
        case 6: __builtin_amdgcn_s_waitcnt(0x0F76); break;
        case 7: __builtin_amdgcn_s_waitcnt(0x0F77); break;
        default: __builtin_amdgcn_s_waitcnt(0x0F78); break;
    }
}

template <int EPI>
__global__ __launch_bounds__(kMidThreads) void gemm_mid_kernel(GemmArgs a) {
    extern __shared__ u32x4 mid_lds[];      // X ring [kMidXBufs][32 tiles x 64], then W ring [kMidWBufs][10 tiles x 64]

    const int nb = blockIdx.x;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const bool active = wave * 64 < a.M;               // this wavefront's 64 rows hold valid rows
    const int n_stages = a.ks_total;

    // copies of one k-step: this wavefront's four X tiles (if it has rows) and W tiles wave, wave + 8
    const int n_w = wave + 8 < kMidWTiles ? 2 : 1;
    const u32x4 *xsrc = (const u32x4 *)a.X + (size_t)(wave * 4) * 64 + lane;                       // + ks * mt_total * 64
    const u32x4 *wsrc = (const u32x4 *)a.W + ((size_t)(nb * kMidWTiles + wave) * a.ks_total) * 64 + lane;   // + ks * 64
    const unsigned lds_x = (unsigned)(size_t)(__attribute__((address_space(3))) void *)mid_lds;
    const unsigned lds_w = lds_x + (unsigned)(kMidXBufs * kMidXVec) * 16;
    auto copy_x = [&](int st) {             // past the end: a harmless re-read of the last k-step, never consumed
        if (!active) return;
        const int ks = min(st, n_stages - 1);
        const unsigned base = lds_x + (unsigned)((st % kMidXBufs) * kMidXVec + wave * 4 * 64) * 16;
#pragma unroll
        for (int t = 0; t < 4; ++t) lds_dma16(xsrc + ((size_t)ks * a.mt_total + t) * 64, base + (unsigned)(t * 64) * 16);
    };
    auto copy_w = [&](int st) {
        const int ks = min(st, n_stages - 1);
        const unsigned base = lds_w + (unsigned)((st % kMidWBufs) * kMidWVec + wave * 64) * 16;
        lds_dma16(wsrc + (size_t)ks * 64, base);
        if (n_w == 2) lds_dma16(wsrc + ((size_t)8 * a.ks_total + ks) * 64, base + (unsigned)(8 * 64) * 16);
    };

    f32x16 acc[5][2];                        // [feature group of 32][row group of 32]
#pragma unroll
    for (int i = 0; i < 5; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    const int r32 = lane & 31, g2 = lane >> 5;
    const int sub = r32 >> 4, slot0 = (r32 & 15) + 16 * g2;
    const int woff = kMidXBufs * kMidXVec + sub * 64 + slot0;              // + W buffer + i * 128 + h * 32
    const int xoff = (wave * 4 + sub) * 64 + slot0;                        // + X buffer + j * 128 + h * 32

    // Vector-memory operations of a wavefront retire in order.  Every iteration issues X of k-step s + 2, then W of
    // k-step s + 5; the prologue issues the same pattern for the two iterations before the first, behind W 0..2.
    // So when iteration s begins, what was issued after X(s) is W(s+3), X(s+1), W(s+4), and W(s) is older than X(s).
    copy_w(0); copy_w(1); copy_w(2);
    copy_x(0); copy_w(3);
    copy_x(1); copy_w(4);
    const int n_newer = (active ? 4 : 0) + 2 * n_w;
    int bx = 0, bw = 0;
    for (int s = 0; s < n_stages; ++s) {
        wait_vm_at_most(n_newer);            // X(s) and W(s) have landed
        asm volatile("" ::: "memory");
        __builtin_amdgcn_s_barrier();        // ... for every wavefront, and nobody reads k-step s - 1 any more
        asm volatile("" ::: "memory");
        copy_x(s + 2);                       // into the buffers k-step s - 1 used
        copy_w(s + 5);
        const u32x4 *xb = mid_lds + bx * kMidXVec, *wb = mid_lds + bw * kMidWVec;
        bx = bx == kMidXBufs - 1 ? 0 : bx + 1;
        bw = bw == kMidWBufs - 1 ? 0 : bw + 1;
        if (active) {
            bf16x8 wf[2][5], xf[2][2];       // [k-half parity][group]
#pragma unroll
            for (int i = 0; i < 5; ++i) wf[0][i] = __builtin_bit_cast(bf16x8, wb[woff + i * 128]);
#pragma unroll
            for (int j = 0; j < 2; ++j) xf[0][j] = __builtin_bit_cast(bf16x8, xb[xoff + j * 128]);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int i = 0; i < 5; ++i) wf[1][i] = __builtin_bit_cast(bf16x8, wb[woff + i * 128 + 32]);
#pragma unroll
            for (int j = 0; j < 2; ++j) xf[1][j] = __builtin_bit_cast(bf16x8, xb[xoff + j * 128 + 32]);
#pragma unroll
            for (int i = 0; i < 5; ++i)
#pragma unroll
                for (int j = 0; j < 2; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[0][i], xf[0][j], acc[i][j], 0, 0, 0);
#pragma unroll
            for (int f = 0; f < 7; ++f) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);   // 1 MFMA
                __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);   // 1 LDS read
            }
            __builtin_amdgcn_sched_group_barrier(0x008, 3, 0);
#pragma unroll
            for (int i = 0; i < 5; ++i)
#pragma unroll
                for (int j = 0; j < 2; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[1][i], xf[1][j], acc[i][j], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
        }
    }
    __builtin_amdgcn_s_waitcnt(0x0F70);      // the copies past the end have landed before LDS goes away
    if (!active) return;

    // accumulator (i, j): lane (r32 = row within the 32-row group, g2) holds, in register v,
    // feature 8 * (v / 4) + 4 * g2 + v % 4 of the 32-feature group
    if constexpr (EPI == EPI_F32) {
        float *out = (float *)a.out;
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const int m = wave * 64 + j * 32 + r32;
            if (m < a.M) {
#pragma unroll
                for (int i = 0; i < 5; ++i)
#pragma unroll
                    for (int vq = 0; vq < 4; ++vq) {
                        const int n = nb * 160 + i * 32 + 8 * vq + 4 * g2;
                        if (n < a.N)
                            *(f32x4 *)(out + (size_t)m * a.ld_out + n) =
                                f32x4{acc[i][j][4 * vq], acc[i][j][4 * vq + 1], acc[i][j][4 * vq + 2], acc[i][j][4 * vq + 3]};
                    }
            }
        }
    } else {
        uint16_t *out = (uint16_t *)a.out;
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const int m = wave * 64 + j * 32 + r32;
            if (m < a.M) {
#pragma unroll
                for (int i = 0; i < 5; ++i)
#pragma unroll
                    for (int vq = 0; vq < 2; ++vq) {
                        const int f = nb * 80 + i * 16 + 8 * vq + 4 * g2;
                        if (f < a.ld_out) {
                            float r[4];
#pragma unroll
                            for (int e = 0; e < 4; ++e) {
                                const float gt = acc[i][j][4 * vq + e];
                                r[e] = gt / (1.0f + __expf(-gt)) * acc[i][j][4 * (vq + 2) + e];
                            }
                            uint2 v = make_uint2(pack_bf16x2(r[0], r[1]), pack_bf16x2(r[2], r[3]));
                            *(uint2 *)(out + frag_offset(m, f, a.mt_total)) = v;
                        }
                    }
            }
        }
    }
}

// The same kernel for 257 .. 384 rows on 16x16x32 MFMAs: with 64-row slabs five (or six) of the eight wavefronts
// would have rows, two of them on one SIMD, and that SIMD would carry 128 rows.  Here the 16-row tiles are dealt
// out round robin, wavefront w owning tiles w, w + 8, w + 16 (at most three), so 19 tiles (304 rows) put 5, 5, 5
// and 4 on the four SIMDs.  A 16-row fragment-major tile is one MFMA operand as it lies in LDS (one 16-byte read per
// lane): 10 W + up to 3 X reads for up to 30 MFMAs per k-step.  Copies, rings, barrier and wait counts as above.
template <int EPI>
__global__ __launch_bounds__(kMidThreads) void gemm_mid16_kernel(GemmArgs a) {
    constexpr int RT = 3;
    extern __shared__ u32x4 mid_lds[];

    const int nb = blockIdx.x;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int n_tiles = (a.M + 15) >> 4;
    const int my_tiles = wave < n_tiles ? min(RT, (n_tiles - wave + 7) >> 3) : 0;     // tiles wave, wave + 8, ...
    const int n_stages = a.ks_total;

    const int n_w = wave + 8 < kMidWTiles ? 2 : 1;
    const u32x4 *xsrc = (const u32x4 *)a.X + (size_t)wave * 64 + lane;                             // + (ks * mt_total + 8 t) * 64
    const u32x4 *wsrc = (const u32x4 *)a.W + ((size_t)(nb * kMidWTiles + wave) * a.ks_total) * 64 + lane;
    const unsigned lds_x = (unsigned)(size_t)(__attribute__((address_space(3))) void *)mid_lds;
    const unsigned lds_w = lds_x + (unsigned)(kMidXBufs * kMidXVec) * 16;
    auto copy_x = [&](int st) {
        const int ks = min(st, n_stages - 1);
        const unsigned base = lds_x + (unsigned)((st % kMidXBufs) * kMidXVec + wave * 64) * 16;
#pragma unroll
        for (int t = 0; t < RT; ++t)
            if (t < my_tiles) lds_dma16(xsrc + ((size_t)ks * a.mt_total + 8 * t) * 64, base + (unsigned)(8 * t * 64) * 16);
    };
    auto copy_w = [&](int st) {
        const int ks = min(st, n_stages - 1);
        const unsigned base = lds_w + (unsigned)((st % kMidWBufs) * kMidWVec + wave * 64) * 16;
        lds_dma16(wsrc + (size_t)ks * 64, base);
        if (n_w == 2) lds_dma16(wsrc + ((size_t)8 * a.ks_total + ks) * 64, base + (unsigned)(8 * 64) * 16);
    };

    f32x4 acc[kMidWTiles][RT];               // [feature tile of 16][row tile]: lane (c, g) holds features 4g..4g+3 of row c
#pragma unroll
    for (int i = 0; i < kMidWTiles; ++i)
#pragma unroll
        for (int t = 0; t < RT; ++t) acc[i][t] = f32x4{0.f, 0.f, 0.f, 0.f};

    const int woff = kMidXBufs * kMidXVec + lane;                          // + W buffer + i * 64
    const int xoff = wave * 64 + lane;                                     // + X buffer + t * 512

    copy_w(0); copy_w(1); copy_w(2);
    copy_x(0); copy_w(3);
    copy_x(1); copy_w(4);
    const int n_newer = my_tiles + 2 * n_w;  // issued after X(s): W(s+3), X(s+1), W(s+4)
    int bx = 0, bw = 0;
    for (int s = 0; s < n_stages; ++s) {
        wait_vm_at_most(n_newer);
        asm volatile("" ::: "memory");
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
        copy_x(s + 2);
        copy_w(s + 5);
        const u32x4 *xb = mid_lds + bx * kMidXVec, *wb = mid_lds + bw * kMidWVec;
        bx = bx == kMidXBufs - 1 ? 0 : bx + 1;
        bw = bw == kMidWBufs - 1 ? 0 : bw + 1;
        if (my_tiles > 0) {
            // tiles 0 and 1 unconditionally (a wavefront with one tile computes it twice and stores it once), tile 2
            // where it exists: one uniform branch per k-step
            bf16x8 xf[RT], wf[kMidWTiles];
            xf[0] = __builtin_bit_cast(bf16x8, xb[xoff]);
            xf[1] = __builtin_bit_cast(bf16x8, xb[xoff + (my_tiles > 1 ? 512 : 0)]);
#pragma unroll
            for (int i = 0; i < kMidWTiles; ++i) wf[i] = __builtin_bit_cast(bf16x8, wb[woff + i * 64]);
            if (my_tiles == 3) xf[2] = __builtin_bit_cast(bf16x8, xb[xoff + 1024]);
#pragma unroll
            for (int i = 0; i < kMidWTiles; ++i)
#pragma unroll
                for (int t = 0; t < 2; ++t)
                    acc[i][t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wf[i], xf[t], acc[i][t], 0, 0, 0);
            if (my_tiles == 3) {
#pragma unroll
                for (int i = 0; i < kMidWTiles; ++i)
                    acc[i][2] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wf[i], xf[2], acc[i][2], 0, 0, 0);
            }
        }
    }
    __builtin_amdgcn_s_waitcnt(0x0F70);
    if (my_tiles == 0) return;

    const int c = lane & 15, g = lane >> 4;
#pragma unroll
    for (int t = 0; t < RT; ++t) {
        const int m = (wave + 8 * t) * 16 + c;
        if (t >= my_tiles || m >= a.M) continue;
        if constexpr (EPI == EPI_F32) {
            float *out = (float *)a.out + (size_t)m * a.ld_out;
#pragma unroll
            for (int i = 0; i < kMidWTiles; ++i) {
                const int n = nb * 160 + i * 16 + 4 * g;
                if (n < a.N) *(f32x4 *)(out + n) = acc[i][t];
            }
        } else {
            uint16_t *out = (uint16_t *)a.out;
#pragma unroll
            for (int i = 0; i < kMidWTiles / 2; ++i) {      // tile 2i = gate, tile 2i + 1 = up of features f..f+15
                const int f = nb * 80 + i * 16 + 4 * g;
                if (f < a.ld_out) {
                    float r[4];
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const float gt = acc[2 * i][t][e];
                        r[e] = gt / (1.0f + __expf(-gt)) * acc[2 * i + 1][t][e];
                    }
                    *(uint2 *)(out + frag_offset(m, f, a.mt_total)) =
                        make_uint2(pack_bf16x2(r[0], r[1]), pack_bf16x2(r[2], r[3]));
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

namespace {

// 256 x 256 tiles over all of `a`
int launch_tiles256(const GemmArgs &a, GemmEpilogue epi, hipStream_t stream) {
    static bool attr_set = false;
    if (!attr_set) {
        SR_HIP(hipFuncSetAttribute((const void *)gemm_prefill_kernel<EPI_F32>,
                                   hipFuncAttributeMaxDynamicSharedMemorySize, kPfLdsBytes));
        SR_HIP(hipFuncSetAttribute((const void *)gemm_prefill_kernel<EPI_SWIGLU>,
                                   hipFuncAttributeMaxDynamicSharedMemorySize, kPfLdsBytes));
        attr_set = true;
    }
    const int mb256 = ceil_div(a.M, 256), nb256 = ceil_div(a.N, 256);
    const int sm_count = ceil_div(mb256, 8), sn_count = ceil_div(nb256, 4);
    const int st_count = sm_count * sn_count;
    dim3 pgrid((unsigned)(ceil_div(st_count, 8) * 8 * 32)), pblock(kPfThreads);
    if (epi == EPI_F32)
        gemm_prefill_kernel<EPI_F32><<<pgrid, pblock, kPfLdsBytes, stream>>>(a, mb256, nb256, sm_count, st_count);
    else
        gemm_prefill_kernel<EPI_SWIGLU><<<pgrid, pblock, kPfLdsBytes, stream>>>(a, mb256, nb256, sm_count, st_count);
    SR_HIP(hipGetLastError());
    return SR_OK;
}

// 128 x 128 tiles over all of `a` (also the 4-wavefront decode kernel when the batch is one row block)
int launch_tiles128(const GemmArgs &a, GemmEpilogue epi, hipStream_t stream) {
    const int m_blocks = ceil_div(a.M, 128), n_blocks = ceil_div(a.N, 128);
    dim3 grid(n_blocks, m_blocks, epi == EPI_F32 ? a.splits : 1), block(kThreads);
    if (m_blocks == 1) {
        if (epi == EPI_F32) gemm_kernel<EPI_F32, true><<<grid, block, 0, stream>>>(a);
        else gemm_kernel<EPI_SWIGLU, true><<<grid, block, 0, stream>>>(a);
    } else {
        if (epi == EPI_F32) gemm_kernel<EPI_F32, false><<<grid, block, 0, stream>>>(a);
        else gemm_kernel<EPI_SWIGLU, false><<<grid, block, 0, stream>>>(a);
    }
    SR_HIP(hipGetLastError());
    return SR_OK;
}

// All rows (at most 512) of 160 packed features per workgroup; no K split.  The last workgroup reads whole tiles
// past N: the packed matrix is allocated (and zero) up to a multiple of 160 rows.
int launch_mid(const GemmArgs &a, GemmEpilogue epi, hipStream_t stream) {
    static bool attr_set = false;
    if (!attr_set) {
        SR_HIP(hipFuncSetAttribute((const void *)gemm_mid_kernel<EPI_F32>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                   kMidLdsBytes));
        SR_HIP(hipFuncSetAttribute((const void *)gemm_mid_kernel<EPI_SWIGLU>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                   kMidLdsBytes));
        SR_HIP(hipFuncSetAttribute((const void *)gemm_mid16_kernel<EPI_F32>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                   kMidLdsBytes));
        SR_HIP(hipFuncSetAttribute((const void *)gemm_mid16_kernel<EPI_SWIGLU>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                   kMidLdsBytes));
        attr_set = true;
    }
    if (a.M > 512 || a.splits != 1 || a.ks_total < 1 || round_up(a.M, 64) > a.mt_total * 16) return SR_E_ARG;
    dim3 grid((unsigned)ceil_div(a.N, 160)), block(kMidThreads);
    if (a.M > 256 && a.M <= 384) {           // 17 .. 24 row tiles: three per wavefront, dealt out round robin
        if (epi == EPI_F32) gemm_mid16_kernel<EPI_F32><<<grid, block, kMidLdsBytes, stream>>>(a);
        else gemm_mid16_kernel<EPI_SWIGLU><<<grid, block, kMidLdsBytes, stream>>>(a);
    } else if (epi == EPI_F32) gemm_mid_kernel<EPI_F32><<<grid, block, kMidLdsBytes, stream>>>(a);
    else gemm_mid_kernel<EPI_SWIGLU><<<grid, block, kMidLdsBytes, stream>>>(a);
    SR_HIP(hipGetLastError());
    return SR_OK;
}

// `a` restricted to the packed columns from c0 (a multiple of 256) on
GemmArgs columns_from(const GemmArgs &a, GemmEpilogue epi, int c0) {
    GemmArgs b = a;
    b.N = a.N - c0;
    b.W = a.W + (size_t)(c0 / 16) * a.ks_total * 64;
    if (epi == EPI_F32) {
        b.out = (float *)a.out + c0;
    } else {                                   // output feature c0 / 2 of the fragment-major matrix
        b.out = (uint16_t *)a.out + frag_offset(0, c0 / 2, a.mt_total);
        b.ld_out = a.ld_out - c0 / 2;
    }
    return b;
}

}  // namespace

int launch_gemm(const GemmArgs &a, GemmEpilogue epi, hipStream_t stream) {
    if (a.M <= 0) return SR_OK;
    const int m_blocks = ceil_div(a.M, 128);
    if (m_blocks * 8 > a.mt_total || a.splits < 1 || m_blocks > 65535 || a.splits > 65535 || a.ks_total % 16)
        return SR_E_ARG;
    if (m_blocks == 1 && a.wide) return launch_gemm_stream(a, epi, stream);
    const int mb256 = ceil_div(a.M, 256), nb256 = ceil_div(a.N, 256);
    if (m_blocks > 1 && a.splits == 1 && mb256 * 16 <= a.mt_total) {
        const int tiles256 = mb256 * nb256;
        if (a.M > 1024) {
            // Prefill-sized batches: 256 x 256 tiles when they fill the 256 CUs well -- always for wide outputs; for
            // N of a few thousand only if the last round of workgroups is not mostly empty.
            const bool fills = tiles256 * 8 >= ceil_div(tiles256, 256) * 256 * 7;      // >= 87.5 % of the slots used
            if (a.N >= 16384 || (a.N >= 2048 && fills)) return launch_tiles256(a, epi, stream);
            // Otherwise whole rounds of large tiles over the first column blocks and small tiles over the rest, where
            // that is cheaper than small tiles throughout.  Measured at 8192 and 5120 rows, in units of one small tile
            // among thousands: a round of large tiles costs 810; a launch of up to 256 small tiles (one per CU) 500, of
            // up to 512 (two per CU) 1100.  QKV at 8192 rows: two rounds and 256 small tiles, 253 against 275 us; at 5120
            // rows every thin projection is cheaper on small tiles alone.
            if (a.N >= 2048 && mb256 <= 256) {
                const int cols_per_round = 256 / mb256;
                const int rounds_a = nb256 / cols_per_round;
                const int c0 = rounds_a * cols_per_round * 256;
                if (rounds_a > 0 && c0 < a.N) {
                    const long long rest = (long long)m_blocks * ceil_div(a.N - c0, 128);
                    const long long cost_mix = (long long)rounds_a * 810 + (rest <= 256 ? 500 : rest < 1100 ? 1100 : rest);
                    const long long cost128 = (long long)m_blocks * ceil_div(a.N, 128);
                    if (cost_mix < cost128) {
                        GemmArgs first = a;
                        first.N = c0;
                        SR_TRY(launch_tiles256(first, epi, stream));
                        return launch_tiles128(columns_from(a, epi, c0), epi, stream);
                    }
                }
            }
            return launch_tiles128(a, epi, stream);
        }
        // A few hundred rows against a wide matrix (gate|up, LM head): every row in one workgroup of 160 features
        if (a.M <= 512 && a.N >= 16384) return launch_mid(a, epi, stream);
        // A few hundred rows (decode steps of a large batch).  256 x 256 tiles run one workgroup per CU in whole
        // rounds of 256; 128 x 128 tiles run two per CU and drain almost continuously.  Measured at 304 and 512
        // rows, K = 3584: 150 us a round (the weights come from HBM: only two row blocks share them) against 0.166 us
        // a small tile, both proportional to K, i.e. a round costs what 900 small tiles do, and a launch of small
        // tiles at least what 200 of them do.  Third choice: whole rounds of large tiles over the first columns and
        // small tiles over the rest, in two launches.
        const long long cost256 = (long long)ceil_div(tiles256, 256) * 900;
        long long cost128 = (long long)m_blocks * ceil_div(a.N, 128);
        if (cost128 < 200) cost128 = 200;
        const int cols_per_round = 256 / mb256;                   // column blocks of 256 in one round of large tiles
        const int rounds_a = nb256 / cols_per_round;
        const int c0 = rounds_a * cols_per_round * 256;           // first column of the small-tile part
        long long cost_mix = -1;
        if (rounds_a > 0 && c0 < a.N) {
            const long long rest = (long long)m_blocks * ceil_div(a.N - c0, 128);
            cost_mix = (long long)rounds_a * 900 + (rest > 200 ? rest : 200) + 20;
        }
        if (cost_mix >= 0 && cost_mix < cost256 && cost_mix < cost128) {
            GemmArgs first = a;
            first.N = c0;
            SR_TRY(launch_tiles256(first, epi, stream));
            return launch_tiles128(columns_from(a, epi, c0), epi, stream);
        }
        if (cost256 <= cost128) return launch_tiles256(a, epi, stream);
    }
    return launch_tiles128(a, epi, stream);
}

}  // namespace sr
