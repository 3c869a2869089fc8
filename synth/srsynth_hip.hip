// Device-side twin of srs_fill_table16 (srsynth.c): fills a bf16 tensor in HBM with the same
// SplitMix64 counter-based stream and the same quantile-table lookup, bit for bit, so that
// multi-gigabyte weight tensors need not cross PCIe.  Input generation only.
#include <hip/hip_runtime.h>
#include <stdint.h>

#define SRS_GOLDEN 0x9E3779B97F4A7C15ULL

__host__ __device__ static inline uint64_t srs_finalize(uint64_t z) {
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ULL;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBULL;
    return z ^ (z >> 31);
}

__global__ void fill_table16_kernel(uint16_t *dst, size_t n, uint64_t key, uint64_t first,
                                    const uint16_t *__restrict__ table) {
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x)
        dst[i] = table[srs_finalize(key + (first + i + 1ULL) * SRS_GOLDEN) >> 48];
}

extern "C" int srs_fill_table16_dev(void *dst, size_t n, uint64_t seed, uint64_t stream_id, uint64_t first,
                                    const void *table_dev, void *hip_stream) {
    if (n == 0) return 0;
    const uint64_t key =
        srs_finalize(srs_finalize(seed + SRS_GOLDEN) ^ (stream_id * 0xD1342543DE82EF95ULL + 1ULL));
    size_t blocks = (n + 255) / 256;
    if (blocks > 65536) blocks = 65536;
    fill_table16_kernel<<<dim3((unsigned)blocks), dim3(256), 0, (hipStream_t)hip_stream>>>(
        (uint16_t *)dst, n, key, first, (const uint16_t *)table_dev);
    return (int)hipGetLastError();
}
