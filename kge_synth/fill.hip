// Device-side twin of kge_synth.uniform_rows(): fills a table with the same pure function of
// (seed, tag, row, column).  Input generation only; no part of the method lives here.
#include <hip/hip_runtime.h>
#include <stdint.h>

__device__ __forceinline__ uint64_t synth_mix(uint64_t base, uint64_t idx) {
    uint64_t z = base + idx * 0xBF58476D1CE4E5B9ull;
    z ^= z >> 30; z *= 0xBF58476D1CE4E5B9ull;
    z ^= z >> 27; z *= 0x94D049BB133111EBull;
    z ^= z >> 31;
    return z;
}

__device__ __forceinline__ uint16_t synth_bf16_rne(float x) {
    uint32_t u = __builtin_bit_cast(uint32_t, x);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

__global__ void synth_fill_kernel(void *dst, int64_t n_rows, int dim, int64_t ld, uint64_t base, float scale,
                                  int bf16, int64_t row0) {
    const int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= n_rows * dim) return;
    const int64_t row = e / dim;
    const int col = (int)(e % dim);
    const uint64_t z = synth_mix(base, (uint64_t)(row0 + row) * 4096ull + (uint64_t)col);
    const float v = (float)((int)(z >> 40) - (1 << 23)) * scale;
    if (bf16) ((uint16_t *)dst)[row * ld + col] = synth_bf16_rne(v);
    else ((float *)dst)[row * ld + col] = v;
}

extern "C" int synth_fill_uniform(void *dst, int64_t n_rows, int dim, int64_t ld, uint64_t seed, uint32_t tag,
                                  float amp, int bf16, int64_t row0, void *stream) {
    if (n_rows <= 0) return 0;
    const uint64_t base = seed * 0xD1342543DE82EF95ull + (uint64_t)tag * 0x9E3779B97F4A7C15ull;
    const float scale = amp / 8388608.0f;
    const int64_t total = n_rows * dim;
    const int64_t chunk_rows = (1ll << 30) / dim;          // keep the grid within 2^31 threads
    for (int64_t r = 0; r < n_rows; r += chunk_rows) {
        const int64_t nr = n_rows - r < chunk_rows ? n_rows - r : chunk_rows;
        const int64_t cnt = nr * dim;
        char *p = (char *)dst + r * ld * (bf16 ? 2 : 4);
        hipLaunchKernelGGL(synth_fill_kernel, dim3((unsigned)((cnt + 255) / 256)), dim3(256), 0, (hipStream_t)stream,
                           (void *)p, nr, dim, ld, base, scale, bf16, row0 + r);
    }
    (void)total;
    return hipGetLastError() == hipSuccess ? 0 : -1;
}
