// Figures of the GPU the library runs on, for benchmarks that quote rooflines: the rate of a loop of independent
// bf16 matrix instructions (what the matrix pipes deliver when nothing else is asked of the machine) - on constant
// operands, and on operands whose signs and mantissas change from element to element, as those of real tables do (the
// rate the chip sustains depends on how many bits toggle: it lowers its clock to stay inside its power limit) - and the
// rate of a plain streaming copy.  None is part of the method; all synchronise the stream they are given.
#include "block_kernel.hpp"

namespace {

// every wave keeps four independent accumulators and issues 4 x iters v_mfma_f32_32x32x16_bf16; VARIED: four different
// operand pairs per lane, every element with sign and mantissa from a hash and magnitude in [2^-8, 2^-6) (the sums stay
// far inside the fp32 range for any iters allowed), else constant operands
template <bool VARIED>
__global__ __attribute__((amdgpu_flat_work_group_size(512, 512)))
void calib_mfma_kernel(int iters, float *sink) {
    const uint32_t one = 0x3c003c00u;                   // two bf16 of 2^-7
    uint4 a[4], b[4];
#pragma unroll
    for (int c = 0; c < 4; ++c) {
        a[c] = make_uint4(one, one, one, one); b[c] = make_uint4(one ^ (threadIdx.x & 1u), one, one, one);
        if constexpr (VARIED) {
            uint32_t w[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                uint32_t h = (threadIdx.x * 2654435761u) ^ ((uint32_t)(c * 8 + j) * 40503u + 977u);
                h ^= h >> 15; h *= 2246822519u; h ^= h >> 13; h *= 3266489917u; h ^= h >> 16;
                w[j] = (h & 0x807f807fu) | 0x3b803c00u; // exponents of 2^-8 and 2^-7, the other bits from the hash
            }
            a[c] = make_uint4(w[0], w[1], w[2], w[3]); b[c] = make_uint4(w[4], w[5], w[6], w[7]);
        }
    }
    kge_f32x16 acc[4];
#pragma unroll
    for (int c = 0; c < 4; ++c)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[c][i] = 0.f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int c = 0; c < 4; ++c) acc[c] = kge_mma16<true>(acc[c], a[c], b[c]);
    }
    float s = 0.f;
#pragma unroll
    for (int c = 0; c < 4; ++c)
#pragma unroll
        for (int i = 0; i < 16; ++i) s += acc[c][i];
    sink[(size_t)blockIdx.x * blockDim.x + threadIdx.x] = s;
}

__global__ void calib_copy_kernel(const uint4 *src, uint4 *dst, size_t n16) {
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += stride) dst[i] = src[i];
}

// milliseconds of `launch()` on `st`, second of two runs (the first brings the clocks up)
template <typename F> int timed(F launch, hipStream_t st, float *ms) {
    hipEvent_t e0 = nullptr, e1 = nullptr;
    if (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess) return KGE_E_HIP;
    int rc = KGE_OK;
    launch();
    if (hipEventRecord(e0, st) != hipSuccess) rc = KGE_E_HIP;
    launch();
    if (hipEventRecord(e1, st) != hipSuccess || hipEventSynchronize(e1) != hipSuccess ||
        hipEventElapsedTime(ms, e0, e1) != hipSuccess) rc = KGE_E_HIP;
    (void)hipEventDestroy(e0); (void)hipEventDestroy(e1);
    return rc != KGE_OK ? rc : kge_launch_status();
}

}  // namespace

static int calibrate_mfma(bool varied, int32_t iters, float *sink, int64_t sink_elems, double *tflops_out, void *hip_stream) {
    constexpr int WGS = 2048, THREADS = 512;            // 8 workgroups of 8 waves per compute unit
    if (iters <= 0 || iters > (1 << 20) || !sink || sink_elems < (int64_t)WGS * THREADS || !tflops_out) return KGE_E_INVALID_ARG;
    hipStream_t st = (hipStream_t)hip_stream;
    float ms = 0.f;
    const int rc = timed([&] {
        if (varied) hipLaunchKernelGGL(calib_mfma_kernel<true>, dim3(WGS), dim3(THREADS), 0, st, iters, sink);
        else hipLaunchKernelGGL(calib_mfma_kernel<false>, dim3(WGS), dim3(THREADS), 0, st, iters, sink);
    }, st, &ms);
    if (rc != KGE_OK) return rc;
    const double flops = (double)WGS * (THREADS / 64) * 4.0 * iters * (2.0 * 32 * 32 * 16);
    *tflops_out = flops / ((double)ms * 1e-3) / 1e12;
    return KGE_OK;
}

extern "C" int kge_calibrate_mfma(int32_t iters, float *sink, int64_t sink_elems, double *tflops_out, void *hip_stream) {
    return calibrate_mfma(false, iters, sink, sink_elems, tflops_out, hip_stream);
}
extern "C" int kge_calibrate_mfma_varied(int32_t iters, float *sink, int64_t sink_elems, double *tflops_out, void *hip_stream) {
    return calibrate_mfma(true, iters, sink, sink_elems, tflops_out, hip_stream);
}

extern "C" int kge_calibrate_copy(const void *src, void *dst, size_t bytes, double *gbs_out, void *hip_stream) {
    if (!src || !dst || bytes < 16 || bytes % 16 || (((uintptr_t)src | (uintptr_t)dst) & 15) || !gbs_out) return KGE_E_INVALID_ARG;
    hipStream_t st = (hipStream_t)hip_stream;
    float ms = 0.f;
    const int rc = timed([&] { hipLaunchKernelGGL(calib_copy_kernel, dim3(256 * 16), dim3(256), 0, st, (const uint4 *)src,
                                                  (uint4 *)dst, bytes / 16); }, st, &ms);
    if (rc != KGE_OK) return rc;
    *gbs_out = 2.0 * (double)bytes / ((double)ms * 1e-3) / 1e9;     // read + written
    return KGE_OK;
}
