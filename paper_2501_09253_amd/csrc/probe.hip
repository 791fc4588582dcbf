// Peak probes for measurements: what this chip reaches on a register-resident stream of bf16 MFMAs and on a plain
// streaming copy.  Roofline fractions are quoted against the datasheet figures and against these.
#include "common.h"

namespace pserve {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

static __device__ float probe_sink;          // keeps the accumulators of the MFMA probe alive

constexpr int PROBE_ACC = 8;                 // independent accumulator tiles per wavefront

// 4 wavefronts per block; every wavefront issues iters * PROBE_ACC independent v_mfma_f32_32x32x16_bf16
__global__ void __launch_bounds__(256) probe_mfma_kernel(int iters) {
    bf16x8 a, b;
#pragma unroll
    for (int i = 0; i < 8; ++i) { a[i] = (__bf16)(0.001f * (float)(threadIdx.x & 7) + (float)i); b[i] = (__bf16)(0.5f * (float)i); }
    f32x16 acc[PROBE_ACC];
#pragma unroll
    for (int n = 0; n < PROBE_ACC; ++n)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[n][e] = 0.f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int n = 0; n < PROBE_ACC; ++n) acc[n] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[n], 0, 0, 0);
    }
    float s = 0.f;
#pragma unroll
    for (int n = 0; n < PROBE_ACC; ++n) s += acc[n][0];
    if (s == 12345.678f) probe_sink = s;
}

__global__ void __launch_bounds__(256) probe_copy_kernel(const u32x4* __restrict__ src, u32x4* __restrict__ dst, int64_t n16) {
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += stride) dst[i] = src[i];
}

// time `reps` launches with a pair of events on the stream; *ms = average per launch
template <class F>
static int time_launches(hipStream_t st, int reps, F&& launch, float* ms) {
    hipEvent_t e0 = nullptr, e1 = nullptr;
    PS_CHECK_HIP(hipEventCreate(&e0));
    hipError_t err = hipEventCreate(&e1);
    if (err != hipSuccess) { (void)hipEventDestroy(e0); PS_CHECK_HIP(err); }
    int status = launch();                                    // warm-up launch
    if (status == PSERVE_OK) {
        err = hipEventRecord(e0, st);
        for (int r = 0; r < reps && status == PSERVE_OK && err == hipSuccess; ++r) status = launch();
        if (err == hipSuccess) err = hipEventRecord(e1, st);
        if (err == hipSuccess) err = hipEventSynchronize(e1);
        if (err == hipSuccess) err = hipEventElapsedTime(ms, e0, e1);
    }
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    PS_TRY(status);
    PS_CHECK_HIP(err);
    *ms /= (float)reps;
    return PSERVE_OK;
}

}  // namespace pserve

using namespace pserve;

extern "C" {

int pserve_probe_mfma_bf16(int iters, double* tflops, void* stream) {
    PS_REQUIRE(tflops && iters > 0 && iters <= (1 << 22), "pserve_probe_mfma_bf16: need tflops and 0 < iters <= 2^22");
    hipStream_t st = (hipStream_t)stream;
    const int blocks = 512;                                   // two blocks of four wavefronts on each of the 256 CUs
    float ms = 0.f;
    PS_TRY(time_launches(st, 3, [&] {
        probe_mfma_kernel<<<blocks, 256, 0, st>>>(iters);
        return check_launch("probe_mfma_kernel");
    }, &ms));
    const double flops = (double)blocks * 4 * (double)iters * PROBE_ACC * (2.0 * 32 * 32 * 16);
    *tflops = flops / ((double)ms * 1e-3) / 1e12;
    return PSERVE_OK;
}

int pserve_probe_copy(void* dst, const void* src, size_t bytes, int reps, double* gbs, void* stream) {
    PS_REQUIRE(dst && src && gbs && bytes >= 16 && bytes % 16 == 0 && reps > 0 && reps <= 1000,
               "pserve_probe_copy: need buffers, bytes a positive multiple of 16, 0 < reps <= 1000");
    PS_REQUIRE(((uintptr_t)dst & 15) == 0 && ((uintptr_t)src & 15) == 0, "pserve_probe_copy: buffers must be 16-byte aligned");
    hipStream_t st = (hipStream_t)stream;
    float ms = 0.f;
    const int64_t n16 = (int64_t)(bytes / 16);
    const unsigned grid = (unsigned)std::min<int64_t>(cdiv(n16, 256), 256 * 32);
    PS_TRY(time_launches(st, reps, [&] {
        probe_copy_kernel<<<grid, 256, 0, st>>>((const u32x4*)src, (u32x4*)dst, n16);
        return check_launch("probe_copy_kernel");
    }, &ms));
    *gbs = 2.0 * (double)bytes / ((double)ms * 1e-3) / 1e9;     // bytes read + bytes written
    return PSERVE_OK;
}

}  // extern "C"
