// Peak probes for measurements: what this chip reaches on a register-resident stream of bf16 MFMAs and on a plain
// streaming copy.  Roofline fractions are quoted against the datasheet figures and against these.
#include "common.h"

namespace pserve {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

static __device__ long long probe_clk[2 * 512];   // per block: shader cycles and 100 MHz ticks of the timed loop

constexpr int PROBE_ACC = 4;                 // independent accumulator tiles per wavefront
constexpr int PROBE_FRAG = 4;                // distinct A and B fragments per wavefront

// a standard normal from a counter (hash -> two uniforms -> Box-Muller); only the distribution matters here
__device__ __forceinline__ float probe_normal(uint32_t n) {
    uint32_t x = n * 2654435761u + 12345u;
    x ^= x >> 16; x *= 0x7feb352du; x ^= x >> 15; x *= 0x846ca68bu; x ^= x >> 16;
    uint32_t y = x * 2246822519u + 977u;
    y ^= y >> 15; y *= 0x2c1b3c6du; y ^= y >> 12;
    const float u1 = ((float)(x >> 8) + 1.f) * (1.f / 16777217.f), u2 = (float)(y >> 8) * (1.f / 16777216.f);
    return sqrtf(-2.f * __logf(u1)) * __cosf(6.2831853f * u2);
}

// 4 wavefronts per block, two blocks per CU; every wavefront issues 8 * iters v_mfma_f32_32x32x16_bf16 on register
// operands: all 1.0 (RANDOM = false) or standard normals rounded to bf16 (RANDOM = true: the bit activity of real
// activations, which is what the chip's power management reacts to)
template <bool RANDOM>
__global__ void __launch_bounds__(256, 2) probe_mfma_kernel(int iters) {
    bf16x8 a[PROBE_FRAG], b[PROBE_FRAG];
#pragma unroll
    for (int n = 0; n < PROBE_FRAG; ++n)
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            a[n][i] = (__bf16)(RANDOM ? probe_normal((threadIdx.x * 64 + n * 16 + i) * 2u) : 1.f);
            b[n][i] = (__bf16)(RANDOM ? probe_normal((threadIdx.x * 64 + n * 16 + i) * 2u + 1u) : 1.f);
        }
    f32x16 acc[PROBE_ACC];
#pragma unroll
    for (int n = 0; n < PROBE_ACC; ++n)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[n][e] = 0.f;
    const long long c0 = clock64(), w0 = wall_clock64();
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int n = 0; n < 8; ++n)
            acc[n % PROBE_ACC] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[n % PROBE_FRAG], b[(n / 2) % PROBE_FRAG], acc[n % PROBE_ACC], 0, 0, 0);
        if ((it & 63) == 63) {                                   // keep the sums finite
#pragma unroll
            for (int n = 0; n < PROBE_ACC; ++n)
#pragma unroll
                for (int e = 0; e < 16; ++e) acc[n][e] *= 1e-3f;
        }
    }
    const long long c1 = clock64(), w1 = wall_clock64();
    if (threadIdx.x == 0 && blockIdx.x < 512) { probe_clk[2 * blockIdx.x] = c1 - c0; probe_clk[2 * blockIdx.x + 1] = w1 - w0; }
    float s = 0.f;
#pragma unroll
    for (int n = 0; n < PROBE_ACC; ++n) s += acc[n][0];
    if (s == 12345.678f) probe_clk[0] = 0;              // keeps the accumulators alive
}

// The same stream with other work between the MFMAs, on standard-normal operands: what a kernel with that instruction
// mix can reach at best on this chip (no global memory, no barriers, every operand in registers or LDS).  The clock
// follows the power drawn, so an added instruction costs issue time or energy; the probe shows the sum.  MIX bits:
//   1  two v_exp_f32 and one v_cvt_pk_bf16_f32 per MFMA (the softmax of 32 scores per lane and MFMA pair)
//   2  one 16-byte LDS fragment read per two MFMAs, into the A operands (they change as in a real kernel)
//   4  one v_mfma_f32_4x4x4_16b_bf16 per two MFMAs (the row sums)
//   8  seven 16-byte LDS fragment reads per ten MFMAs instead of bit 2 (a 64 x 160 wavefront tile of a GEMM)
//  16  two v_add_f32 per MFMA (the row sums on the vector unit)
// 19 is the inner loop of the self-attention kernel (7 with the row sums it had before), 8 that of the convolution.
template <int MIX>
__global__ void __launch_bounds__(256, 2) probe_mix_kernel(int iters) {
    __shared__ __attribute__((aligned(16))) uint8_t frag[16384];
    for (int i = threadIdx.x; i < 4096; i += 256) {
        const __bf16 lo = (__bf16)probe_normal((blockIdx.x * 4096 + i) * 2u), hi = (__bf16)probe_normal((blockIdx.x * 4096 + i) * 2u + 1u);
        reinterpret_cast<uint32_t*>(frag)[i] = (uint32_t)__builtin_bit_cast(uint16_t, lo) | ((uint32_t)__builtin_bit_cast(uint16_t, hi) << 16);
    }
    __syncthreads();
    bf16x8 a[PROBE_FRAG], b[PROBE_FRAG];
#pragma unroll
    for (int n = 0; n < PROBE_FRAG; ++n)
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            a[n][i] = (__bf16)probe_normal((threadIdx.x * 64 + n * 16 + i) * 2u);
            b[n][i] = (__bf16)probe_normal((threadIdx.x * 64 + n * 16 + i) * 2u + 1u);
        }
    f32x16 acc[PROBE_ACC];
#pragma unroll
    for (int n = 0; n < PROBE_ACC; ++n)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[n][e] = 0.f;
    typedef __attribute__((ext_vector_type(4))) float f32x4;
    typedef __attribute__((ext_vector_type(4))) short s16x4;
    f32x4 accl = {0.f, 0.f, 0.f, 0.f};
    const s16x4 ones = {0x3f80, 0x3f80, 0x3f80, 0x3f80};
    float ex[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) ex[i] = probe_normal(threadIdx.x * 8 + i);
    uint32_t pk[4] = {0u, 0u, 0u, 0u};
    const int lane = threadIdx.x & 63;
    // fragment address: row lane % 32 of a 128-byte-row tile, chunk swizzled as in the kernels (no bank conflicts)
    uint32_t addr = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) uint8_t*)frag + (lane & 31) * 128 +
                    16 * ((lane >> 5) ^ (((lane & 31) >> 1) & 7));
    const long long c0 = clock64(), w0 = wall_clock64();
    for (int it = 0; it < iters; ++it) {
        constexpr int NM = (MIX & 8) ? 10 : 8;
#pragma unroll
        for (int j = 0; j < NM; ++j) {
            asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(acc[j & 3]) : "v"(a[j & 3]), "v"(b[(j >> 1) & 3]));
            if (MIX & 1) {
                asm volatile("v_exp_f32 %0, %1" : "=v"(ex[j & 7]) : "v"(acc[(j + 1) & 3][j]));
                asm volatile("v_exp_f32 %0, %1" : "=v"(ex[(j + 4) & 7]) : "v"(acc[(j + 1) & 3][(j + 8) & 15]));
                asm volatile("s_nop 0\n\tv_cvt_pk_bf16_f32 %0, %1, %2" : "=v"(pk[j & 3]) : "v"(ex[j & 7]), "v"(ex[(j + 3) & 7]));
            }
            if (((MIX & 2) && (j & 1)) || ((MIX & 8) && j < 7))
                asm volatile("ds_read_b128 %0, %1" : "=v"(a[(j + 2) & 3]) : "v"(addr));
            if (MIX & 16) {
                asm volatile("v_add_f32 %0, %0, %1" : "+v"(accl[0]) : "v"(ex[(j + 2) & 7]));
                asm volatile("v_add_f32 %0, %0, %1" : "+v"(accl[1]) : "v"(ex[(j + 6) & 7]));
            }
            if ((MIX & 4) && !(j & 1)) {
                const s16x4 p4 = {(short)pk[j & 2], (short)(pk[j & 2] >> 16), (short)pk[(j & 2) + 1], (short)(pk[(j & 2) + 1] >> 16)};
                asm volatile("v_mfma_f32_4x4x4_16b_bf16 %0, %1, %2, %0" : "+v"(accl) : "v"(ones), "v"(p4));
            }
        }
        addr ^= 4096u << (it & 1);                              // other fragments next time
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        if ((it & 63) == 63) {
#pragma unroll
            for (int n = 0; n < PROBE_ACC; ++n)
#pragma unroll
                for (int e = 0; e < 16; ++e) acc[n][e] *= 1e-3f;
        }
    }
    const long long c1 = clock64(), w1 = wall_clock64();
    if (threadIdx.x == 0 && blockIdx.x < 512) { probe_clk[2 * blockIdx.x] = c1 - c0; probe_clk[2 * blockIdx.x + 1] = w1 - w0; }
    float s = accl[0];
#pragma unroll
    for (int n = 0; n < PROBE_ACC; ++n) s += acc[n][0] + __uint_as_float(pk[n]);
#pragma unroll
    for (int i = 0; i < 8; ++i) s += ex[i];
    if (s == 12345.678f) probe_clk[0] = 0;
}

// four independent 16-byte loads in flight per lane, then the four stores
__global__ void __launch_bounds__(256) probe_copy_kernel(const u32x4* __restrict__ src, u32x4* __restrict__ dst, int64_t n16) {
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    for (; i + 3 * stride < n16; i += 4 * stride) {
        const u32x4 v0 = __builtin_nontemporal_load(src + i), v1 = __builtin_nontemporal_load(src + i + stride);
        const u32x4 v2 = __builtin_nontemporal_load(src + i + 2 * stride), v3 = __builtin_nontemporal_load(src + i + 3 * stride);
        __builtin_nontemporal_store(v0, dst + i);
        __builtin_nontemporal_store(v1, dst + i + stride);
        __builtin_nontemporal_store(v2, dst + i + 2 * stride);
        __builtin_nontemporal_store(v3, dst + i + 3 * stride);
    }
    for (; i < n16; i += stride) dst[i] = src[i];
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

int pserve_probe_mfma_bf16(int iters, int random_operands, double* tflops, double* mhz, void* stream) {
    PS_REQUIRE(tflops && iters > 0 && iters <= (1 << 22), "pserve_probe_mfma_bf16: need tflops and 0 < iters <= 2^22");
    hipStream_t st = (hipStream_t)stream;
    const int blocks = 512;                                   // two blocks of four wavefronts on each of the 256 CUs
    float ms = 0.f;
    PS_TRY(time_launches(st, 3, [&] {
        if (random_operands) probe_mfma_kernel<true><<<blocks, 256, 0, st>>>(iters);
        else probe_mfma_kernel<false><<<blocks, 256, 0, st>>>(iters);
        return check_launch("probe_mfma_kernel");
    }, &ms));
    const double flops = (double)blocks * 4 * (double)iters * 8 * (2.0 * 32 * 32 * 16);
    *tflops = flops / ((double)ms * 1e-3) / 1e12;
    if (mhz) {
        static long long h[2 * 512];
        PS_CHECK_HIP(hipMemcpyFromSymbol(h, HIP_SYMBOL(probe_clk), sizeof(h)));
        double cycles = 0.0, ticks = 0.0;
        for (int i = 0; i < blocks; ++i) { cycles += (double)h[2 * i]; ticks += (double)h[2 * i + 1]; }
        *mhz = ticks > 0.0 ? cycles / ticks * 100.0 : 0.0;
    }
    return PSERVE_OK;
}

int pserve_probe_mfma_mix(int iters, int mix, double* tflops, double* mhz, void* stream) {
    PS_REQUIRE(tflops && iters > 0 && iters <= (1 << 22), "pserve_probe_mfma_mix: need tflops and 0 < iters <= 2^22");
    PS_REQUIRE(mix == 8 || (mix >= 0 && mix < 32 && !(mix & 8)), "pserve_probe_mfma_mix: mix is a sum of 1, 2, 4, 16, or 8 alone");
    hipStream_t st = (hipStream_t)stream;
    const int blocks = 512;
    float ms = 0.f;
#define PS_MIX_CASE(m_) case m_: probe_mix_kernel<m_><<<blocks, 256, 0, st>>>(iters); break;
    auto launch = [&] {
        switch (mix) {
        PS_MIX_CASE(0) PS_MIX_CASE(1) PS_MIX_CASE(2) PS_MIX_CASE(3) PS_MIX_CASE(4) PS_MIX_CASE(5) PS_MIX_CASE(6) PS_MIX_CASE(7)
        PS_MIX_CASE(16) PS_MIX_CASE(17) PS_MIX_CASE(18) PS_MIX_CASE(19) PS_MIX_CASE(20) PS_MIX_CASE(21) PS_MIX_CASE(22) PS_MIX_CASE(23)
        default: probe_mix_kernel<8><<<blocks, 256, 0, st>>>(iters); break;
        }
        return check_launch("probe_mix_kernel");
    };
#undef PS_MIX_CASE
    PS_TRY(time_launches(st, 3, launch, &ms));
    const double flops = (double)blocks * 4 * (double)iters * (mix == 8 ? 10 : 8) * (2.0 * 32 * 32 * 16);   // the 32 x 32 x 16 MFMAs only
    *tflops = flops / ((double)ms * 1e-3) / 1e12;
    if (mhz) {
        static long long h[2 * 512];
        PS_CHECK_HIP(hipMemcpyFromSymbol(h, HIP_SYMBOL(probe_clk), sizeof(h)));
        double cycles = 0.0, ticks = 0.0;
        for (int i = 0; i < blocks; ++i) { cycles += (double)h[2 * i]; ticks += (double)h[2 * i + 1]; }
        *mhz = ticks > 0.0 ? cycles / ticks * 100.0 : 0.0;
    }
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
