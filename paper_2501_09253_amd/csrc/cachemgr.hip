// Cache manager pieces around the block: the per-patch mean squared error the reuse predictor looks at
// ("Patch-aware Caching Strategy", step 1) and the Common / New / Expired id sets of "Batching Patches in Cache".
#include "common.h"

#include <mutex>
#include <new>
#include <unordered_map>

namespace pserve {

// Partial sums of pserve_patch_mse_static: a fixed array in device memory (one copy per GPU, held until the process
// ends) for callers that may not allocate.  Host code never uses this name as an address: it asks the runtime for
// the array's address on the current device once and passes that pointer on.
constexpr int MSE_STATIC_MAX_PATCHES = PSERVE_MSE_STATIC_MAX_PATCHES;
static __device__ __align__(256) float scratch[MSE_STATIC_MAX_PATCHES * 16];
constexpr int MSE_MAX_DEVICES = 64;
static float* g_scratch_ptr[MSE_MAX_DEVICES] = {};
static std::mutex g_scratch_mutex;

// address of `scratch` on the current device (looked up once per device, with that device current)
static int static_scratch(float** out) {
    int dev = -1;
    PS_CHECK_HIP(hipGetDevice(&dev));
    PS_REQUIRE(dev >= 0 && dev < MSE_MAX_DEVICES, "pserve_patch_mse_static: device index %d not supported", dev);
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        float* ptr = nullptr;
        PS_CHECK_HIP(hipGetSymbolAddress((void**)&ptr, HIP_SYMBOL(scratch)));
        PS_REQUIRE(ptr != nullptr, "pserve_patch_mse_static: no address for the scratch array on device %d", dev);
        g_scratch_ptr[dev] = ptr;
    }
    *out = g_scratch_ptr[dev];
    return PSERVE_OK;
}

typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(4))) float f32x4;

constexpr int MSE_U = 4;          // row pairs a thread keeps in flight
constexpr int MSE_SPLIT = 16;     // token chunks per patch (partial sums per patch)

// sum of squared differences of 16 bytes of a and b
template <typename T> __device__ __forceinline__ float sq_diff16(const T* a, const T* b);
template <> __device__ __forceinline__ float sq_diff16<float>(const float* a, const float* b) {
    const f32x4 x = *reinterpret_cast<const f32x4*>(a), y = *reinterpret_cast<const f32x4*>(b);
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < 4; ++i) { const float d = x[i] - y[i]; s = fmaf(d, d, s); }
    return s;
}
template <> __device__ __forceinline__ float sq_diff16<uint16_t>(const uint16_t* a, const uint16_t* b) {
    const u32x4 x = *reinterpret_cast<const u32x4*>(a), y = *reinterpret_cast<const u32x4*>(b);
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const float d0 = __uint_as_float(x[i] << 16) - __uint_as_float(y[i] << 16);
        const float d1 = __uint_as_float(x[i] & 0xFFFF0000u) - __uint_as_float(y[i] & 0xFFFF0000u);
        s = fmaf(d0, d0, s);
        s = fmaf(d1, d1, s);
    }
    return s;
}

// block (patch p, chunk sp): thread (token lane tl, 16-byte channel vector cv); partial[p][sp] = sum over the chunk
template <typename T>
__global__ void __launch_bounds__(1024)
patch_mse_partial_kernel(const T* __restrict__ a, const T* __restrict__ b, int32_t C, int32_t S, int32_t TL,
                         float* __restrict__ partial) {
    constexpr int VN = 16 / sizeof(T);
    __shared__ float red[16];
    const int CV = C / VN;
    const int cv = threadIdx.x % CV, tl = threadIdx.x / CV;
    const int p = blockIdx.x, sp = blockIdx.y;
    const int chunk = (S + MSE_SPLIT - 1) / MSE_SPLIT;
    const int t0 = sp * chunk, t1 = min(S, t0 + chunk);
    const int64_t base = ((int64_t)p * S) * C + cv * VN;
    float acc = 0.f;
    // the block is rounded up to whole wavefronts; the extra threads (tl >= TL) add nothing
    for (int tb = t0 + tl; tl < TL && tb < t1; tb += MSE_U * TL) {
        float part[MSE_U];
#pragma unroll
        for (int u = 0; u < MSE_U; ++u) {
            const int64_t off = base + (int64_t)min(tb + u * TL, t1 - 1) * C;      // rows past the chunk: last row, ignored
            part[u] = sq_diff16<T>(a + off, b + off);
        }
#pragma unroll
        for (int u = 0; u < MSE_U; ++u)
            if (tb + u * TL < t1) acc += part[u];
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) acc += __shfl_down(acc, off, 64);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = acc;
    __syncthreads();
    if (threadIdx.x == 0) {
        float s = 0.f;
        for (int w = 0; w < (int)((blockDim.x + 63) >> 6); ++w) s += red[w];          // fixed order: deterministic
        partial[p * MSE_SPLIT + sp] = s;
    }
}

__global__ void patch_mse_final_kernel(const float* __restrict__ partial, int32_t P, float inv_count, float* __restrict__ out) {
    const int p = blockIdx.x * blockDim.x + threadIdx.x;
    if (p >= P) return;
    double s = 0.0;
    for (int i = 0; i < MSE_SPLIT; ++i) s += (double)partial[p * MSE_SPLIT + i];
    out[p] = (float)(s * (double)inv_count);
}

}  // namespace pserve

using namespace pserve;

extern "C" {

// both entry points: partial sums of every (patch, chunk) into `partial` [P][16], then one thread per patch
static int patch_mse_launch(const pserve_plan_t* plan, const void* a, const void* b, int32_t C, int dtype, float* partial,
                            float* out, void* stream) {
    PS_REQUIRE(plan && a && b && out, "pserve_patch_mse: NULL argument");
    PS_REQUIRE(dtype == PSERVE_F32 || dtype == PSERVE_BF16, "pserve_patch_mse: unknown dtype %d", dtype);
    const int vn = dtype == PSERVE_BF16 ? 8 : 4;
    PS_REQUIRE(C > 0 && C % vn == 0 && C / vn <= 1024, "pserve_patch_mse: C=%d must be a multiple of %d and at most %d", C, vn, 1024 * vn);
    PS_REQUIRE(((uintptr_t)a & 15) == 0 && ((uintptr_t)b & 15) == 0, "pserve_patch_mse: tensors must be 16-byte aligned");
    hipStream_t st = (hipStream_t)stream;
    const int CV = C / vn;
    int TL = std::max(1, 256 / CV);
    while (TL * CV > 1024) --TL;
    dim3 grid(plan->P, MSE_SPLIT);
    const int nt = (int)cdiv(TL * CV, 64) * 64;
    if (dtype == PSERVE_BF16)
        patch_mse_partial_kernel<uint16_t><<<grid, nt, 0, st>>>((const uint16_t*)a, (const uint16_t*)b, C, plan->S, TL, partial);
    else
        patch_mse_partial_kernel<float><<<grid, nt, 0, st>>>((const float*)a, (const float*)b, C, plan->S, TL, partial);
    PS_TRY(check_launch("patch_mse_partial_kernel"));
    patch_mse_final_kernel<<<(unsigned)cdiv(plan->P, 256), 256, 0, st>>>(partial, plan->P, 1.f / ((float)plan->S * (float)C), out);
    return check_launch("patch_mse_final_kernel");
}

int pserve_patch_mse(const pserve_plan_t* plan, const void* a, const void* b, int32_t C, int dtype, float* out, void* stream) {
    PS_REQUIRE(plan, "pserve_patch_mse: NULL argument");
    return patch_mse_launch(plan, a, b, C, dtype, plan->mse_partial, out, stream);
}

int pserve_patch_mse_static(const pserve_plan_t* plan, const void* a, const void* b, int32_t C, int dtype, float* out,
                            void* stream) {
    PS_REQUIRE(plan, "pserve_patch_mse_static: NULL argument");
    PS_REQUIRE(plan->P <= MSE_STATIC_MAX_PATCHES, "pserve_patch_mse_static: %d patches exceed the fixed scratch of %d patches",
               plan->P, MSE_STATIC_MAX_PATCHES);
    float* partial = nullptr;
    PS_TRY(static_scratch(&partial));
    // every (patch, chunk) entry the second kernel reads is written by the first one: nothing to clear between calls
    return patch_mse_launch(plan, a, b, C, dtype, partial, out, stream);
}

int pserve_cache_sets(const pserve_plan_t* old_plan, const int64_t* old_ids, const pserve_plan_t* new_plan,
                      const int64_t* new_ids, int32_t* req_src, uint8_t* expired, int32_t* patch_src, void* stream) {
    PS_REQUIRE(old_plan && new_plan && old_ids && new_ids && patch_src, "pserve_cache_sets: NULL argument");
    PS_REQUIRE(old_plan->ph == new_plan->ph && old_plan->pw == new_plan->pw,
               "pserve_cache_sets: the two plans use different patch sizes (%dx%d vs %dx%d)", old_plan->ph, old_plan->pw,
               new_plan->ph, new_plan->pw);
    try {
    // ids the cache holds -> caller index in the old batch
    std::unordered_map<int64_t, int32_t> held;
    held.reserve((size_t)old_plan->n * 2);
    for (int j = 0; j < old_plan->n; ++j)
        PS_REQUIRE(held.emplace(old_ids[j], j).second, "pserve_cache_sets: duplicate id %lld in the old batch", (long long)old_ids[j]);
    const auto& perm_o = old_plan->h_tab[PSERVE_TAB_PERM];
    const auto& perm_n = new_plan->h_tab[PSERVE_TAB_PERM];
    const auto& ro_o = old_plan->h_tab[PSERVE_TAB_REQUEST_OFFSET];
    const auto& ro_n = new_plan->h_tab[PSERVE_TAB_REQUEST_OFFSET];
    std::vector<int32_t> slot_of_old(old_plan->n);                   // caller index -> sorted slot (old plan)
    for (int s = 0; s < old_plan->n; ++s) slot_of_old[perm_o[s]] = s;
    std::vector<int32_t> src_of_new(new_plan->n, -1);                // caller index (new) -> caller index (old)
    std::unordered_map<int64_t, int32_t> seen;
    seen.reserve((size_t)new_plan->n * 2);
    for (int i = 0; i < new_plan->n; ++i) {
        PS_REQUIRE(seen.emplace(new_ids[i], i).second, "pserve_cache_sets: duplicate id %lld in the new batch", (long long)new_ids[i]);
        auto it = held.find(new_ids[i]);
        if (it != held.end()) src_of_new[i] = it->second;
    }
    // Common requests keep their patch grid: same resolution in both plans
    std::vector<int32_t> h_src((size_t)new_plan->P, -1);
    for (int s = 0; s < new_plan->n; ++s) {
        const int i = perm_n[s], j = src_of_new[i];
        if (j < 0) continue;
        const int so = slot_of_old[j];
        PS_REQUIRE(old_plan->h_sorted_hw[2 * so] == new_plan->h_sorted_hw[2 * s] &&
                   old_plan->h_sorted_hw[2 * so + 1] == new_plan->h_sorted_hw[2 * s + 1],
                   "pserve_cache_sets: request id %lld changed its resolution", (long long)new_ids[i]);
        const int np = ro_n[s + 1] - ro_n[s];
        for (int k = 0; k < np; ++k) h_src[ro_n[s] + k] = ro_o[so] + k;        // same row-major grid position
    }
    if (req_src) for (int i = 0; i < new_plan->n; ++i) req_src[i] = src_of_new[i];
    if (expired) for (int j = 0; j < old_plan->n; ++j) expired[j] = seen.count(old_ids[j]) ? 0 : 1;
    hipStream_t st = (hipStream_t)stream;
    PS_CHECK_HIP(hipMemcpyAsync(patch_src, h_src.data(), h_src.size() * sizeof(int32_t), hipMemcpyHostToDevice, st));
    PS_CHECK_HIP(hipStreamSynchronize(st));                          // h_src dies with this call
    return PSERVE_OK;
    } catch (const std::bad_alloc&) {                                // nothing may unwind across the C boundary
        set_error("pserve_cache_sets: out of host memory");
        return PSERVE_ENOMEM;
    } catch (...) {
        set_error("pserve_cache_sets: unexpected exception");
        return PSERVE_EINVAL;
    }
}

}  // extern "C"
