// Segmented GroupNorm over the patch batch and the 3x3 halo gather.
//
// GroupNorm statistics of a patch batch must be those of the whole image: mean and
// variance of a group are reduced over ALL patches of the owning request (the patches of
// request s are RequestOffset[s] .. RequestOffset[s+1], "Compressed Sparse Patch Format").
// The halo gather is the pull form of the paper's edge stitching ("Patch Edge Stitcher"):
// border pixels of same-image neighbour patches, zeros where the neighbour is absent
// ("Patch-Tailored Diffusion Operators").
//
// Three kernels for the norm:
//   gn_partial_kernel   per (patch, token chunk): per-group mean and sum of squared deviations
//                       (fp32, shifted sums), 16-byte loads, per-thread channel accumulators,
//                       LDS tree to groups
//   gn_finalize_kernel  per (request, group): the partial moments merged in fp64 (shuffles +
//                       LDS) -> mean, rstd -> per (request, channel) scale and shift
//   gn_apply_kernel     y = x*scale + shift (+SiLU), written plain or into the interior of
//                       the padded patch buffer the convolution reads
// Reductions are deterministic (no float atomics).
#include "kernels.h"

namespace pserve {

template <typename T> struct Vec;
template <> struct Vec<float> { static constexpr int N = 4; };
template <> struct Vec<uint16_t> { static constexpr int N = 8; };

template <typename T>
__device__ __forceinline__ void load_vec(const T* p, float (&v)[Vec<T>::N]);
template <>
__device__ __forceinline__ void load_vec<float>(const float* p, float (&v)[4]) {
    const float4 q = *reinterpret_cast<const float4*>(p);
    v[0] = q.x; v[1] = q.y; v[2] = q.z; v[3] = q.w;
}
template <>
__device__ __forceinline__ void load_vec<uint16_t>(const uint16_t* p, float (&v)[8]) {
    const uint4 q = *reinterpret_cast<const uint4*>(p);
    const uint32_t w[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        v[2 * i] = __uint_as_float(w[i] << 16);
        v[2 * i + 1] = __uint_as_float(w[i] & 0xFFFF0000u);
    }
}
template <typename T>
__device__ __forceinline__ void store_vec(T* p, const float (&v)[Vec<T>::N]);
template <>
__device__ __forceinline__ void store_vec<float>(float* p, const float (&v)[4]) {
    *reinterpret_cast<float4*>(p) = make_float4(v[0], v[1], v[2], v[3]);
}
template <>
__device__ __forceinline__ void store_vec<uint16_t>(uint16_t* p, const float (&v)[8]) {
    uint32_t w[4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
        w[i] = pack_bf16x2(v[2 * i], v[2 * i + 1]);
    *reinterpret_cast<uint4*>(p) = make_uint4(w[0], w[1], w[2], w[3]);
}

// 16 raw bytes of a row now, floats later: lets a kernel issue its row loads before loads it would otherwise wait for
template <typename T>
__device__ __forceinline__ void unpack_vec(const uint4& q, float (&v)[Vec<T>::N]);
template <>
__device__ __forceinline__ void unpack_vec<float>(const uint4& q, float (&v)[4]) {
    v[0] = __uint_as_float(q.x); v[1] = __uint_as_float(q.y); v[2] = __uint_as_float(q.z); v[3] = __uint_as_float(q.w);
}
template <>
__device__ __forceinline__ void unpack_vec<uint16_t>(const uint4& q, float (&v)[8]) {
    const uint32_t w[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        v[2 * i] = __uint_as_float(w[i] << 16);
        v[2 * i + 1] = __uint_as_float(w[i] & 0xFFFF0000u);
    }
}

constexpr int GN_U = 8;     // token rows a thread keeps in flight

// thread (tl, cv): cv = channel vector (fixed channels for the whole kernel), tl = token lane.
// Moments that can be merged (Chan, Golub, LeVeque: combining the moments of two samples): a block leaves, per group,
// the mean and the sum of squared deviations M2 of its n = (tokens of the chunk) x (channels per group) elements.  The
// sums run over x - K with K = the channel's value in the chunk's first token, so that nothing is lost when the mean
// is far from zero (sum of squares minus square of the sum would lose the variance at |mean| >> deviation).
template <typename T>
__global__ void gn_partial_kernel(const T* __restrict__ x, int32_t C, int32_t G, int32_t S, int32_t nsplit,
                                  int32_t TL, float* __restrict__ partial) {
    constexpr int VN = Vec<T>::N;
    extern __shared__ float red[];             // [2][TL][C]
    const int CV = C / VN;
    const int cv = threadIdx.x % CV, tl = threadIdx.x / CV;
    const int p = blockIdx.x, sp = blockIdx.y;
    const int chunk = (S + nsplit - 1) / nsplit;
    const int t0 = sp * chunk, t1 = min(S, t0 + chunk);
    float s1[VN], s2[VN], k0[VN];
#pragma unroll
    for (int e = 0; e < VN; ++e) { s1[e] = 0.f; s2[e] = 0.f; }
    const T* base = x + ((int64_t)p * S) * C + cv * VN;
    load_vec<T>(base + (int64_t)min(t0, S - 1) * C, k0);       // the shift: this channel vector in the chunk's first token
    // up to GN_U independent 16-byte loads in flight per thread; rows past the chunk re-read its last row and are skipped
    for (int tb = t0 + tl; tb < t1; tb += GN_U * TL) {
        float v[GN_U][VN];
#pragma unroll
        for (int u = 0; u < GN_U; ++u) load_vec<T>(base + (int64_t)min(tb + u * TL, t1 - 1) * C, v[u]);
#pragma unroll
        for (int u = 0; u < GN_U; ++u) {
            if (tb + u * TL < t1) {
#pragma unroll
                for (int e = 0; e < VN; ++e) { const float d = v[u][e] - k0[e]; s1[e] += d; s2[e] = fmaf(d, d, s2[e]); }
            }
        }
    }
#pragma unroll
    for (int e = 0; e < VN; ++e) {
        red[tl * C + cv * VN + e] = s1[e];
        red[(TL + tl) * C + cv * VN + e] = s2[e];
    }
    __syncthreads();
    // two short phases instead of one long serial loop per group: first the token lanes of every channel (plain sums:
    // one shift per channel), which leave the channel's mean and M2 over the chunk ...
    const float nt = (float)max(t1 - t0, 0);
    for (int c = threadIdx.x; c < C; c += blockDim.x) {
        float a = 0.f, b = 0.f;
        for (int l = 0; l < TL; ++l) { a += red[l * C + c]; b += red[(TL + l) * C + c]; }
        const float kc = ld_f<T>(x + ((int64_t)p * S + min(t0, S - 1)) * C + c);
        const float inv = nt > 0.f ? 1.f / nt : 0.f;
        red[c] = kc + a * inv;                          // mean of the channel over the chunk
        red[TL * C + c] = fmaxf(b - a * a * inv, 0.f);  // M2 around it
    }
    __syncthreads();
    // ... then the channels of every group (equal counts: mean of the means, M2 by the merge formula; fixed order)
    const int cg = C / G;
    for (int g = threadIdx.x; g < G; g += blockDim.x) {
        float m = 0.f;
        for (int c = g * cg; c < (g + 1) * cg; ++c) m += red[c];
        m /= (float)cg;
        float m2 = 0.f;
        for (int c = g * cg; c < (g + 1) * cg; ++c) { const float d = red[c] - m; m2 += red[TL * C + c] + nt * d * d; }
        float* dst = partial + (((int64_t)p * nsplit + sp) * G + g) * 2;
        dst[0] = m;
        dst[1] = m2;
    }
}

constexpr int GN_FIN_THREADS = 256;

// block = four wavefronts per (request slot s, group g): merges the moments of all partials of the request in fp64.
// Partial i of a patch covers rows(i) = the tokens of chunk i (S split into `nsplit` chunks) times C/G channels;
// sum n_i mean_i and sum (M2_i + n_i mean_i^2) in fp64 give the mean and the M2 of the whole request (the fp64 sums
// carry 16 digits against the eight or so that |mean| / deviation can cost).
// epg = entries per group in a partial row: 1 (moments of whole groups) or C/G (moments of single channels, as the
// split pass leaves them: partial[p][chunk][C][2]).
template <typename T, int THREADS>
__global__ void __launch_bounds__(THREADS)
gn_finalize_kernel(const float* __restrict__ partial, const int32_t* __restrict__ request_offset,
                                   const T* __restrict__ gamma, const T* __restrict__ beta, int32_t C, int32_t G,
                                   int32_t S, int32_t nsplit, int32_t epg, float eps, float* __restrict__ scale_shift) {
    const int s = blockIdx.x, g = blockIdx.y;
    const int p0 = request_offset[s], p1 = request_offset[s + 1];
    const int items = (p1 - p0) * nsplit * epg;
    const int cg = C / G;
    const int chunk = (S + nsplit - 1) / nsplit;
    double a = 0.0, b = 0.0;
#pragma unroll 4
    for (int i = threadIdx.x; i < items; i += THREADS) {      // independent loads: several in flight per thread
        const int row = i / epg, e = i - row * epg;
        const float* src = partial + (((int64_t)p0 * nsplit + row) * G * epg + g * epg + e) * 2;
        const int sp = row % nsplit;
        const double n = (double)max(min(S, (sp + 1) * chunk) - sp * chunk, 0) * (cg / epg);
        const double m = (double)src[0];
        a += n * m;
        b += (double)src[1] + n * m * m;
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        a += __shfl_down(a, off, 64);
        b += __shfl_down(b, off, 64);
    }
    __shared__ double red[THREADS / 64][2];
    if ((threadIdx.x & 63) == 0) { red[threadIdx.x >> 6][0] = a; red[threadIdx.x >> 6][1] = b; }
    __syncthreads();
    a = 0.0;
    b = 0.0;
#pragma unroll
    for (int w = 0; w < THREADS / 64; ++w) { a += red[w][0]; b += red[w][1]; }    // fixed order: deterministic
    const double cnt = (double)(p1 - p0) * S * cg;
    const double mean = a / cnt;
    double var = b / cnt - mean * mean;
    var = var > 0.0 ? var : 0.0;
    const double rstd = 1.0 / sqrt(var + (double)eps);
    for (int c = g * cg + threadIdx.x; c < (g + 1) * cg; c += THREADS) {
        const double sc = rstd * (double)ld_f<T>(gamma + c);
        float* dst = scale_shift + ((int64_t)s * C + c) * 2;
        dst[0] = (float)sc;
        dst[1] = (float)((double)ld_f<T>(beta + c) - mean * sc);
    }
}

// v * sigmoid(v) with the hardware reciprocal (1 ulp): a true division expands to ten instructions per element
__device__ __forceinline__ float silu_f(float v) { return v * __builtin_amdgcn_rcpf(1.f + __expf(-v)); }

// Edge stitching fused into the normalisation (the push form of the paper's "Patch Edge Stitcher"): a border
// token's normalised value is also written into the ring slot of every same-image neighbour patch that needs
// it; where that neighbour is absent (image edge) the token zero-fills the matching ring slot of its OWN patch.
// Every ring slot of every patch is written by exactly one thread, so there is no race and no extra pass.
template <typename T>
__device__ __forceinline__ void stitch_store(T* __restrict__ out, const int32_t (&nb)[8], const PatchGeom& gm,
                                             int p, int y, int x, int C, int coff, const float (&v)[Vec<T>::N]) {
    if (y != 0 && y != gm.ph - 1 && x != 0 && x != gm.pw - 1) return;
    float z[Vec<T>::N];
#pragma unroll
    for (int e = 0; e < Vec<T>::N; ++e) z[e] = 0.f;
    int k = 0;
#pragma unroll
    for (int dy = -1; dy <= 1; ++dy)
#pragma unroll
        for (int dx = -1; dx <= 1; ++dx) {
            if (dy == 0 && dx == 0) continue;
            const bool on = (dy == 0 || (dy < 0 ? y == 0 : y == gm.ph - 1)) && (dx == 0 || (dx < 0 ? x == 0 : x == gm.pw - 1));
            if (on) {
                const int q = nb[k];
                if (q >= 0)
                    store_vec<T>(out + ((int64_t)q * gm.pS + (y - dy * gm.ph + 1) * gm.ppw + (x - dx * gm.pw + 1)) * C + coff, v);
                else
                    store_vec<T>(out + ((int64_t)p * gm.pS + (y + dy + 1) * gm.ppw + (x + dx + 1)) * C + coff, z);
            }
            ++k;
        }
}

// rim_only (padded output): patches with rim_only[p] != 0 are not convolved themselves (their result is reused); only
// their border tokens are normalised, because the neighbours' rings need them.
template <typename T, bool SILU, bool PADDED, bool STITCH>
__global__ void gn_apply_kernel(const T* __restrict__ x, const float* __restrict__ scale_shift,
                                const int32_t* __restrict__ owner, const int32_t* __restrict__ neighbour, PatchGeom gm,
                                int32_t C, int32_t nsplit, int32_t TL, ActiveList act, const uint8_t* __restrict__ rim_only,
                                T* __restrict__ out) {
    constexpr int VN = Vec<T>::N;
    int p = blockIdx.x;
    if (act.active) {
        if (p >= *act.count) return;
        p = act.active[p];
    }
    if (PADDED && rim_only && rim_only[p]) {
        // border token b of the patch: top row, bottom row, then left / right column of the rows between
        const int CVb = C / VN, cvb = threadIdx.x % CVb;
        const int nb_tok = gm.ph > 1 ? 2 * gm.pw + 2 * (gm.ph - 2) : gm.pw;
        // a few blocks with about four border tokens per thread row (as for whole patches); the others leave at once
        const int per = max((nb_tok + nsplit - 1) / nsplit, 4 * TL);
        const int b0 = blockIdx.y * per, b1 = min(nb_tok, b0 + per);
        if (b0 >= b1) return;
        float sc[VN], sh[VN];
        const float* ss = scale_shift + ((int64_t)owner[p] * C + cvb * VN) * 2;
#pragma unroll
        for (int e = 0; e < VN; ++e) { sc[e] = scale_shift ? ss[2 * e] : 1.f; sh[e] = scale_shift ? ss[2 * e + 1] : 0.f; }
        int32_t nbr[8];
#pragma unroll
        for (int k = 0; k < 8; ++k) nbr[k] = STITCH ? neighbour[8 * p + k] : -1;
        for (int b = b0 + (int)threadIdx.x / CVb; b < b1; b += TL) {
            int y, xx;
            if (b < gm.pw) { y = 0; xx = b; }
            else if (b < 2 * gm.pw) { y = gm.ph - 1; xx = b - gm.pw; }
            else { const int r = b - 2 * gm.pw; y = 1 + (r >> 1); xx = (r & 1) ? gm.pw - 1 : 0; }
            float v[VN];
            load_vec<T>(x + ((int64_t)p * gm.S + y * gm.pw + xx) * C + cvb * VN, v);
#pragma unroll
            for (int e = 0; e < VN; ++e) {
                v[e] = fmaf(v[e], sc[e], sh[e]);
                if (SILU) v[e] = silu_f(v[e]);
            }
            store_vec<T>(out + ((int64_t)p * gm.pS + (y + 1) * gm.ppw + xx + 1) * C + cvb * VN, v);
            if (STITCH) stitch_store<T>(out, nbr, gm, p, y, xx, C, cvb * VN, v);
        }
        return;
    }
    const int CV = C / VN;
    const int cv = threadIdx.x % CV, tl = threadIdx.x / CV;
    const int sp = blockIdx.y;
    const int chunk = (gm.S + nsplit - 1) / nsplit;
    const int t0 = sp * chunk, t1 = min(gm.S, t0 + chunk);
    // Rows of this thread: t0 + tl + k*TL.  Their pixel coordinates and offsets advance by additions (a division and
    // 64-bit multiplications per row were a third of the kernel's vector instructions).
    const int pw = gm.pw;
    const int dyy = TL / pw, dxx = TL - dyy * pw;                       // one row step in pixel rows / columns
    const int step_in = TL * C;
    const int step_out = PADDED ? (dyy * gm.ppw + dxx) * C : TL * C;
    const int wrap_out = PADDED ? (gm.ppw - pw) * C : 0;                // extra when the column wraps into the next pixel row
    int tb = t0 + tl;
    int py = tb / pw, px = tb - py * pw;
    const T* xin = x + ((int64_t)p * gm.S) * C + cv * VN;
    T* po = out + ((int64_t)p * (PADDED ? gm.pS : gm.S)) * C + cv * VN;
    int in_off = tb * C;
    int out_off = (PADDED ? (py + 1) * gm.ppw + px + 1 : tb) * C;
    const int last_in = (t1 - 1) * C;
    // The row loads of the first batch go first: they depend on the patch only, while scale / shift hang on the
    // owner table (two dependent loads).  Up to GN_U independent 16-byte loads in flight per thread; rows past the
    // chunk re-read its last row and are skipped.
    uint4 raw[GN_U];
    if (tb < t1) {
#pragma unroll
        for (int u = 0; u < GN_U; ++u) raw[u] = *reinterpret_cast<const uint4*>(xin + min(in_off + u * step_in, last_in));
    }
    float sc[VN], sh[VN];
    if (scale_shift) {
        const int s = owner[p];
        const float* ss = scale_shift + ((int64_t)s * C + cv * VN) * 2;
#pragma unroll
        for (int e = 0; e < VN; ++e) { sc[e] = ss[2 * e]; sh[e] = ss[2 * e + 1]; }
    } else {                                    // no table: plain copy into the padded layout (with the rims)
#pragma unroll
        for (int e = 0; e < VN; ++e) { sc[e] = 1.f; sh[e] = 0.f; }
    }
    int32_t nb[8];                              // neighbour patches, read once (no dependent loads behind the stores)
#pragma unroll
    for (int k = 0; k < 8; ++k) nb[k] = (PADDED && STITCH) ? neighbour[8 * p + k] : -1;
    for (; tb < t1; tb += GN_U * TL) {
        float v[GN_U][VN];
#pragma unroll
        for (int u = 0; u < GN_U; ++u) unpack_vec<T>(raw[u], v[u]);
        in_off += GN_U * step_in;
        if (tb + GN_U * TL < t1) {              // next batch in flight while this one is finished
#pragma unroll
            for (int u = 0; u < GN_U; ++u) raw[u] = *reinterpret_cast<const uint4*>(xin + min(in_off + u * step_in, last_in));
        }
#pragma unroll
        for (int u = 0; u < GN_U; ++u) {
            if (tb + u * TL < t1) {
#pragma unroll
                for (int e = 0; e < VN; ++e) {
                    v[u][e] = fmaf(v[u][e], sc[e], sh[e]);
                    if (SILU) v[u][e] = silu_f(v[u][e]);
                }
                store_vec<T>(po + out_off, v[u]);
                if (PADDED && STITCH) stitch_store<T>(out, nb, gm, p, py, px, C, cv * VN, v[u]);
            }
            // next row of this thread
            px += dxx;
            py += dyy;
            out_off += step_out;
            if (px >= pw) { px -= pw; ++py; out_off += wrap_out; }
        }
    }
}

// ---- per-token LayerNorm over the channels -------------------------------------------------------------------
// LPT lanes (a power of two) share a token; lane `sub` holds the 16-byte vectors sub, sub + LPT, ... (VPL of them) of
// the row in registers.  Mean, then variance around it (two passes over the registers), each reduced by a butterfly
// over the LPT lanes; fp32 throughout.  One 16-byte load and one 16-byte store per vector: 2*b*C bytes per token.
template <typename T, int VPL>
__global__ void __launch_bounds__(256)
layer_norm_kernel(const T* __restrict__ x, const T* __restrict__ gamma, const T* __restrict__ beta,
                  const float* __restrict__ mod, int64_t mod_ld, const int32_t* __restrict__ owner, int32_t C, int32_t S,
                  int32_t LPT, float eps, ActiveList act, T* __restrict__ out) {
    constexpr int VN = Vec<T>::N;
    int p = blockIdx.x;
    if (act.active) {
        if (p >= *act.count) return;
        p = act.active[p];
    }
    const int CV = C / VN;
    const int sub = threadIdx.x % LPT, tl = threadIdx.x / LPT, tpb = blockDim.x / LPT;
    uint4 graw[VPL], braw[VPL];
    const float* mrow = mod ? mod + (int64_t)owner[p] * mod_ld : nullptr;     // adaptive form: [shift | scale] of the request
    if (!mod) {
#pragma unroll
        for (int k = 0; k < VPL; ++k) {
            const int cv = min(sub + k * LPT, CV - 1);
            graw[k] = *reinterpret_cast<const uint4*>(gamma + cv * VN);
            braw[k] = *reinterpret_cast<const uint4*>(beta + cv * VN);
        }
    }
    const float inv_c = 1.f / (float)C;
    for (int t = blockIdx.y * tpb + tl; t < S; t += gridDim.y * tpb) {
        const int64_t row = ((int64_t)p * S + t) * C;
        float v[VPL][VN];
        float s1 = 0.f;
#pragma unroll
        for (int k = 0; k < VPL; ++k) {
            const int cv = sub + k * LPT;
            if (cv < CV) {
                load_vec<T>(x + row + cv * VN, v[k]);
#pragma unroll
                for (int e = 0; e < VN; ++e) s1 += v[k][e];
            }
        }
        for (int m = LPT >> 1; m > 0; m >>= 1) s1 += __shfl_xor(s1, m, 64);
        const float mean = s1 * inv_c;
        float s2 = 0.f;
#pragma unroll
        for (int k = 0; k < VPL; ++k) {
            if (sub + k * LPT < CV) {
#pragma unroll
                for (int e = 0; e < VN; ++e) { v[k][e] -= mean; s2 = fmaf(v[k][e], v[k][e], s2); }
            }
        }
        for (int m = LPT >> 1; m > 0; m >>= 1) s2 += __shfl_xor(s2, m, 64);
        const float rstd = 1.f / sqrtf(s2 * inv_c + eps);
#pragma unroll
        for (int k = 0; k < VPL; ++k) {
            const int cv = sub + k * LPT;
            if (cv < CV) {
                float g[VN], b[VN];
                if (mod) {
#pragma unroll
                    for (int e = 0; e < VN; ++e) { b[e] = mrow[cv * VN + e]; g[e] = 1.f + mrow[C + cv * VN + e]; }
                } else {
                    unpack_vec<T>(graw[k], g);
                    unpack_vec<T>(braw[k], b);
                }
#pragma unroll
                for (int e = 0; e < VN; ++e) v[k][e] = fmaf(v[k][e] * rstd, g[e], b[e]);
                store_vec<T>(out + row + cv * VN, v[k]);
            }
        }
    }
}

// one thread per (ring entry, channel vector) of an active patch
template <typename T>
__global__ void halo_gather_kernel(T* __restrict__ apad, const int32_t* __restrict__ halo_src, PatchGeom gm,
                                   int32_t C, int32_t ring, ActiveList act) {
    constexpr int VN = Vec<T>::N;
    int p = blockIdx.x;
    if (act.active) {
        if (p >= *act.count) return;
        p = act.active[p];
    }
    const int CV = C / VN;
    const int items = ring * CV;
    for (int i = blockIdx.y * blockDim.x + threadIdx.x; i < items; i += gridDim.y * blockDim.x) {
        const int k = i / CV, cv = i - k * CV;
        int y, x;                          // ring pixel relative to the patch origin
        if (k < gm.pw + 2) { y = -1; x = k - 1; }
        else if (k < 2 * (gm.pw + 2)) { y = gm.ph; x = k - (gm.pw + 2) - 1; }
        else if (k < 2 * (gm.pw + 2) + gm.ph) { y = k - 2 * (gm.pw + 2); x = -1; }
        else { y = k - 2 * (gm.pw + 2) - gm.ph; x = gm.pw; }
        const int tok = halo_src[(int64_t)p * ring + k];
        uint4 v = make_uint4(0, 0, 0, 0);
        if (tok >= 0) {
            const int q = tok / gm.S, r = tok - q * gm.S;
            const int ys = r / gm.pw, xs = r - ys * gm.pw;
            v = *reinterpret_cast<const uint4*>(apad + ((int64_t)q * gm.pS + (ys + 1) * gm.ppw + xs + 1) * C + cv * VN);
        }
        *reinterpret_cast<uint4*>(apad + ((int64_t)p * gm.pS + (y + 1) * gm.ppw + x + 1) * C + cv * VN) = v;
    }
}

// ---- host side ---------------------------------------------------------------------------------
static int norm_layout(int32_t C, int dtype, int* CV, int* TL) {
    const int vn = dtype == PSERVE_BF16 ? 8 : 4;
    PS_REQUIRE(C % vn == 0, "GroupNorm: C=%d must be a multiple of %d for this dtype", C, vn);
    *CV = C / vn;
    PS_REQUIRE(*CV <= 1024, "GroupNorm: C=%d too wide", C);
    int tl = (256 + *CV / 2) / *CV;
    if (tl < 1) tl = 1;
    while (tl * *CV > 1024) --tl;
    *TL = tl;
    return PSERVE_OK;
}

int gn_stats(const GroupNormArgs& a, const PatchGeom& g, int dtype, hipStream_t st) {
    int CV, TL;
    PS_TRY(norm_layout(a.C, dtype, &CV, &TL));
    PS_REQUIRE(a.C % a.G == 0, "GroupNorm: C %% G != 0");
    const size_t lds = sizeof(float) * 2 * TL * a.C;
    PS_REQUIRE(lds <= 64 * 1024, "GroupNorm: C=%d too wide for the reduction buffer", a.C);
    dim3 grid(g.P, a.nsplit);
    if (dtype == PSERVE_BF16)
        gn_partial_kernel<uint16_t><<<grid, TL * CV, lds, st>>>((const uint16_t*)a.x, a.C, a.G, g.S, a.nsplit, TL, a.partial);
    else
        gn_partial_kernel<float><<<grid, TL * CV, lds, st>>>((const float*)a.x, a.C, a.G, g.S, a.nsplit, TL, a.partial);
    PS_TRY(check_launch("gn_partial_kernel"));
    return gn_finalize(a, g, dtype, a.nsplit, st, false);
}

int gn_finalize(const GroupNormArgs& a, const PatchGeom& g, int dtype, int32_t slots, hipStream_t st, bool per_channel) {
    dim3 fgrid(a.n, a.G);
    const int epg = per_channel ? a.C / a.G : 1;
    // per-channel entries: C / G times as many per (request, group): 1,024 threads (a 256^2 latent in 32 x 32 patches
    // has 10,240 of them; with 256 threads that block alone took 27 us)
#define PS_FIN(T, TH)                                                                                              \
    gn_finalize_kernel<T, TH><<<fgrid, TH, 0, st>>>(a.partial, a.request_offset, (const T*)a.gamma, (const T*)a.beta, a.C, \
                                                    a.G, g.S, slots, epg, a.eps, a.scale_shift)
    if (dtype == PSERVE_BF16) { if (per_channel) PS_FIN(uint16_t, 1024); else PS_FIN(uint16_t, GN_FIN_THREADS); }
    else { if (per_channel) PS_FIN(float, 1024); else PS_FIN(float, GN_FIN_THREADS); }
#undef PS_FIN
    return check_launch("gn_finalize_kernel");
}

constexpr int APPLY_ROWS = 4;        // rows per thread of the apply pass (measured: 1-2 too many blocks, 6-8 too few)

template <typename T>
static void launch_apply(const GroupNormArgs& a, const PatchGeom& g, bool silu, bool padded, bool stitch, void* out,
                         ActiveList act, int CV, int TL, hipStream_t st) {
    // Own chunking (independent of the statistics pass): about APPLY_ROWS rows per thread.  Many short blocks are
    // dispatched over time, so some load while others compute or store; with few long blocks every wavefront of
    // the chip is in the same phase at once.
    const int nsplit = (int)std::max<int64_t>(1, std::min<int64_t>(cdiv(g.S, (int64_t)APPLY_ROWS * TL), 65535));
    dim3 grid(g.P, nsplit);
    const int nt = TL * CV;
#define PS_APPLY(SI, PA, ST)                                                                                      \
    gn_apply_kernel<T, SI, PA, ST><<<grid, nt, 0, st>>>((const T*)a.x, a.scale_shift, a.owner, a.neighbour, g, a.C, \
                                                        nsplit, TL, act, a.rim_only, (T*)out)
    if (silu && padded && stitch) PS_APPLY(true, true, true);
    else if (padded && stitch) PS_APPLY(false, true, true);
    else if (silu && padded) PS_APPLY(true, true, false);
    else if (silu) PS_APPLY(true, false, false);
    else if (padded) PS_APPLY(false, true, false);
    else PS_APPLY(false, false, false);
#undef PS_APPLY
}

int gn_apply(const GroupNormArgs& a, const PatchGeom& g, int dtype, bool silu, bool padded, bool stitch, void* out,
             ActiveList act, hipStream_t st) {
    int CV, TL;
    PS_TRY(norm_layout(a.C, dtype, &CV, &TL));
    PS_REQUIRE(!stitch || (padded && a.neighbour && !act.active), "gn_apply: stitching needs the padded layout and all patches");
    if (dtype == PSERVE_BF16) launch_apply<uint16_t>(a, g, silu, padded, stitch, out, act, CV, TL, st);
    else launch_apply<float>(a, g, silu, padded, stitch, out, act, CV, TL, st);
    return check_launch("gn_apply_kernel");
}

template <typename T>
static void launch_layer_norm(const void* x, const void* gamma, const void* beta, const float* mod, int64_t mod_ld,
                              const int32_t* owner, int32_t C, float eps, const PatchGeom& g, void* out, ActiveList act,
                              int LPT, int VPL, hipStream_t st) {
    const int tpb = 256 / LPT;
    // one token per lane group while that gives at most ~16 blocks per CU, else more tokens per group
    int64_t per = 1;
    while (per < 8 && g.P * cdiv(g.S, tpb * per) > 4096) per *= 2;
    dim3 grid(g.P, (unsigned)std::max<int64_t>(1, std::min<int64_t>(cdiv(g.S, tpb * per), 65535)));
#define PS_LN(V) case V: layer_norm_kernel<T, V><<<grid, 256, 0, st>>>((const T*)x, (const T*)gamma, (const T*)beta, mod, mod_ld, owner, C, g.S, LPT, eps, act, (T*)out); break
    switch (VPL) { PS_LN(1); PS_LN(2); PS_LN(3); PS_LN(4); PS_LN(5); PS_LN(6); PS_LN(7); PS_LN(8); }
#undef PS_LN
}

int layer_norm(const void* x, const void* gamma, const void* beta, const float* mod, int64_t mod_ld, const int32_t* owner,
               int32_t C, float eps, const PatchGeom& g, int dtype, void* out, ActiveList act, hipStream_t st) {
    PS_REQUIRE((gamma && beta) || (mod && owner), "LayerNorm: neither gamma / beta nor a modulation table");
    if (gamma) mod = nullptr;
    const int vn = dtype == PSERVE_BF16 ? 8 : 4;
    PS_REQUIRE(C % vn == 0, "LayerNorm: C=%d must be a multiple of %d for this dtype", C, vn);
    const int CV = C / vn;
    PS_REQUIRE(CV <= 512, "LayerNorm: C=%d too wide", C);
    // lanes per token: the power of two that wastes the fewest vector slots (ties: more lanes)
    int LPT = 64, VPL = (int)cdiv(CV, 64), waste = VPL * 64 - CV;
    for (int l = 32; l >= 1; l >>= 1) {
        const int v = (int)cdiv(CV, l);
        if (v <= 8 && v * l - CV < waste) { LPT = l; VPL = v; waste = v * l - CV; }
    }
    if (dtype == PSERVE_BF16) launch_layer_norm<uint16_t>(x, gamma, beta, mod, mod_ld, owner, C, eps, g, out, act, LPT, VPL, st);
    else launch_layer_norm<float>(x, gamma, beta, mod, mod_ld, owner, C, eps, g, out, act, LPT, VPL, st);
    return check_launch("layer_norm_kernel");
}

int halo_gather(void* apad, const int32_t* halo_src, const PatchGeom& g, int32_t C, int32_t ring, int dtype,
                ActiveList act, hipStream_t st) {
    int CV, TL;
    PS_TRY(norm_layout(C, dtype, &CV, &TL));
    const int items = ring * CV;
    dim3 grid(g.P, (unsigned)std::max<int64_t>(1, std::min<int64_t>(cdiv(items, 256 * 4), 64)));
    if (dtype == PSERVE_BF16)
        halo_gather_kernel<uint16_t><<<grid, 256, 0, st>>>((uint16_t*)apad, halo_src, g, C, ring, act);
    else
        halo_gather_kernel<float><<<grid, 256, 0, st>>>((float*)apad, halo_src, g, C, ring, act);
    return check_launch("halo_gather_kernel");
}

}  // namespace pserve
