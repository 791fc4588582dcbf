// Per-image variable-length attention over the patch batch.
//
// Self-attention needs every token of the OWN image as key/value ("Patch-based
// Self-Attention Module").  The paper rebuilds full images and batches them by resolution;
// because attention carries no positional term inside the block, the token order within an
// image does not matter, so the patch-major token matrix is used as it is: the keys of a
// query token are the contiguous token range cu_seqlens[s] .. cu_seqlens[s+1] of its request
// slot s (RequestOffset of the CSP format times the tokens per patch).  Cross-attention
// ("pixel-wise" operator) attends to the request's own text tokens.
//
// Softmax runs in base 2 on logits pre-multiplied by log2(e)/sqrt(d) (done by the Q projection).
#include "kernels.h"

namespace pserve {

// ---- plain reference kernel: one wavefront per (query token, head), keys spread over lanes ------
template <typename T, int DMAX>
__global__ void __launch_bounds__(256)
attn_simple_kernel(AttnArgs a) {
    __shared__ float sQ[4][DMAX];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int64_t item = (int64_t)blockIdx.x * 4 + wave;
    const int ri = (int)(item / a.heads), h = (int)(item - (int64_t)ri * a.heads);
    const int S = a.geom.S;
    int64_t rows = (int64_t)a.geom.P * S;
    if (a.act.active) rows = (int64_t)(*a.act.count) * S;
    const bool live = ri < rows;            // wave-uniform
    int64_t tok = 0;
    int p = 0;
    if (live) {
        const int pi = ri / S;
        p = a.act.active ? a.act.active[pi] : pi;
        tok = (int64_t)p * S + (ri - pi * S);
    }
    const int d = a.d;
    const T* Q = (const T*)a.Q;
    const T* K = (const T*)a.K;
    const T* V = (const T*)a.V;
    if (live)
        for (int c = lane; c < d; c += 64) sQ[wave][c] = ld_f<T>(Q + tok * a.C + h * d + c);
    __syncthreads();
    if (!live) return;
    const int s = a.owner[p];
    int64_t k0, nk;
    if (a.cross_len) { k0 = (int64_t)a.perm[s] * a.cross_ld; nk = a.cross_len; }
    else { k0 = a.cu_seqlens[s]; nk = a.seq_len ? a.seq_len[s] : a.cu_seqlens[s + 1] - k0; }

    float m = -INFINITY, l = 0.f;
    float acc[DMAX];
#pragma unroll
    for (int c = 0; c < DMAX; ++c) acc[c] = 0.f;
    for (int64_t j = lane; j < nk; j += 64) {
        const int64_t kr = k0 + j;
        const T* kp = K + kr * a.C + h * d;
        float sc = 0.f;
#pragma unroll
        for (int c = 0; c < DMAX; ++c)
            if (c < d) sc = fmaf(sQ[wave][c], ld_f<T>(kp + c), sc);
        const float mn = fmaxf(m, sc);
        const float corr = exp2f(m - mn), pr = exp2f(sc - mn);
        l = l * corr + pr;
        m = mn;
#pragma unroll
        for (int c = 0; c < DMAX; ++c)
            if (c < d) {
                const float v = a.v_transposed ? ld_f<T>(V + (int64_t)(h * d + c) * a.ldv + kr)
                                               : ld_f<T>(V + kr * a.ldv + h * d + c);
                acc[c] = fmaf(pr, v, acc[c] * corr);
            }
    }
    float mall = m;
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) mall = fmaxf(mall, __shfl_xor(mall, off, 64));
    const float sc = (m == -INFINITY) ? 0.f : exp2f(m - mall);
    float lall = l * sc;
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) lall += __shfl_xor(lall, off, 64);
    const float inv = 1.f / lall;
    T* O = (T*)a.O;
#pragma unroll
    for (int c = 0; c < DMAX; ++c) {
        float v = acc[c] * sc;
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
        if (c < d && lane == (c & 63)) st_f<T>(O + tok * a.C + h * d + c, v * inv);
    }
}

int attention_mfma_bf16(const AttnArgs& a, hipStream_t st, bool* handled);     // attn_mfma.hip

int attention(const AttnArgs& a, int dtype, int mode, hipStream_t st) {
    PS_REQUIRE(a.d > 0 && a.d <= 128, "attention: head dim %d not supported (max 128)", a.d);
    if (mode == 0 && dtype == PSERVE_BF16) {
        bool handled = false;
        PS_TRY(attention_mfma_bf16(a, st, &handled));
        if (handled) return PSERVE_OK;
    }
    const int64_t items = (int64_t)a.geom.P * a.geom.S * a.heads;
    const unsigned grid = (unsigned)cdiv(items, 4);
#define PS_ATTN(TT, DM) attn_simple_kernel<TT, DM><<<grid, 256, 0, st>>>(a)
    if (dtype == PSERVE_BF16) {
        if (a.d <= 32) PS_ATTN(uint16_t, 32); else if (a.d <= 64) PS_ATTN(uint16_t, 64); else PS_ATTN(uint16_t, 128);
    } else {
        if (a.d <= 32) PS_ATTN(float, 32); else if (a.d <= 64) PS_ATTN(float, 64); else PS_ATTN(float, 128);
    }
#undef PS_ATTN
    return check_launch("attn_simple_kernel");
}

}  // namespace pserve
