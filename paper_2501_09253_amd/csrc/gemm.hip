// GEMM / implicit-GEMM 3x3 convolution over the patch batch, and weight packing.
//
// out[t][co] = bias[co] + sum_{tap, ci} a[nbr(t, tap)][ci] * W[co][ci][tap]  (+ residual)
// The 3x3 convolution reads the padded patch buffer [P][ph+2][pw+2][C] whose one-pixel ring
// was filled from same-image neighbours (zeros at image edges), so every patch is a
// self-contained tile and the nine taps are nine shifted views of it (patch-based
// convolution, "Patch-Tailored Diffusion Operators").  Pixel-wise operators (linear layers,
// feed-forward, attention projections) are the one-tap case and run on the patch batch
// unchanged.
//
// Packed weights: B[tap][n][k], k contiguous (conv W[co][ci][ky][kx] -> tap = ky*3+kx;
// linear W[k][n] -> transposed).  Accumulation is fp32.
#include "kernels.h"

namespace pserve {

// ---- row / column addressing shared by the kernels ------------------------------------------------
struct RowInfo {
    int64_t tok;       // input row id
    int64_t out_row;   // row id used for output / residual addressing
    int64_t a_off;     // element offset of the row's first A element (tap 0)
    bool valid;
};

__device__ __forceinline__ RowInfo row_info(const GemmArgs& a, int ri) {
    RowInfo r;
    int64_t tok = ri;
    bool valid;
    if (a.tokens_are_rows && a.act.active) {
        const int cnt = *a.act.count;
        const int pi = ri / a.geom.S;
        valid = pi < cnt;
        tok = valid ? (int64_t)a.act.active[pi] * a.geom.S + (ri - pi * a.geom.S) : 0;
    } else {
        valid = ri < a.M;
        if (!valid) tok = 0;
    }
    r.out_row = (!a.tokens_are_rows && a.row_group > 0) ? (tok / a.row_group) * a.row_group_pad + tok % a.row_group : tok;
    r.tok = tok;
    r.valid = valid;
    if (a.conv) {
        const int p = (int)(tok / a.geom.S), q = (int)(tok - (int64_t)p * a.geom.S);
        const int y = q / a.geom.pw, x = q - y * a.geom.pw;
        const int am = a.a_mul ? a.a_mul : 1;
        r.a_off = ((int64_t)p * a.geom.pS + (am * y + a.a_dy) * a.geom.ppw + am * x + a.a_dx) * a.lda;
        if (a.o_mul) r.out_row = (int64_t)p * a.o_S + (a.o_mul * y + a.o_dy) * a.o_pw + a.o_mul * x + a.o_dx;
    } else {
        r.a_off = tok * a.lda;
    }
    return r;
}

// tanh form: v/2 (1 + tanh(sqrt(2/pi) (v + 0.044715 v^3)))
__device__ __forceinline__ float gelu_tanh_f(float v) {
    return 0.5f * v * (1.f + tanhf(0.7978845608028654f * (v + 0.044715f * v * v * v)));
}
__device__ __forceinline__ float gelu_f(float v) { return 0.5f * v * (1.f + erff(v * 0.70710678118654752f)); }

template <typename T>
__device__ __forceinline__ void route_store(const GemmArgs& a, int64_t tok, int col, float v) {
    const int sg = col / a.seg_cols, c = col - sg * a.seg_cols;
    const GemmSeg& s = a.seg[sg];
    v *= s.scale;
    T* o = (T*)s.ptr;
    if (s.transposed) st_f<T>(o + (int64_t)c * s.ld + tok, v);
    else st_f<T>(o + tok * s.ld + c, v);
}

// ---- plain reference kernel: 64x64 tile, fp32 FMA, any shape --------------------------------------
template <typename T, bool GEGLU>
__global__ void __launch_bounds__(256)
gemm_simple_kernel(GemmArgs a) {
    constexpr int BM = 64, BN = 64, BK = 16;
    constexpr int NB = GEGLU ? 2 : 1;                 // B tiles per block (value + gate)
    __shared__ float sA[BK][BM + 1];
    __shared__ float sB[NB][BK][BN + 1];
    __shared__ int64_t s_aoff[BM];
    __shared__ int64_t s_tok[BM];
    __shared__ int s_valid[BM];
    const int tid = threadIdx.x;
    const int m0 = blockIdx.x * BM;
    const int n0 = blockIdx.y * BN;                   // output column (GEGLU: in F space)
    if (a.tokens_are_rows && a.act.active && m0 >= *a.act.count * a.geom.S) return;
    if (tid < BM) {
        const RowInfo r = row_info(a, m0 + tid);
        s_aoff[tid] = r.a_off;
        s_tok[tid] = r.out_row;
        s_valid[tid] = r.valid;
    }
    __syncthreads();
    const T* A = (const T*)a.A;
    const T* B = (const T*)a.B;
    const int tx = tid & 15, ty = tid >> 4;
    float acc[NB][4][4] = {};
    for (int tap = 0; tap < a.taps; ++tap) {
        const int tw = a.tap_w ? a.tap_w : 3;
        const int64_t tap_off = a.conv ? ((int64_t)(tap / tw) * a.geom.ppw + (tap % tw)) * a.lda : 0;
        for (int k0 = 0; k0 < a.K; k0 += BK) {
            for (int i = tid; i < BM * BK; i += 256) {
                const int m = i / BK, k = i - m * BK;
                float v = 0.f;
                if (s_valid[m] && k0 + k < a.K) v = ld_f<T>(A + s_aoff[m] + tap_off + k0 + k);
                sA[k][m] = v;
            }
            for (int h = 0; h < NB; ++h)
                for (int i = tid; i < BN * BK; i += 256) {
                    const int n = i / BK, k = i - n * BK;
                    // GEGLU: packed columns hold [GROUP values | GROUP gates] per group
                    int col = n0 + n;
                    bool ok = col < (GEGLU ? a.N / 2 : a.N);
                    if (GEGLU) col = (col / GEGLU_GROUP) * 2 * GEGLU_GROUP + h * GEGLU_GROUP + col % GEGLU_GROUP;
                    float v = 0.f;
                    if (ok && k0 + k < a.K) v = ld_f<T>(B + ((int64_t)tap * a.N + col) * a.K + k0 + k);
                    sB[h][k][n] = v;
                }
            __syncthreads();
#pragma unroll
            for (int k = 0; k < BK; ++k) {
                float av[4], bv[NB][4];
#pragma unroll
                for (int i = 0; i < 4; ++i) av[i] = sA[k][ty * 4 + i];
#pragma unroll
                for (int h = 0; h < NB; ++h)
#pragma unroll
                    for (int j = 0; j < 4; ++j) bv[h][j] = sB[h][k][tx * 4 + j];
#pragma unroll
                for (int h = 0; h < NB; ++h)
#pragma unroll
                    for (int i = 0; i < 4; ++i)
#pragma unroll
                        for (int j = 0; j < 4; ++j) acc[h][i][j] = fmaf(av[i], bv[h][j], acc[h][i][j]);
            }
            __syncthreads();
        }
    }
    const int ncols = GEGLU ? a.N / 2 : a.N;
    for (int i = 0; i < 4; ++i) {
        const int m = ty * 4 + i;
        if (!s_valid[m]) continue;
        const int64_t tok = s_tok[m];
        for (int j = 0; j < 4; ++j) {
            const int col = n0 + tx * 4 + j;
            if (col >= ncols) continue;
            float v;
            if (GEGLU) {
                const int pc = (col / GEGLU_GROUP) * 2 * GEGLU_GROUP + col % GEGLU_GROUP;
                const float val = acc[0][i][j] + (a.bias ? a.bias[pc] : 0.f);
                const float gate = acc[NB - 1][i][j] + (a.bias ? a.bias[pc + GEGLU_GROUP] : 0.f);
                v = val * gelu_f(gate);
                st_f<T>((T*)a.seg[0].ptr + tok * a.seg[0].ld + col, v);
            } else {
                v = acc[0][i][j] + (a.bias ? a.bias[col] : 0.f);
                if (a.rowbias) v += a.rowbias[(int64_t)a.row_owner[tok / a.geom.S] * a.N + col];
                if (a.act_gelu) v = gelu_tanh_f(v);
                if (a.rowscale) v *= a.rowscale[(int64_t)a.row_owner[tok / a.geom.S] * a.rowscale_ld + col];
                if (a.res) v += ld_f<T>((const T*)a.res + tok * a.ldr + col);
                route_store<T>(a, tok, col, v);
            }
        }
    }
}

// ---- packing kernels -----------------------------------------------------------------------------------
template <typename T>
__global__ void pack_conv_kernel(const T* __restrict__ w, T* __restrict__ dst, int32_t Cout, int32_t Cin) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;       // over dst [9][Cout][Cin]
    if (i >= (int64_t)9 * Cout * Cin) return;
    const int ci = (int)(i % Cin);
    const int co = (int)((i / Cin) % Cout);
    const int tap = (int)(i / ((int64_t)Cin * Cout));
    dst[i] = w[((int64_t)co * Cin + ci) * 9 + tap];
}

// four parity classes x four taps of the nearest-up convolution (see pack_conv_up2 in kernels.h)
template <typename T>
__global__ void pack_conv_up2_kernel(const T* __restrict__ w, T* __restrict__ dst, int32_t Cout, int32_t Cin) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;       // over dst [4][4][Cout][Cin]
    if (i >= (int64_t)16 * Cout * Cin) return;
    const int ci = (int)(i % Cin);
    const int co = (int)((i / Cin) % Cout);
    const int t = (int)(i / ((int64_t)Cin * Cout));
    const int cls = t >> 2, a = cls >> 1, b = cls & 1, j = (t >> 1) & 1, ii = t & 1;
    // 3x3 rows merged into 2x2 row j: a = 0: {0}, {1, 2};  a = 1: {0, 1}, {2}
    const int y0 = a == 0 ? (j == 0 ? 0 : 1) : (j == 0 ? 0 : 2), y1 = a == 0 ? (j == 0 ? 0 : 2) : (j == 0 ? 1 : 2);
    const int x0 = b == 0 ? (ii == 0 ? 0 : 1) : (ii == 0 ? 0 : 2), x1 = b == 0 ? (ii == 0 ? 0 : 2) : (ii == 0 ? 1 : 2);
    float acc = 0.f;
    for (int ty = y0; ty <= y1; ++ty)
        for (int tx = x0; tx <= x1; ++tx) acc += ld_f<T>(w + ((int64_t)co * Cin + ci) * 9 + ty * 3 + tx);
    st_f<T>(dst + i, acc);
}

// dst row (row0 + perm(n)) = column n of w[K][Ncols]; geglu_F > 0 applies the value/gate interleave
template <typename T>
__global__ void pack_linear_kernel(const T* __restrict__ w, T* __restrict__ dst, int32_t K, int32_t Ncols, int32_t row0,
                                   int32_t geglu_F) {
    __shared__ T tile[32][33];
    const int k0 = blockIdx.x * 32, n0 = blockIdx.y * 32;
    const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;      // 256 threads: ty 0..7
    for (int r = ty; r < 32; r += 8)
        if (k0 + r < K && n0 + tx < Ncols) tile[r][tx] = w[(int64_t)(k0 + r) * Ncols + n0 + tx];
    __syncthreads();
    for (int r = ty; r < 32; r += 8) {
        const int n = n0 + r, k = k0 + tx;
        if (n < Ncols && k < K) {
            int row = n;
            if (geglu_F > 0) {
                const int half = n >= geglu_F, c = half ? n - geglu_F : n;
                row = (c / GEGLU_GROUP) * 2 * GEGLU_GROUP + half * GEGLU_GROUP + c % GEGLU_GROUP;
            }
            dst[(int64_t)(row0 + row) * K + k] = tile[tx][r];
        }
    }
}

template <typename T>
__global__ void pack_bias_kernel(const T* __restrict__ b, float* __restrict__ dst, int32_t N, int32_t geglu_F) {
    const int n = blockIdx.x * blockDim.x + threadIdx.x;
    if (n >= N) return;
    int row = n;
    if (geglu_F > 0) {
        const int half = n >= geglu_F, c = half ? n - geglu_F : n;
        row = (c / GEGLU_GROUP) * 2 * GEGLU_GROUP + half * GEGLU_GROUP + c % GEGLU_GROUP;
    }
    dst[row] = ld_f<T>(b + n);
}

int pack_conv(const void* w, void* dst, int32_t Cout, int32_t Cin, int dtype, hipStream_t st) {
    const int64_t total = (int64_t)9 * Cout * Cin;
    const unsigned grid = (unsigned)cdiv(total, 256);
    if (dtype == PSERVE_BF16) pack_conv_kernel<uint16_t><<<grid, 256, 0, st>>>((const uint16_t*)w, (uint16_t*)dst, Cout, Cin);
    else pack_conv_kernel<float><<<grid, 256, 0, st>>>((const float*)w, (float*)dst, Cout, Cin);
    return check_launch("pack_conv_kernel");
}

int pack_conv_up2(const void* w, void* dst, int32_t Cout, int32_t Cin, int dtype, hipStream_t st) {
    const unsigned grid = (unsigned)cdiv((int64_t)16 * Cout * Cin, 256);
    if (dtype == PSERVE_BF16) pack_conv_up2_kernel<uint16_t><<<grid, 256, 0, st>>>((const uint16_t*)w, (uint16_t*)dst, Cout, Cin);
    else pack_conv_up2_kernel<float><<<grid, 256, 0, st>>>((const float*)w, (float*)dst, Cout, Cin);
    return check_launch("pack_conv_up2_kernel");
}

static int pack_linear_impl(const void* w, void* dst, int32_t K, int32_t Ncols, int32_t row0, int32_t gF, int dtype,
                            hipStream_t st) {
    dim3 grid((unsigned)cdiv(K, 32), (unsigned)cdiv(Ncols, 32));
    if (dtype == PSERVE_BF16)
        pack_linear_kernel<uint16_t><<<grid, 256, 0, st>>>((const uint16_t*)w, (uint16_t*)dst, K, Ncols, row0, gF);
    else
        pack_linear_kernel<float><<<grid, 256, 0, st>>>((const float*)w, (float*)dst, K, Ncols, row0, gF);
    return check_launch("pack_linear_kernel");
}

int pack_linear(const void* w, void* dst, int32_t K, int32_t Ncols, int32_t row0, int dtype, hipStream_t st) {
    return pack_linear_impl(w, dst, K, Ncols, row0, 0, dtype, st);
}

static int pack_bias_impl(const void* b, float* dst, int32_t N, int32_t gF, int dtype, hipStream_t st) {
    const unsigned grid = (unsigned)cdiv(N, 256);
    if (dtype == PSERVE_BF16) pack_bias_kernel<uint16_t><<<grid, 256, 0, st>>>((const uint16_t*)b, dst, N, gF);
    else pack_bias_kernel<float><<<grid, 256, 0, st>>>((const float*)b, dst, N, gF);
    return check_launch("pack_bias_kernel");
}

int pack_bias(const void* b, float* dst, int32_t N, int dtype, hipStream_t st) { return pack_bias_impl(b, dst, N, 0, dtype, st); }

int pack_geglu(const void* w1, const void* b1, void* dst, float* bias_dst, int32_t K, int32_t F, int dtype, hipStream_t st) {
    PS_REQUIRE(F % GEGLU_GROUP == 0, "FFN: hidden width %d must be a multiple of %d", F, GEGLU_GROUP);
    PS_TRY(pack_linear_impl(w1, dst, K, 2 * F, 0, F, dtype, st));
    return pack_bias_impl(b1, bias_dst, 2 * F, F, dtype, st);
}

// ---- dispatch -------------------------------------------------------------------------------------------
int gemm_mfma_bf16(const GemmArgs& a, hipStream_t st, bool* handled);     // gemm_mfma.hip

int gemm(const GemmArgs& a, int dtype, int mode, hipStream_t st) {
    PS_REQUIRE(a.M > 0 && a.N > 0 && a.K > 0, "gemm: empty problem");
    if (mode == 0 && dtype == PSERVE_BF16) {
        bool handled = false;
        PS_TRY(gemm_mfma_bf16(a, st, &handled));
        if (handled) return PSERVE_OK;
    }
    const bool geglu = a.epi == EPI_GEGLU;
    const int ncols = geglu ? a.N / 2 : a.N;
    dim3 grid((unsigned)cdiv(a.M, 64), (unsigned)cdiv(ncols, 64));
    if (dtype == PSERVE_BF16) {
        if (geglu) gemm_simple_kernel<uint16_t, true><<<grid, 256, 0, st>>>(a);
        else gemm_simple_kernel<uint16_t, false><<<grid, 256, 0, st>>>(a);
    } else {
        if (geglu) gemm_simple_kernel<float, true><<<grid, 256, 0, st>>>(a);
        else gemm_simple_kernel<float, false><<<grid, 256, 0, st>>>(a);
    }
    return check_launch("gemm_simple_kernel");
}

}  // namespace pserve
