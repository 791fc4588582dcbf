// bf16 MFMA GEMM / implicit-GEMM 3x3 convolution for gfx950.
//
// Block tile BM x BN, 256 threads = 4 wavefronts in a 2 x 2 grid, each wavefront owns a
// (BM/2) x (BN/2) tile made of 32x32 MFMA tiles (v_mfma_f32_32x32x16_bf16, fp32 accumulate).
// K is walked tap by tap (nine shifted views of the padded patch buffer for the 3x3
// convolution, one view for linear layers) in steps of BK = 64.  Global -> register -> LDS
// staging with a register prefetch of the next K step and double-buffered LDS (one barrier per
// step).  LDS rows are 128 bytes; the 16-byte chunk c of row r is stored at chunk position
// c ^ (r & 7), which makes both the staging writes and the MFMA fragment reads (32 rows at one
// chunk position) bank-conflict free without padding.
#include "kernels.h"

namespace pserve {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;

__device__ __forceinline__ float gelu_erf(float v) { return 0.5f * v * (1.f + erff(v * 0.70710678118654752f)); }

template <int BM, int BN, bool GEGLU>
__global__ void __launch_bounds__(256)
gemm_mfma_kernel(GemmArgs a) {
    constexpr int BK = 64;
    constexpr int CH = BK / 8;                      // 16-byte chunks per row
    constexpr int WM = BM / 2, WN = BN / 2;         // wavefront tile
    constexpr int TM = WM / 32, TN = WN / 32;       // 32x32 MFMA tiles per wavefront
    constexpr int A_LD = BM * CH / 256;             // 16-byte loads per thread and K step
    constexpr int B_LD = BN * CH / 256;
    static_assert(BM % 64 == 0 && BN % 64 == 0 && (BM * CH) % 256 == 0 && (BN * CH) % 256 == 0, "tile shape");
    extern __shared__ __attribute__((aligned(16))) uint8_t smem[];
    uint4* sA = reinterpret_cast<uint4*>(smem);                       // [2][BM*CH]
    uint4* sB = sA + 2 * BM * CH;                                     // [2][BN*CH]
    int32_t* s_tok = reinterpret_cast<int32_t*>(sB + 2 * BN * CH);    // [BM] token of each row, -1 = no row

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int m0 = blockIdx.x * BM, n0 = blockIdx.y * BN;
    if (a.tokens_are_rows && a.act.active && m0 >= *a.act.count * a.geom.S) return;

    // rows this thread stages: chunk (tid % CH) of rows tid / CH + i * (256 / CH)
    const int lc = tid % CH, lr = tid / CH;
    const uint16_t* A = (const uint16_t*)a.A;
    const uint16_t* B = (const uint16_t*)a.B;
    const uint16_t* a_ptr[A_LD];
#pragma unroll
    for (int i = 0; i < A_LD; ++i) {
        const int row = lr + i * (256 / CH);
        int64_t tok = m0 + row;
        bool valid;
        if (a.tokens_are_rows && a.act.active) {
            const int pi = (int)(tok / a.geom.S);
            valid = pi < *a.act.count;
            tok = valid ? (int64_t)a.act.active[pi] * a.geom.S + (tok - (int64_t)pi * a.geom.S) : 0;
        } else {
            valid = tok < a.M;
            if (!valid) tok = 0;
        }
        int64_t off;
        if (a.conv) {
            const int p = (int)(tok / a.geom.S), q = (int)(tok - (int64_t)p * a.geom.S);
            const int y = q / a.geom.pw, x = q - y * a.geom.pw;
            off = ((int64_t)p * a.geom.pS + y * a.geom.ppw + x) * a.lda;
        } else {
            off = tok * a.lda;
        }
        a_ptr[i] = A + off + lc * 8;
        if (lc == 0) s_tok[row] = valid ? (int32_t)tok : -1;
    }
    const uint16_t* b_ptr[B_LD];
#pragma unroll
    for (int i = 0; i < B_LD; ++i) b_ptr[i] = B + (int64_t)(n0 + lr + i * (256 / CH)) * a.K + lc * 8;

    const int kchunks = a.K / BK;
    const int KT = a.taps * kchunks;

    uint4 ra[A_LD], rb[B_LD];
    auto load_global = [&](int kt) {
        const int tap = kt / kchunks, kc = kt - tap * kchunks;
        const int64_t a_off = (a.conv ? ((int64_t)(tap / 3) * a.geom.ppw + (tap % 3)) * a.lda : 0) + kc * BK;
        const int64_t b_off = (int64_t)tap * a.N * a.K + kc * BK;
#pragma unroll
        for (int i = 0; i < A_LD; ++i) ra[i] = *reinterpret_cast<const uint4*>(a_ptr[i] + a_off);
#pragma unroll
        for (int i = 0; i < B_LD; ++i) rb[i] = *reinterpret_cast<const uint4*>(b_ptr[i] + b_off);
    };
    auto store_lds = [&](int buf) {
#pragma unroll
        for (int i = 0; i < A_LD; ++i) {
            const int row = lr + i * (256 / CH);
            sA[buf * BM * CH + row * CH + (lc ^ (row & 7))] = ra[i];
        }
#pragma unroll
        for (int i = 0; i < B_LD; ++i) {
            const int row = lr + i * (256 / CH);
            sB[buf * BN * CH + row * CH + (lc ^ (row & 7))] = rb[i];
        }
    };

    f32x16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

    load_global(0);
    store_lds(0);
    __syncthreads();

    const int fr = lane & 31, fh = lane >> 5;       // fragment row within a 32-row tile, k half
    for (int kt = 0; kt < KT; ++kt) {
        const int buf = kt & 1;
        if (kt + 1 < KT) load_global(kt + 1);
        const uint4* cA = sA + buf * BM * CH;
        const uint4* cB = sB + buf * BN * CH;
#pragma unroll
        for (int ks = 0; ks < BK / 16; ++ks) {
            const int c = ks * 2 + fh;              // 16-byte chunk holding k = ks*16 + fh*8 .. +8
            bf16x8 fa[TM], fb[TN];
#pragma unroll
            for (int i = 0; i < TM; ++i) {
                const int row = wm * WM + i * 32 + fr;
                const uint4 v = cA[row * CH + (c ^ (row & 7))];
                fa[i] = *reinterpret_cast<const bf16x8*>(&v);
            }
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                const int row = wn * WN + j * 32 + fr;
                const uint4 v = cB[row * CH + (c ^ (row & 7))];
                fb[j] = *reinterpret_cast<const bf16x8*>(&v);
            }
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[i], fb[j], acc[i][j], 0, 0, 0);
        }
        if (kt + 1 < KT) store_lds(buf ^ 1);
        __syncthreads();
    }

    // ---- epilogue: lane holds column (lane % 32) of each 32x32 tile, rows 8*(e/4) + 4*(lane/32) + e%4
    if (GEGLU) {
        static_assert(!GEGLU || (WN == 2 * GEGLU_GROUP), "GEGLU needs a wavefront tile of [GROUP values | GROUP gates]");
        uint16_t* out = (uint16_t*)a.seg[0].ptr;
        const int64_t ld = a.seg[0].ld;
#pragma unroll
        for (int j = 0; j < TN / 2; ++j) {
            const int pc = n0 + wn * WN + j * 32 + fr;                // packed value column; gate at + GROUP
            const int oc = (n0 + wn * WN) / 2 + j * 32 + fr;          // output column
            const float bv = a.bias ? a.bias[pc] : 0.f, bg = a.bias ? a.bias[pc + GEGLU_GROUP] : 0.f;
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    const int row = wm * WM + i * 32 + 8 * (e >> 2) + 4 * fh + (e & 3);
                    const int tok = s_tok[row];
                    if (tok < 0) continue;
                    const float v = (acc[i][j][e] + bv) * gelu_erf(acc[i][j + TN / 2][e] + bg);
                    out[(int64_t)tok * ld + oc] = float_to_bf16_bits(v);
                }
        }
    } else {
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            const int col = n0 + wn * WN + j * 32 + fr;
            const int sg = col / a.seg_cols, c = col - sg * a.seg_cols;
            const GemmSeg sgm = a.seg[sg];
            uint16_t* out = (uint16_t*)sgm.ptr;
            const float bias = a.bias ? a.bias[col] : 0.f;
            const uint16_t* res = (const uint16_t*)a.res;
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    const int row = wm * WM + i * 32 + 8 * (e >> 2) + 4 * fh + (e & 3);
                    const int tok = s_tok[row];
                    if (tok < 0) continue;
                    float v = acc[i][j][e] + bias;
                    if (res) v += bf16_bits_to_float(res[(int64_t)tok * a.ldr + col]);
                    v *= sgm.scale;
                    if (sgm.transposed) out[(int64_t)c * sgm.ld + tok] = float_to_bf16_bits(v);
                    else out[(int64_t)tok * sgm.ld + c] = float_to_bf16_bits(v);
                }
        }
    }
}

template <int BM, int BN, bool GEGLU>
static int launch(const GemmArgs& a, hipStream_t st) {
    constexpr size_t lds = (size_t)2 * (BM + BN) * 8 * 16 + BM * sizeof(int32_t);
    static bool attr_set = false;
    if (!attr_set) {
        PS_CHECK_HIP(hipFuncSetAttribute((const void*)gemm_mfma_kernel<BM, BN, GEGLU>,
                                         hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
        attr_set = true;
    }
    dim3 grid((unsigned)cdiv(a.M, BM), (unsigned)(a.N / BN));
    gemm_mfma_kernel<BM, BN, GEGLU><<<grid, 256, lds, st>>>(a);
    return check_launch("gemm_mfma_kernel");
}

int gemm_mfma_bf16(const GemmArgs& a, hipStream_t st, bool* handled) {
    *handled = false;
    if (a.K % 64 != 0 || a.lda % 8 != 0 || ((uintptr_t)a.A & 15) || ((uintptr_t)a.B & 15)) return PSERVE_OK;
    if (a.epi == EPI_GEGLU) {
        if (a.N % 256 != 0) return PSERVE_OK;
        *handled = true;
        return launch<128, 256, true>(a, st);
    }
    if (a.seg_cols % 32 != 0) return PSERVE_OK;      // a 32-column tile must not straddle output segments
    if (a.N % 320 == 0) { *handled = true; return launch<128, 320, false>(a, st); }
    if (a.N % 256 == 0) { *handled = true; return launch<128, 256, false>(a, st); }
    if (a.N % 128 == 0) { *handled = true; return launch<128, 128, false>(a, st); }
    if (a.N % 64 == 0) { *handled = true; return launch<128, 64, false>(a, st); }
    return PSERVE_OK;
}

}  // namespace pserve
