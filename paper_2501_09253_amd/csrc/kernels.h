// Internal launch interface between the block executor and the kernel files.
#pragma once

#include "common.h"

namespace pserve {

// ---- element access helpers (device) ------------------------------------------------------
__device__ __forceinline__ float bf16_bits_to_float(uint16_t b) { return __uint_as_float((uint32_t)b << 16); }
__device__ __forceinline__ uint16_t float_to_bf16_bits(float f) {       // round to nearest even (v_cvt_pk_bf16_f32)
    return __builtin_bit_cast(uint16_t, (__bf16)f);
}
// two floats -> packed bf16 pair (lo in bits 0..15), one v_cvt_pk_bf16_f32
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
    typedef __attribute__((ext_vector_type(2))) float f32x2_t;
    typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_t;
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(f32x2_t{lo, hi}, bf16x2_t));
}
template <typename T> __device__ __forceinline__ float ld_f(const T* p);
template <> __device__ __forceinline__ float ld_f<float>(const float* p) { return *p; }
template <> __device__ __forceinline__ float ld_f<uint16_t>(const uint16_t* p) { return bf16_bits_to_float(*p); }
template <typename T> __device__ __forceinline__ void st_f(T* p, float v);
template <> __device__ __forceinline__ void st_f<float>(float* p, float v) { *p = v; }
template <> __device__ __forceinline__ void st_f<uint16_t>(uint16_t* p, float v) { *p = float_to_bf16_bits(v); }

// Patch geometry shared by the kernels that walk tokens.
struct PatchGeom {
    int32_t P, S, ph, pw;      // patches, tokens per patch, patch height / width
    int32_t ppw, pS;           // padded patch width (pw+2) and padded pixels per patch ((ph+2)*(pw+2))
};

// Optional compaction of the patches that are computed (reuse mask == 0).  active == nullptr means
// "all patches, identity order".
struct ActiveList {
    const int32_t* active;     // [P] patch ids, first *count entries valid
    const int32_t* count;      // device scalar
};

// ---- GroupNorm (norm.hip) -------------------------------------------------------------------
struct GroupNormArgs {
    const void* x;             // [T][C]
    const void* gamma;         // [C] block dtype
    const void* beta;          // [C]
    int32_t C, G, n;
    float eps;
    int32_t nsplit;            // token chunks per patch used for the partial sums
    float* partial;            // [P][nsplit][G][2] (sum, sum of squares)
    float* scale_shift;        // [n][C][2]: y = x*scale + shift for sorted slot s
    const int32_t* request_offset;   // [n+1]
    const int32_t* owner;      // [P]
    const int32_t* neighbour;  // [P][8] (stitching only)
    const uint8_t* rim_only = nullptr;   // [P] or nullptr; apply pass into the padded layout: only the border tokens of these patches
};
int gn_stats(const GroupNormArgs& a, const PatchGeom& g, int dtype, hipStream_t st);
// second half of gn_stats alone: a.partial already holds [P][slots][G][2] partial sums (filled by a convolution)
int gn_finalize(const GroupNormArgs& a, const PatchGeom& g, int dtype, int32_t slots, hipStream_t st, bool per_channel = false);
// bf16 split that also leaves per-channel moments stats[P][nch][C][2] behind (plan.hip); *done = false where its
// fast path does not apply (nothing is written then)
int split_with_stats(const pserve_plan_t* plan, const void* const* images, int32_t C, void* x, float* stats, int32_t nch,
                     hipStream_t st, bool* done);
// y = x*scale+shift (then SiLU if silu).  padded: write into the interior of the padded patch buffer
// [P][ph+2][pw+2][C]; else plain [T][C].  Only patches of `act` are written.  stitch (padded, all patches):
// border tokens also fill the neighbours' ring slots / zero the own ring at image edges (no halo_gather needed).
int gn_apply(const GroupNormArgs& a, const PatchGeom& g, int dtype, bool silu, bool padded, bool stitch, void* out,
             ActiveList act, hipStream_t st);
// Per-token LayerNorm over the C channels (biased variance) of the patches of `act`; out [T][C] at the same token
// positions.  Affine part: gamma / beta [C] of the block dtype, or (gamma == nullptr) the adaptive form
// xhat * (1 + scale) + shift with shift = mod[slot * mod_ld + c], scale = mod[slot * mod_ld + C + c], slot = owner[patch].
int layer_norm(const void* x, const void* gamma, const void* beta, const float* mod, int64_t mod_ld, const int32_t* owner,
               int32_t C, float eps, const PatchGeom& g, int dtype, void* out, ActiveList act, hipStream_t st);
// Fill the one-pixel ring of every active padded patch from the interiors of its neighbours (zeros outside the image).
int halo_gather(void* apad, const int32_t* halo_src, const PatchGeom& g, int32_t C, int32_t ring, int dtype,
                ActiveList act, hipStream_t st);

// ---- GEMM / implicit-GEMM convolution (gemm.hip) -----------------------------------------------
struct GemmSeg {
    void* ptr;                 // output of this column segment
    int64_t ld;                // row stride (elements); for transposed: stride between channels
    int32_t transposed;        // 1: out[col][row] instead of out[row][col]
    float scale;               // multiplies the result (after bias)
};
enum { EPI_ROUTE = 0, EPI_GEGLU = 1 };
struct GemmArgs {
    const void* A;             // linear: [rows][lda]; conv: padded patch buffer
    int64_t lda;
    int32_t conv;              // 1: rows are tokens read through the padded layout with `taps` taps
    // conv only (0 = the defaults 3 / 1 / identity): taps are laid out tap_w per pixel row; row token (p, y, x) reads
    // the padded pixels (a_mul*y + a_dy + ty, a_mul*x + a_dx + tx) of patch p (a_mul = 2: stride-2 convolution whose
    // rows are OUTPUT tokens of the half-size patch geometry in `geom.S / geom.pw`, while geom.ppw / geom.pS stay those
    // of the input); with o_mul = 2 the result of row (p, y, x) goes to token p*o_S + (2y + o_dy)*o_pw + 2x + o_dx
    // (one parity class of a nearest-up convolution, whose rows are INPUT tokens)
    int32_t tap_w, a_mul, a_dy, a_dx;
    int32_t o_mul, o_dy, o_dx, o_S, o_pw;
    PatchGeom geom;
    ActiveList act;            // row compaction by patch (rows are tokens)
    int32_t tokens_are_rows;   // 1: row ids are token ids (act applies); 0: plain row ids (M rows)
    int32_t M;                 // number of rows (upper bound when act is used: P*S)
    int32_t row_group, row_group_pad;   // plain rows only: output row = (r / row_group) * row_group_pad + r % row_group (0 = identity)
    int32_t N, K;              // N packed output columns, K reduction length per tap
    int32_t taps;              // 1 or 9
    const void* B;             // packed weights [taps][N][K]
    const float* bias;         // [N] packed order, or nullptr
    const float* rowbias;      // optional [n][N]: row r also gets rowbias[row_owner[token / S]][col] (rows are tokens)
    const int32_t* row_owner;  // [P] request slot of each patch (with rowbias / rowscale)
    const float* rowscale;     // optional: (acc + bias [+ rowbias]) is multiplied by rowscale[slot * rowscale_ld + col]
    int64_t rowscale_ld;       //           before the residual is added (gated residual of an adaLN sub-layer)
    int32_t act_gelu;          // 1: tanh-form GELU of (acc + bias) (EPI_ROUTE only)
    const void* res;           // residual [rows][ldr] or nullptr (added after bias)
    int64_t ldr;
    int32_t epi;               // EPI_ROUTE: columns go to segment col / seg_cols; EPI_GEGLU: value*GELU(gate) pairs
    int32_t seg_cols;
    GemmSeg seg[3];
    // Optional GroupNorm partial sums of the OUTPUT (bias included, before the residual), in the layout gn_finalize
    // reads: stats[P][stats_slots][stats_G][2] = (sum, sum of squares) of 64 consecutive tokens of a patch
    // (stats_slots = S / 64) and one group.  Only the kernels gemm_emits_stats() accepts fill it (plain stores).
    float* stats;
    int32_t stats_G, stats_slots;
};
// true if gemm(a, ...) will take a kernel that fills a.stats (the caller otherwise runs gn_stats on the output)
bool gemm_emits_stats(const GemmArgs& a, int dtype, int mode);
int gemm(const GemmArgs& a, int dtype, int mode, hipStream_t st);

// weight packing into [taps][N][K] (K contiguous); all on device
int pack_conv(const void* w, void* dst, int32_t Cout, int32_t Cin, int dtype, hipStream_t st);
// linear W[K][Ncols] -> rows [row0, row0+Ncols) of dst[Ntotal][K]
int pack_linear(const void* w, void* dst, int32_t K, int32_t Ncols, int32_t row0, int dtype, hipStream_t st);
// GEGLU: W1[K][2F] -> dst[2F][K] with value / gate columns interleaved in groups of GEGLU_GROUP
int pack_geglu(const void* w1, const void* b1, void* dst, float* bias_dst, int32_t K, int32_t F, int dtype, hipStream_t st);
int pack_bias(const void* b, float* dst, int32_t N, int dtype, hipStream_t st);
// Nearest-up 2x followed by a 3x3 convolution = four 2x2-tap convolutions on the input, one per output parity (a, b):
// dst[(2a+b)][2j+i][Cout][Cin] = sum of the 3x3 taps (ty, tx) that fall on input pixel (y - 1 + a + j, x - 1 + b + i),
// i.e. rows {0 | 1,2} for a = 0 and {0,1 | 2} for a = 1 (same for columns); summed in fp32, rounded once.
int pack_conv_up2(const void* w, void* dst, int32_t Cout, int32_t Cin, int dtype, hipStream_t st);
constexpr int GEGLU_GROUP = 64;

// ---- attention (attn.hip) -------------------------------------------------------------------------
struct AttnArgs {
    const void* Q;             // [T][C], already multiplied by log2(e)/sqrt(d)
    const void* K;             // self: [T][C]; cross: [n*L][C]
    const void* V;             // [rows][C], or transposed [C][ldv] when v_transposed
    int64_t ldv;
    int32_t v_transposed;
    void* O;                   // [T][C]
    int32_t C, heads, d;
    PatchGeom geom;
    ActiveList act;
    const int32_t* owner;      // [P] sorted slot of a patch
    const int32_t* cu_seqlens; // self: [n+1] token range of slot s
    const int32_t* seq_len;    // self: [n] valid tokens of slot s (keys cu_seqlens[s] .. + seq_len[s]); nullptr: the whole range
    const int32_t* perm;       // cross: caller index of slot s
    int32_t cross_len;         // 0 = self-attention; else keys of slot s are rows perm[s]*cross_len .. +cross_len
    int32_t cross_ld;          // cross: padded key rows per request (>= cross_len)
    // query tiling of the MFMA kernel (attention_tiles fills the two prefix tables)
    const int32_t* act_off;    // [n+1] computed patches before slot s (== RequestOffset without a mask)
    const int32_t* tile_off;   // [n+1] query tiles before slot s
    int32_t n;                 // request slots
    int32_t max_tiles;         // host upper bound of tile_off[n]
    int32_t qt;                // 1 or 2: the tables were built for query tiles of 128 * qt rows
    int32_t max_rows;          // host upper bound of the query rows of one request (its tokens)
};
int attention_tiles(const int32_t* request_offset, const uint8_t* mask, int32_t n, int32_t S, int32_t qt, int32_t* act_off,
                    int32_t* tile_off, hipStream_t st);
int attention_max_tiles(const pserve_plan_t* plan, int32_t qt);
int attention(const AttnArgs& a, int dtype, int mode, hipStream_t st);

// ---- reuse (block.hip) -------------------------------------------------------------------------------

}  // namespace pserve
