// bf16 MFMA GEMM / implicit-GEMM 3x3 convolution for gfx950.
//
// Two kernels share one epilogue:
//   gemm_mfma_kernel  block tile 256 x 160 / 256 x 128 / 128 x 160 (four wavefronts stacked along M) or 128 x BN
//                     (2 x 2), K in steps of 64, A and B tiles staged by direct global -> LDS loads into a ring of
//                     2-4 stages (one barrier per step); linear layers (one tap) and the fallback form of the
//                     convolution (nine taps re-load A).  The 128-row tiles with two stages run two blocks per CU.
//   conv_mfma_kernel  3x3 convolution with the haloed activation tile kept in LDS across the nine taps;
//                     preferred tile 256 x 160 with four wavefronts stacked along M, each doubled by a second
//                     wavefront that takes the other half of every K step (two wavefronts per SIMD).
// In both, every LDS fragment read and every global load is issued behind an MFMA (a wavefront issues in order,
// and with one block per CU and four wavefronts there is no other wavefront on the SIMD to fill a bubble).
// MFMA shape v_mfma_f32_32x32x16_bf16, fp32 accumulation.  LDS rows are 128 bytes (8 chunks of 16 bytes); chunk c of
// row r sits at position c ^ ((r >> 1) & 7), which keeps the fragment reads (32 rows at one chunk position)
// bank-conflict free; the swizzle is applied by choosing which global chunk each lane of a load fetches.
#include "kernels.h"
#include <type_traits>

namespace pserve {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(4))) float f32x4;

// GELU(v) = v/2 (1 + erf(v/sqrt 2)) with erf from the 5-term rational-exponential form (Abramowitz & Stegun
// 7.1.26, |error| < 1.5e-7): far below the bf16 resolution of the output and several times cheaper than erff.
// With u = |v|, t = 1/(1 + p u/sqrt 2) and y = (a1 t + .. + a5 t^5)/2 * exp(-u^2/2):  erf(u/sqrt 2) = 1 - 2y, so
// GELU(v) = v (1 - y) for v >= 0 and v y for v < 0.  Hardware reciprocal and exp2 (1 ulp each); 15 instructions.
__device__ __forceinline__ float gelu_erf(float v) {
    const float u = fabsf(v);
    const float t = __builtin_amdgcn_rcpf(fmaf(0.3275911f * 0.70710678118654752f, u, 1.f));
    float p = fmaf(0.5f * 1.061405429f, t, 0.5f * -1.453152027f);
    p = fmaf(p, t, 0.5f * 1.421413741f);
    p = fmaf(p, t, 0.5f * -0.284496736f);
    p = fmaf(p, t, 0.5f * 0.254829592f);
    const float y = p * t * __builtin_amdgcn_exp2f(u * u * (-0.5f * 1.4426950408889634f));
    const float r = v * y;
    return v >= 0.f ? v - r : r;
}

// GELU, tanh form: v/2 (1 + tanh(u)) = v / (1 + exp(-2u)), u = sqrt(2/pi) (v + 0.044715 v^3); hardware exp2 and reciprocal
__device__ __forceinline__ float gelu_tanh(float v) {
    const float u2 = v * fmaf(0.044715f * v, v, 1.f) * (-2.f * 0.7978845608028654f * 1.4426950408889634f);   // -2u log2(e)
    return v * __builtin_amdgcn_rcpf(1.f + __builtin_amdgcn_exp2f(u2));
}

// value of lane l ^ 32 (v_permlane32_swap: upper half of the first operand <-> lower half of the second)
__device__ __forceinline__ float other_half_f(float v) {
    const uint32_t u = __float_as_uint(v);
    const auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
    return __uint_as_float((threadIdx.x & 32) ? r[0] : r[1]);
}

// ---- epilogue shared by the kernels.  A lane holds column (lane % 32) of each 32x32 tile and rows
// 8*(e/4) + 4*(lane/32) + e%4.  One tile column (WM rows x 32 columns) at a time is finished in registers (bias,
// scale, GEGLU), staged as fp32 in this wavefront's private LDS region and read back row-wise, so that residual
// loads and output stores are 16 bytes per lane and 64 contiguous bytes per row.  Residual loads of the next tile
// column are issued before the current one is staged.  `smem` must be free (all staged operands consumed).
// bias_pre: the lane's bias of each of its TN tile columns, loaded by the caller (a kernel that has other loads in
// flight reads it before issuing those: a wait for a later load waits for all earlier ones).
// FEAT: which of the rarely taken paths are compiled in.  The epilogue is straight-line code that a block runs once per
// tile, fully unrolled over the tile columns: every path that is present but skipped costs a jump to an instruction
// line that is not in the cache (per-column timestamps showed 2 us per column, about five such jumps each, whatever
// the memory traffic), so a kernel that can rule a path out by its launch conditions leaves it out.
enum : int {
    EPF_TRANS = 1,      // transposed output segments
    EPF_GELU = 2,       // tanh GELU on the result
    EPF_GATE = 4,       // per-request gate (rowscale)
    EPF_MIXED = 8,      // rows of several requests in one wavefront tile: per-element look-ups of rowbias / rowscale
    EPF_SCALE = 16,     // output segments with a scale other than 1 (the pre-multiplied Q)
    EPF_ALL = 31
};
template <int BM, int BN, bool GEGLU, int WGM = 2, int WGN = 2, bool MAY_STAT = true, int FEAT = EPF_ALL>
__device__ __forceinline__ void gemm_epilogue(const GemmArgs& a, f32x16 (&acc)[BM / WGM / 32][BN / WGN / 32], uint8_t* smem,
                                              const int32_t* s_tok, int n0, const float* bias_pre = nullptr) {
    constexpr int WM = BM / WGM, WN = BN / WGN, TM = WM / 32, TN = WN / 32;     // WGM x WGN wavefront grid
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int wm = wave / WGN, wn = wave % WGN;
    const int fr = lane & 31, fh = lane >> 5;
    constexpr int EP_LD = 36;                                       // floats per staged row (16-byte aligned, skewed banks)
    float* ep = reinterpret_cast<float*>(smem) + wave * (WM * EP_LD);
    const int32_t* w_tok = s_tok + wm * WM;
    constexpr int TNO = GEGLU ? TN / 2 : TN;                        // output tile columns per wavefront
    static_assert(!GEGLU || (WN == 2 * GEGLU_GROUP), "GEGLU needs a wavefront tile of [GROUP values | GROUP gates]");
    // residual rows of this lane's read-back items (row = item / 4, 8-column chunk = item % 4)
    constexpr int NIT = WM * 4 / 64;
    const bool HAS_RES = !GEGLU && a.res != nullptr;
    const uint16_t* res_row[NIT];
    // residual of the lane's items: with a small wavefront tile all tile columns are fetched at once (every column
    // otherwise waits out a memory round trip of its own, with one column of work to cover it), else one column ahead
    constexpr bool RES_ALL = TNO * NIT <= 12;
    constexpr int RSETS = RES_ALL ? TNO : 2;
    u32x4 rres[RSETS][NIT];
#pragma unroll
    for (int t = 0; t < NIT; ++t) {
        const int item = t * 64 + lane;
        const int tok = w_tok[item >> 2];
        res_row[t] = (const uint16_t*)a.res + (int64_t)(tok < 0 ? 0 : tok) * a.ldr + (item & 3) * 8;
    }
    if (HAS_RES) {
#pragma unroll
        for (int jj = 0; jj < (RES_ALL ? TNO : 1); ++jj)
#pragma unroll
            for (int t = 0; t < NIT; ++t) rres[jj][t] = *reinterpret_cast<const u32x4*>(res_row[t] + n0 + wn * WN + jj * 32);
    }
    // per-request bias (time embedding): one value per column when all rows of the wavefront's tile belong to one
    // request (rows are ordered by request, so first == last decides), else looked up per element
    bool rb_uniform = false;
    int rb_slot = 0;
    if (!GEGLU && (a.rowbias || ((FEAT & EPF_GATE) && a.rowscale))) {
        const int t_first = w_tok[0], t_last = w_tok[WM - 1];
        if (t_first >= 0 && t_last >= 0) {
            rb_slot = a.row_owner[t_first / a.geom.S];
            rb_uniform = rb_slot == a.row_owner[t_last / a.geom.S];
        }
    }
    // GroupNorm partial sums of the output (optional): column sums over this wavefront's 64 rows, which lie in one patch
    const bool STATS = MAY_STAT && !GEGLU && a.stats != nullptr;     // only the convolution kernels leave the sums behind
    float* colsum = reinterpret_cast<float*>(smem) + WGM * WGN * (WM * EP_LD) + wave * (2 * WN + 2);    // [WN][2] + row count
    uint32_t row_ok[TM];                                            // bit e: row 8*(e/4) + 4*fh + e%4 of tile i exists
    const bool all_rows = STATS && w_tok[WM - 1] >= 0;              // existing rows are a prefix of the tile
    if (STATS && !all_rows) {
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            row_ok[i] = 0;
#pragma unroll
            for (int e = 0; e < 16; ++e) row_ok[i] |= (w_tok[i * 32 + 8 * (e >> 2) + 4 * fh + (e & 3)] >= 0 ? 1u : 0u) << e;
        }
    }
#pragma unroll
    for (int j = 0; j < TNO; ++j) {
        const int pcol = n0 + wn * WN + j * 32;                     // first packed column of the tile
        int ocol0;                                                  // first output column within its segment
        GemmSeg sgm;
        float vals[TM][16];
        if (GEGLU) {
            const float bv = bias_pre ? bias_pre[j] : (a.bias ? a.bias[pcol + fr] : 0.f);
            const float bg = bias_pre ? bias_pre[j + TN / 2] : (a.bias ? a.bias[pcol + fr + GEGLU_GROUP] : 0.f);
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int e = 0; e < 16; ++e) vals[i][e] = (acc[i][j][e] + bv) * gelu_erf(acc[i][j + TN / 2][e] + bg);
            sgm = a.seg[0];
            ocol0 = (n0 + wn * WN) / 2 + j * 32;
        } else {
            const int sg = pcol / a.seg_cols;
            sgm = sg == 0 ? a.seg[0] : (sg == 1 ? a.seg[1] : a.seg[2]);
            ocol0 = pcol - sg * a.seg_cols;
            float bias = bias_pre ? bias_pre[j] : (a.bias ? a.bias[pcol + fr] : 0.f);
            if (rb_uniform && a.rowbias) bias += a.rowbias[(int64_t)rb_slot * a.N + pcol + fr];
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int e = 0; e < 16; ++e) vals[i][e] = acc[i][j][e] + bias;
            if ((FEAT & EPF_MIXED) && a.rowbias && !rb_uniform) {   // rows of several requests in this wavefront's tile
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int e = 0; e < 16; ++e) {
                        const int tok = w_tok[i * 32 + 8 * (e >> 2) + 4 * fh + (e & 3)];
                        if (tok >= 0) vals[i][e] += a.rowbias[(int64_t)a.row_owner[tok / a.geom.S] * a.N + pcol + fr];
                    }
            }
            if ((FEAT & EPF_GELU) && a.act_gelu) {
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int e = 0; e < 16; ++e) vals[i][e] = gelu_tanh(vals[i][e]);
            }
            if ((FEAT & EPF_GATE) && a.rowscale) {              // gate of the request, before the residual is added
                if (rb_uniform || !(FEAT & EPF_MIXED)) {
                    const float gate = a.rowscale[(int64_t)rb_slot * a.rowscale_ld + pcol + fr];
#pragma unroll
                    for (int i = 0; i < TM; ++i)
#pragma unroll
                        for (int e = 0; e < 16; ++e) vals[i][e] *= gate;
                } else {
#pragma unroll
                    for (int i = 0; i < TM; ++i)
#pragma unroll
                        for (int e = 0; e < 16; ++e) {
                            const int tok = w_tok[i * 32 + 8 * (e >> 2) + 4 * fh + (e & 3)];
                            if (tok >= 0) vals[i][e] *= a.rowscale[(int64_t)a.row_owner[tok / a.geom.S] * a.rowscale_ld + pcol + fr];
                        }
                }
            }
            if (STATS) {
                // column moments over the wavefront's 64 rows, around the value of the column's first row (shifted sums:
                // nothing is lost when the mean is far from zero); stored as (mean, M2) of the column
                const float own0 = vals[0][0], oth0 = other_half_f(own0);
                const float kc = fh == 0 ? own0 : oth0;             // both lane halves of a column use the lower half's value
                float s1 = 0.f, s2 = 0.f, nr = 0.f;
                if (all_rows) {
#pragma unroll
                    for (int i = 0; i < TM; ++i)
#pragma unroll
                        for (int e = 0; e < 16; ++e) { const float d = vals[i][e] - kc; s1 += d; s2 = fmaf(d, d, s2); }
                    nr = (float)(TM * 16);
                } else {
#pragma unroll
                    for (int i = 0; i < TM; ++i)
#pragma unroll
                        for (int e = 0; e < 16; ++e) {
                            const bool ok = (row_ok[i] >> e) & 1u;
                            const float d = ok ? vals[i][e] - kc : 0.f;
                            s1 += d;
                            s2 = fmaf(d, d, s2);
                            nr += ok ? 1.f : 0.f;
                        }
                }
                s1 += other_half_f(s1);
                s2 += other_half_f(s2);
                nr += other_half_f(nr);
                if (fh == 0) {
                    const float inv = nr > 0.f ? 1.f / nr : 0.f;
                    colsum[2 * (j * 32 + fr)] = kc + s1 * inv;
                    colsum[2 * (j * 32 + fr) + 1] = fmaxf(s2 - s1 * s1 * inv, 0.f);
                    if (j == 0 && fr == 0) colsum[2 * WN] = nr;     // rows of this wavefront's tile that exist
                }
            }
        }
        uint16_t* out = (uint16_t*)sgm.ptr;
        if ((FEAT & EPF_TRANS) && sgm.transposed) {
            // out[col][token]: the four rows e%4 of a lane are consecutive tokens -> one 8-byte store
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int eg = 0; eg < 4; ++eg) {
                    const int row = i * 32 + 8 * eg + 4 * fh;
                    const int t0 = w_tok[row], t3 = w_tok[row + 3];
                    uint16_t* dst = out + (int64_t)(ocol0 + fr) * sgm.ld;
                    if (t0 >= 0 && t3 == t0 + 3 && (t0 & 3) == 0 && (sgm.ld & 3) == 0) {
                        const uint32_t lo = pack_bf16x2(vals[i][4 * eg] * sgm.scale, vals[i][4 * eg + 1] * sgm.scale);
                        const uint32_t hi = pack_bf16x2(vals[i][4 * eg + 2] * sgm.scale, vals[i][4 * eg + 3] * sgm.scale);
                        *reinterpret_cast<uint2*>(dst + t0) = make_uint2(lo, hi);
                    } else {
#pragma unroll
                        for (int q = 0; q < 4; ++q) {
                            const int t = w_tok[row + q];
                            if (t >= 0) dst[t] = float_to_bf16_bits(vals[i][4 * eg + q] * sgm.scale);
                        }
                    }
                }
            continue;
        }
        // stage the tile column: ep[row][col]
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int e = 0; e < 16; ++e) ep[(i * 32 + 8 * (e >> 2) + 4 * fh + (e & 3)) * EP_LD + fr] = vals[i][e];
        __builtin_amdgcn_wave_barrier();
        // prefetch the residual of the next tile column while this one is finished
        if (HAS_RES && !RES_ALL && j + 1 < TNO) {
#pragma unroll
            for (int t = 0; t < NIT; ++t) rres[(j + 1) & 1][t] = *reinterpret_cast<const u32x4*>(res_row[t] + pcol + 32);
        }
#pragma unroll
        for (int t = 0; t < NIT; ++t) {
            const int item = t * 64 + lane;
            const int row = item >> 2, ch = item & 3;
            const int tok = w_tok[row];
            const f32x4 lo = *reinterpret_cast<const f32x4*>(ep + row * EP_LD + ch * 8);
            const f32x4 hi = *reinterpret_cast<const f32x4*>(ep + row * EP_LD + ch * 8 + 4);
            const int64_t tk = tok < 0 ? 0 : tok;                   // rows past the end read row 0 and store nothing
            float v[8] = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
            if (HAS_RES) {
                const u32x4 r = rres[RES_ALL ? j : (j & 1)][t];
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    v[2 * q] += __uint_as_float(r[q] << 16);
                    v[2 * q + 1] += __uint_as_float(r[q] & 0xFFFF0000u);
                }
            }
            u32x4 o;
#pragma unroll
            for (int q = 0; q < 4; ++q)
                o[q] = (FEAT & EPF_SCALE) ? pack_bf16x2(v[2 * q] * sgm.scale, v[2 * q + 1] * sgm.scale) : pack_bf16x2(v[2 * q], v[2 * q + 1]);
            if (tok >= 0) *reinterpret_cast<u32x4*>(out + tk * sgm.ld + ocol0 + ch * 8) = o;
        }
        __builtin_amdgcn_wave_barrier();
    }
    if (STATS) {
        __builtin_amdgcn_wave_barrier();
        const int cg = a.N / a.stats_G;                             // channels per group (divides WN, see gemm_emits_stats)
        const int tok0 = w_tok[0];
        if (lane < WN / cg && tok0 >= 0) {
            // the group's columns cover the same rows: mean of the column means, M2 by the merge formula
            const float nr = colsum[2 * WN];
            float m = 0.f;
            for (int c = lane * cg; c < (lane + 1) * cg; ++c) m += colsum[2 * c];
            m /= (float)cg;
            float m2 = 0.f;
            for (int c = lane * cg; c < (lane + 1) * cg; ++c) { const float d = colsum[2 * c] - m; m2 += colsum[2 * c + 1] + nr * d * d; }
            const int p = tok0 / a.geom.S, slot = (tok0 - p * a.geom.S) / WM;
            float* dst = a.stats + (((int64_t)p * a.stats_slots + slot) * a.stats_G + (n0 + wn * WN) / cg + lane) * 2;
            dst[0] = m;
            dst[1] = m2;
        }
    }
}

typedef __attribute__((address_space(3))) void lds_void;

// LDS bytes of one kernel instance: NS stages of (BM + BN) rows x 128 bytes, two row -> token tables and, with
// OVERLAP, a staging region of the epilogue of its own (otherwise the epilogue stages in the drained ring)
template <int BM, int BN, int NS, bool OVERLAP> struct GemmCfg {
    static constexpr int STAGE = (BM + BN) * 128;
    static constexpr int EPI = 4 * (BM / 4 >= 64 ? BM / 4 : 64) * 36 * 4;      // >= 4 wavefronts x WM rows x 36 floats
    static constexpr size_t LDS = (size_t)NS * STAGE + 2 * BM * sizeof(int32_t) + (OVERLAP ? EPI : 0);
    static_assert(LDS <= 160 * 1024, "ring does not fit the LDS");
    static_assert(OVERLAP || NS * STAGE >= EPI, "epilogue staging does not fit the ring");
};

// Block tile BM x BN, WGM x WGN wavefront grid (four wavefronts), ring of NS stages.
// Step = 64 columns of K: 4 sub-steps of TM*TN MFMAs.  Every memory instruction rides behind an MFMA: during sub-steps
// 0..2 the fragment reads of the next sub-step, during sub-step 3 the first fragments of the NEXT step and the refill
// of this step's stage with step + NS.  The block barrier sits before sub-step 3: by then every wavefront has read all
// of this step's fragments (its stage is free) and has seen its own loads of the next step land, NS - 2 further steps
// still being in flight.
// A block walks over tiles (grid = the blocks that fit the chip at once).  With OVERLAP the first NS steps of the next
// tile are issued BEFORE the epilogue of the current one, so that the load latency of a tile start and the vector work
// and stores of a tile end (about 4 us and 6 us of a 19 us tile at K = 640) run beside each other.
template <int BM, int BN, bool GEGLU, int WGM, int WGN, int NS, bool OVERLAP>
__global__ void __launch_bounds__(256, (GemmCfg<BM, BN, NS, OVERLAP>::LDS <= 80 * 1024 ? 2 : 1))
gemm_mfma_kernel(GemmArgs a) {
    constexpr int BK = 64;
    constexpr int CH = BK / 8;                      // 16-byte chunks per row
    constexpr int WM = BM / WGM, WN = BN / WGN;     // wavefront tile
    constexpr int TM = WM / 32, TN = WN / 32;       // 32x32 MFMA tiles per wavefront
    constexpr int A_LD = BM * CH / 256;             // 16-byte loads per thread and K step
    constexpr int B_LD = BN * CH / 256;
    constexpr int LD = A_LD + B_LD;
    constexpr int STAGE_V = (BM + BN) * CH;         // 16-byte slots per stage: A rows then B rows
    static_assert(WGM * WGN == 4 && WM % 32 == 0 && WN % 32 == 0 && (BM * CH) % 256 == 0 && (BN * CH) % 256 == 0 &&
                  NS >= 2 && (NS - 1) * LD <= 63, "tile shape");
    static_assert(4 * WM * 36 * 4 <= GemmCfg<BM, BN, NS, OVERLAP>::EPI, "epilogue staging size");
    // Without a staging region of its own the epilogue stages in the drained ring.  Where the stages behind the first
    // hold that staging (4 wavefronts x WM rows x 36 floats), the first step of the next tile is loaded into stage 0
    // BEFORE the epilogue and the remaining stages after it: the load latency of a tile start (the long part of the
    // ~4 us a tile start costs at K = 640) passes beside the epilogue's vector work and stores.
    constexpr bool HALF = !OVERLAP && (NS - 1) * (BM + BN) * 128 >= 4 * WM * 36 * 4;
    extern __shared__ __attribute__((aligned(16))) uint8_t smem[];
    u32x4* ring = reinterpret_cast<u32x4*>(smem);                     // [NS][STAGE_V]
    int32_t* s_tok2 = reinterpret_cast<int32_t*>(ring + NS * STAGE_V); // [2][BM] output row of each tile row, -1 = none
    uint8_t* ep_smem = OVERLAP ? reinterpret_cast<uint8_t*>(s_tok2 + 2 * BM) : smem;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);      // scalar: LDS destinations of the loads are SGPR math
    const int wm = wave / WGN, wn = wave % WGN;
    // XCD-aware tile order.  Block ids are dealt round-robin to the 8 XCDs (each with its own L2), so the blocks of one
    // residue mod 8 run on one XCD; they take that XCD's slots in order, gridDim / 8 at a time.  An XCD owns every 8th
    // M tile; it takes them in groups of `gm` whose A panels together fit its L2, and walks a group M tile fastest,
    // then N tile: the blocks in flight share `gm` A panels and a few B panels, A is fetched once and B once per group
    // (N fastest, i.e. gm = 1, re-streams all of B for every M tile: 375 MB instead of 145 MB for a 5120 x 640 weight).
    const int n_tiles = a.N / BN, m_tiles = (a.M + BM - 1) / BM;
    const int mx = (m_tiles + 7) >> 3;              // M tiles per XCD
    const int64_t a_panel = (int64_t)BM * a.K * a.taps * 2;
    const int gm = (int)max((int64_t)1, min((int64_t)mx, (int64_t)(2560 * 1024) / a_panel));
    const int slots = mx * n_tiles, slot_step = gridDim.x >> 3;
    const int act_count = (a.tokens_are_rows && a.act.active) ? *a.act.count : 0;              // computed patches
    const int m_limit = (a.tokens_are_rows && a.act.active) ? act_count * a.geom.S : a.M;      // rows that exist
    // tile of a slot; false when it has no rows
    auto decode = [&](int slot, int& m0, int& n0) -> bool {
        const int grp = slot / (gm * n_tiles), r_in = slot - grp * (gm * n_tiles);
        const int gm_here = min(gm, mx - grp * gm); // the last group may be short
        const int n_tile = r_in / gm_here;
        const int m_tile = (grp * gm + (r_in - n_tile * gm_here)) * 8 + (blockIdx.x & 7);
        m0 = m_tile * BM;
        n0 = n_tile * BN;
        return m_tile < m_tiles && m0 < m_limit;
    };
    auto next_tile = [&](int slot, int& m0, int& n0) -> int {       // first slot >= `slot` of this block with rows
        while (slot < slots && !decode(slot, m0, n0)) slot += slot_step;
        return slot;
    };
    int m0 = 0, n0 = 0;
    int slot = next_tile(blockIdx.x >> 3, m0, n0);
    if (slot >= slots) return;

    // Staging by direct global -> LDS loads.  One wavefront instruction fills 64 consecutive 16-byte slots
    // (8 rows x 8 chunk positions); the lane at (row, position pos) fetches global chunk pos ^ f(row),
    // f(row) = (row >> 1) & 7, so the swizzle costs nothing.  Thread rows: lr + 32*i, position lc.
    const int lc = lane & 7, lr = 8 * wave + (lane >> 3);
    const int gc = lc ^ ((lr >> 1) & 7);            // global chunk this lane fetches (same for every i)
    int a_lane[A_LD], b_lane;                       // byte offsets of this lane's rows from the tensors' bases
    const int64_t b_row32 = (int64_t)32 * a.K;
    const int kchunks = a.K / BK;
    const int KT = a.taps * kchunks;
    const int64_t b_tap_stride = (int64_t)a.N * a.K;
    const int tap_w = a.tap_w ? a.tap_w : 3;
    int tap, kc, issued;                            // K step that is issued next (stays at the last one past the end:
                                                    // it is fetched again into a free stage and never read)

    // operand pointers and the row -> token table `tok_tab` of tile (tm0, tn0)
#define PS_SETUP(tm0, tn0, tok_tab)                                                                               \
    {                                                                                                             \
        /* the patch ids of all rows first (one memory round trip for the tile, not one per row) */              \
        int act_p[A_LD];                                                                                          \
        if (a.tokens_are_rows && a.act.active) {                                                                  \
            _Pragma("unroll") for (int i = 0; i < A_LD; ++i) {                                                    \
                const int pi = ((tm0) + lr + i * 32) / a.geom.S;                                                  \
                act_p[i] = pi < act_count ? a.act.active[pi] : -1;                                                \
            }                                                                                                     \
        }                                                                                                         \
        _Pragma("unroll") for (int i = 0; i < A_LD; ++i) {                                                        \
            const int row = lr + i * 32;                                                                          \
            int64_t tok = (tm0) + row;                                                                            \
            bool valid;                                                                                           \
            if (a.tokens_are_rows && a.act.active) {                                                              \
                const int pi = (int)tok / a.geom.S;                                                               \
                valid = act_p[i] >= 0;                                                                            \
                tok = valid ? (int64_t)act_p[i] * a.geom.S + ((int)tok - pi * a.geom.S) : 0;                      \
            } else {                                                                                              \
                valid = tok < a.M;                                                                                \
                if (!valid) tok = 0;                                                                              \
            }                                                                                                     \
            int64_t off, orow = tok;                                                                              \
            if (a.conv) {                                                                                         \
                const int p = (int)(tok / a.geom.S), q = (int)(tok - (int64_t)p * a.geom.S);                      \
                const int y = q / a.geom.pw, x = q - y * a.geom.pw;                                               \
                const int am = a.a_mul ? a.a_mul : 1;                                                             \
                off = ((int64_t)p * a.geom.pS + (am * y + a.a_dy) * a.geom.ppw + am * x + a.a_dx) * a.lda;        \
                if (a.o_mul) orow = (int64_t)p * a.o_S + (a.o_mul * y + a.o_dy) * a.o_pw + a.o_mul * x + a.o_dx;  \
            } else {                                                                                              \
                off = tok * a.lda;                                                                                \
            }                                                                                                     \
            a_lane[i] = (int)((off + gc * 8) * 2);                                                                \
            if (lc == 0) {                                                                                        \
                if (!a.tokens_are_rows && a.row_group > 0)                                                        \
                    orow = (tok / a.row_group) * a.row_group_pad + tok % a.row_group;                             \
                (tok_tab)[row] = valid ? (int32_t)orow : -1;                                                      \
            }                                                                                                     \
        }                                                                                                         \
        b_lane = (int)(((int64_t)((tn0) + lr) * a.K + gc * 8) * 2);                                               \
    }
    // one direct global->LDS load (64 lanes x 16 bytes): l < A_LD an A row group, else a B row group
    // (buffer loads rather than global loads into LDS: behind a flat-class load the compiler turns every wait for one
    // fragment into a wait for all LDS reads in flight; 2-4 % on every linear layer)
#if defined(__HIP_DEVICE_COMPILE__)
    const __amdgpu_buffer_rsrc_t ga_rsrc = __builtin_amdgcn_make_buffer_rsrc((void*)a.A, 0, 0x7fffffff, 0x00020000);
    const __amdgpu_buffer_rsrc_t gb_rsrc = __builtin_amdgcn_make_buffer_rsrc((void*)a.B, 0, 0x7fffffff, 0x00020000);
#define PS_LOAD(dst_, a_off_, b_off_, l_)                                                                         \
    {                                                                                                             \
        if ((l_) < A_LD)                                                                                          \
            __builtin_amdgcn_raw_ptr_buffer_load_lds(ga_rsrc, (lds_void*)((dst_) + (l_) * 256), 16,               \
                                                     a_lane[(l_) < A_LD ? (l_) : 0], (int)((a_off_) * 2), 0, 0);  \
        else if ((l_) < LD)                                                                                       \
            __builtin_amdgcn_raw_ptr_buffer_load_lds(gb_rsrc, (lds_void*)((dst_) + BM * CH + ((l_) - A_LD) * 256), 16, \
                                                     b_lane, (int)((((l_) - A_LD) * b_row32 + (b_off_)) * 2), 0, 0); \
    }
#else       // the host pass only needs the kernel's stub
#define PS_LOAD(dst_, a_off_, b_off_, l_) (void)0
#endif
    // global offsets of K step (tap, kc)
#define PS_OFFSETS(tap_, kc_)                                                                                     \
    const int ty_ = (tap_) / tap_w, tx_ = (tap_) - ty_ * tap_w;                                                   \
    const int64_t a_off = (a.conv ? ((int64_t)ty_ * a.geom.ppw + tx_) * a.lda : 0) + (kc_) * BK;                  \
    const int64_t b_off = (tap_) * b_tap_stride + (kc_) * BK;
    // the first NS steps of a tile: all stages in flight
#define PS_PROLOGUE_STAGES(st0_, st1_)                                                                            \
    {                                                                                                             \
        if ((st0_) == 0) { tap = 0; kc = 0; issued = 0; }                                                         \
        _Pragma("unroll") for (int st = (st0_); st < (st1_); ++st) {                                              \
            PS_OFFSETS(tap, kc);                                                                                  \
            u32x4* dst = ring + st * STAGE_V + wave * 64;                                                         \
            _Pragma("unroll") for (int l = 0; l < LD; ++l) PS_LOAD(dst, a_off, b_off, l);                         \
            if (++issued < KT) { if (++kc == kchunks) { kc = 0; ++tap; } } else { issued = KT - 1; }              \
        }                                                                                                         \
    }
#define PS_PROLOGUE() PS_PROLOGUE_STAGES(0, NS)

    const int fr = lane & 31, fh = lane >> 5;       // fragment row within a 32-row tile, k half
    // LDS fragment slots of this lane: row*CH + ((2*ks + fh) ^ f(row))
    int fa_base[TM], fa_sw[TM], fb_base[TN], fb_sw[TN];
#pragma unroll
    for (int i = 0; i < TM; ++i) { const int r = wm * WM + i * 32 + fr; fa_base[i] = r * CH; fa_sw[i] = (r >> 1) & 7; }
#pragma unroll
    for (int j = 0; j < TN; ++j) { const int r = wn * WN + j * 32 + fr; fb_base[j] = BM * CH + r * CH; fb_sw[j] = (r >> 1) & 7; }

    bf16x8 fa[2][TM], fb[2][TN];                    // register double buffer of the MFMA fragments
    // one fragment read (16 bytes per lane) of K sub-step ks_ into register set dst; r_ = 0: A tile 0, 1 .. TN: B tiles,
    // TN+1 ..: the remaining A tiles (the order in which the MFMAs of a sub-step first need them)
#define PS_READ_ONE(dst, stage_, ks_, r_)                                                                         \
    {                                                                                                             \
        const int c_ = (ks_) * 2 + fh;                                                                            \
        const int jb_ = ((r_) >= 1 && (r_) <= TN) ? (r_) - 1 : 0;                                             \
        const int ia_ = ((r_) > TN && (r_) < TM + TN) ? (r_) - TN : 0;                                        \
        if ((r_) == 0) fa[dst][0] = __builtin_bit_cast(bf16x8, (stage_)[fa_base[0] + (c_ ^ fa_sw[0])]);           \
        else if ((r_) <= TN) fb[dst][jb_] = __builtin_bit_cast(bf16x8, (stage_)[fb_base[jb_] + (c_ ^ fb_sw[jb_])]); \
        else if ((r_) < TM + TN) fa[dst][ia_] = __builtin_bit_cast(bf16x8, (stage_)[fa_base[ia_] + (c_ ^ fa_sw[ia_])]); \
    }
    constexpr int NM = TM * TN;                     // MFMAs per 16-wide sub-step
    constexpr int NR = TM + TN;                     // fragment reads per sub-step
    constexpr int R_PER = (NR + NM - 1) / NM;       // fragment reads slipped in behind one MFMA
    constexpr int L_PER = (LD + NM - 1) / NM;       // loads slipped in behind one MFMA of sub-step 3
    constexpr bool SKIP_TAIL = NS == 2;

    int buf = 0;                                    // token table of the current tile
    PS_SETUP(m0, n0, s_tok2);
    PS_PROLOGUE();
#pragma unroll 1
    for (;;) {
        f32x16 acc[TM][TN];
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;
        // stage 0 has landed when at most the NS - 1 later stages (and nothing issued after them) are in flight
        asm volatile("s_waitcnt vmcnt(%0)" ::"n"((NS - 1) * LD) : "memory");
        __syncthreads();                            // step 0 and the token table visible to everyone
#pragma unroll
        for (int r = 0; r < NR; ++r) PS_READ_ONE(0, ring, 0, r);

        int rd = 0;                                 // ring stage of the current step
#pragma unroll 1
        for (int kt = 0; kt < KT; ++kt) {
            const u32x4* cur = ring + rd * STAGE_V;
            const int nst = rd + 1 == NS ? 0 : rd + 1;
            const u32x4* nxt = ring + nst * STAGE_V;
            PS_OFFSETS(tap, kc);                    // step kt + NS goes into this step's stage
            if (++issued < KT) { if (++kc == kchunks) { kc = 0; ++tap; } } else { issued = KT - 1; }
            u32x4* dst = ring + rd * STAGE_V + wave * 64;
            // With two stages the barrier waits for ALL loads in flight (vmcnt(0)), so the last steps of a tile need not
            // keep the count up with loads of steps that do not exist: they issue none, and nothing is in flight when
            // the tile's epilogue starts (it used to wait out a memory round trip for them).
            const bool refill = kt + NS < KT;
#pragma unroll
            for (int ks = 0; ks < BK / 16; ++ks) {
                if (ks == BK / 16 - 1) {
                    // own fragment reads of this step are complete; own loads of the next step have landed.  A bare
                    // s_barrier: __syncthreads() carries a fence that waits for ALL loads in flight (vmcnt(0)), which
                    // would cut the ring down to one step ahead whatever its depth.
                    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_waitcnt vmcnt(%0)\n\ts_barrier" ::"n"((NS - 2) * LD) : "memory");
                }
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int j = 0; j < TN; ++j) {
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[ks & 1][i], fb[ks & 1][j], acc[i][j], 0, 0, 0);
                        const int q = i * TN + j;
#pragma unroll
                        for (int u = 0; u < R_PER; ++u) {
                            if (ks < BK / 16 - 1) { PS_READ_ONE((ks + 1) & 1, cur, ks + 1, q * R_PER + u); }
                            else { PS_READ_ONE(0, nxt, 0, q * R_PER + u); }
                        }
                        if (ks == BK / 16 - 1 && (!SKIP_TAIL || refill)) {
#pragma unroll
                            for (int u = 0; u < L_PER; ++u) PS_LOAD(dst, a_off, b_off, q * L_PER + u);
                        }
                        __builtin_amdgcn_sched_barrier(0);
                    }
            }
            rd = nst;
        }
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();                            // ring drained: free for the next tile (or the epilogue's staging)

        int nm0 = 0, nn0 = 0;
        const int nslot = next_tile(slot + slot_step, nm0, nn0);
        const int32_t* tok_cur = s_tok2 + buf * BM;
        const int n0_cur = n0;
        // the bias is read before the next tile's loads are issued: a wait for a load waits for all loads issued
        // before it, so a bias load behind them would stall the epilogue until the whole next tile start has landed
        float bias_t[TN];
#pragma unroll
        for (int j = 0; j < TN; ++j) bias_t[j] = a.bias ? a.bias[n0_cur + wn * WN + j * 32 + fr] : 0.f;
        asm volatile("" ::: "memory");              // keeps the compiler from sinking these loads below the next ones
        if (OVERLAP && nslot < slots) {             // next tile's first steps in flight during this tile's epilogue
            PS_SETUP(nm0, nn0, s_tok2 + (buf ^ 1) * BM);
            PS_PROLOGUE();
        } else if (HALF && nslot < slots) {         // its first step only: the epilogue stages in the stages behind it
            PS_SETUP(nm0, nn0, s_tok2 + (buf ^ 1) * BM);
            PS_PROLOGUE_STAGES(0, 1);
        }
        gemm_epilogue<BM, BN, GEGLU, WGM, WGN, false>(a, acc, HALF ? smem + STAGE_V * 16 : ep_smem, tok_cur, n0_cur, bias_t);
        if (nslot >= slots) break;
        if (!OVERLAP) {
            __syncthreads();                        // every wavefront is done with its staging region in the ring
            if (HALF) {
                PS_PROLOGUE_STAGES(1, NS);
            } else {
                PS_SETUP(nm0, nn0, s_tok2 + (buf ^ 1) * BM);
                PS_PROLOGUE();
            }
        }
        slot = nslot; m0 = nm0; n0 = nn0; buf ^= 1;
    }
#undef PS_READ_ONE
#undef PS_PROLOGUE
#undef PS_PROLOGUE_STAGES
#undef PS_OFFSETS
#undef PS_LOAD
#undef PS_SETUP
}

// ---- 3x3 convolution with the A operand kept in LDS across the nine taps -------------------------------------
// The M tile is a set of segments, each `seg_rows` whole pixel rows of one patch.  For every 64-channel chunk
// the haloed pixels of the segments ((seg_rows+2) x (pw+2) per segment, taken from the padded patch buffer) are
// loaded into LDS ONCE and the nine taps read them as nine shifted views, so the activation traffic from L2 /
// MALL is ~5x lower than re-loading a 128-row tile per tap.  Only the weights stream per (tap, chunk) step.
// LDS: [2 weight stages][2 halo stages of CONV_APIX pixel slots][row -> token table].
struct ConvTile {
    int32_t seg_rows, seg_tokens, nseg, seg_pix;    // seg_tokens = seg_rows*pw, seg_pix = (seg_rows+2)*(pw+2)
    // ceil(2^32 / d) for d = seg_pix, pw + 2, seg_tokens, pw: x / d == __umulhi(x, m) for the small x of the set-up
    // (x * d < 2^32; a true integer division is ~40 instructions, and 28 of them sat in front of the first halo load)
    uint32_t m_seg_pix, m_hw, m_seg_tokens, m_pw;
};
__device__ __forceinline__ int div_small(int x, uint32_t m, int d) { return d == 1 ? x : (int)__umulhi((uint32_t)x, m); }

// Template: block tile BM x BN, WGM x WGN wavefront grid (4 wavefronts), APIX halo pixel slots per stage
// (multiple of 32), NSB weight stages.
// KS = 2: eight wavefronts, two per SIMD.  Wavefronts w and w + 4 own the same output rows and split every 64-wide
// K step (sub-steps 0, 1 / 2, 3); the first four fetch the weights, the last four the halo; the partial sums meet in
// LDS before the epilogue, which the first four run.
template <int BM, int BN, int WGM, int WGN, int APIX, int NSB, int KS>
__global__ void __launch_bounds__(256 * KS)
conv_mfma_kernel(GemmArgs a, ConvTile ct) {
    constexpr int BK = 64, CH = 8;
    constexpr int WM = BM / WGM, WN = BN / WGN, TM = WM / 32, TN = WN / 32;
    constexpr int B_LD = BN * CH / 256, A_LD = APIX * CH / 256;
    constexpr int BSTAGE = BN * CH, ASTAGE = APIX * CH;            // 16-byte slots
    static_assert(WGM * WGN == 4 && (BN * CH) % 256 == 0 && (APIX * CH) % 256 == 0 && (NSB == 2 || NSB == 3), "conv tile");
    static_assert(KS == 1 || KS == 2, "K split");
    extern __shared__ __attribute__((aligned(16))) uint8_t smem[];
    u32x4* sB = reinterpret_cast<u32x4*>(smem);                    // [NSB][BSTAGE]
    u32x4* sA = sB + NSB * BSTAGE;                                 // [2][ASTAGE]
    int32_t* s_tok = reinterpret_cast<int32_t*>(sA + 2 * ASTAGE);  // [BM]
    int32_t* s_seg = s_tok + BM;                                   // [nseg] padded-pixel index of each segment's halo origin

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave_all = __builtin_amdgcn_readfirstlane(tid >> 6);  // scalar: LDS destinations of the loads are SGPR math
    const int wave = wave_all & 3, kg = KS == 1 ? 0 : wave_all >> 2;    // place in the wavefront grid, K group
    const bool pro_b = kg == 0, pro_a = kg == KS - 1;            // who issues the first weight stages / the first halo
    const int wm = wave / WGN, wn = wave % WGN;
    // XCD-aware tile order: block ids are dealt round-robin to the 8 XCDs, so all N tiles of one M tile get ids of
    // the same residue mod 8 and consecutive slots: they run on one XCD back to back and share the A tile in its L2
    const int n_tiles = a.N / BN, m_tiles = (a.M + BM - 1) / BM;
    const int slot = blockIdx.x >> 3;
    const int m_tile = (slot / n_tiles) * 8 + (blockIdx.x & 7);
    if (m_tile >= m_tiles) return;
    const int m0 = m_tile * BM, n0 = (slot % n_tiles) * BN;
    if (a.act.active && m0 >= *a.act.count * a.geom.S) return;
    const int S = a.geom.S, pw = a.geom.pw, hw = pw + 2;

    // one direct global->LDS load (64 lanes x 16 bytes) of the weight / halo stage
    // Buffer loads into LDS rather than global loads into LDS: behind a flat-class load the compiler takes the LDS
    // counter for out of order and turns every wait for ONE fragment into a wait for all reads in flight
    // (lgkmcnt(0)), the read issued an instruction earlier included; behind buffer loads it counts (lgkmcnt(4..0)
    // down a row of MFMAs): 498 -> 487 us at C = 640 on 79 k rows, 374 -> 358 us at C = 1280.  Offsets are 32-bit
    // byte offsets from the tensor's base (the launch checks that both tensors stay below 2^31 bytes).
#if defined(__HIP_DEVICE_COMPILE__)
    const __amdgpu_buffer_rsrc_t b_rsrc = __builtin_amdgcn_make_buffer_rsrc((void*)a.B, 0, 0x7fffffff, 0x00020000);
    const __amdgpu_buffer_rsrc_t a_rsrc = __builtin_amdgcn_make_buffer_rsrc((void*)a.A, 0, 0x7fffffff, 0x00020000);
#define PS_LOAD_B(dstB_, off_, i_) \
    __builtin_amdgcn_raw_ptr_buffer_load_lds(b_rsrc, (lds_void*)((dstB_) + (i_) * 256), 16, b_lane, (int)(((i_) * b_row32 + (off_)) * 2), 0, 0)
#define PS_LOAD_A(dstA_, off_, i_) \
    __builtin_amdgcn_raw_ptr_buffer_load_lds(a_rsrc, (lds_void*)((dstA_) + (i_) * 256), 16, a_pos[i_], (int)((off_) * 2), 0, 0)
#else       // the host pass only needs the kernel's stub
#define PS_LOAD_B(dstB_, off_, i_) (void)0
#define PS_LOAD_A(dstA_, off_, i_) (void)0
#endif

    // The weights of the first NSB steps go first: they need no table, and the index arithmetic below runs while
    // they are in flight.  Thread rows lr + 32*i, chunk position lc; the lane fetches global chunk lc ^ f(row).
    const int lc = lane & 7, lr = 8 * wave + (lane >> 3);
    const int gc = lc ^ ((lr >> 1) & 7);
    const int b_lane = (int)(((int64_t)(n0 + lr) * a.K + gc * 8) * 2);   // byte offset of this lane's first weight row
    const int64_t b_row32 = (int64_t)32 * a.K;
    const int64_t b_tap_stride = (int64_t)a.N * a.K;
    const int kchunks = a.K / BK;
    int itap = 0, ikc = 0;                          // (tap, chunk) of the next weight stage to issue; clamps at the last step
#pragma unroll
    for (int t = 0; t < NSB; ++t) {
        u32x4* dB = sB + t * BSTAGE + wave * 64;
        const int64_t off = itap * b_tap_stride + ikc * BK;
        if (pro_b) {
#pragma unroll
            for (int i = 0; i < B_LD; ++i) PS_LOAD_B(dB, off, i);
        }
        if (!(itap == 8 && ikc == kchunks - 1)) { if (++itap == 9) { itap = 0; ++ikc; } }
    }

    // row -> token table and segment origins
    if (tid < BM) {
        const int ri = m0 + tid;
        int64_t tok;
        bool valid;
        if (a.act.active) {
            const int pi = ri / S;
            valid = pi < *a.act.count;
            tok = valid ? (int64_t)a.act.active[pi] * S + (ri - pi * S) : 0;
        } else {
            valid = ri < a.M;
            tok = valid ? ri : 0;
        }
        s_tok[tid] = valid ? (int32_t)tok : -1;
        if (tid % ct.seg_tokens == 0) {
            const int p = (int)(tok / S), q = (int)(tok - (int64_t)p * S);
            s_seg[tid / ct.seg_tokens] = p * a.geom.pS + (q / pw) * a.geom.ppw;    // padded pixel of halo (0, 0)
        }
    }
    __syncthreads();

    const uint16_t* A = (const uint16_t*)a.A;
    int32_t a_pos[A_LD];                            // byte offsets (the launch checks that the padded buffer stays below 2^31 bytes)
    const int apix = ct.nseg * ct.seg_pix;
#pragma unroll
    for (int i = 0; i < A_LD; ++i) {
        int sl = lr + 32 * i;
        if (sl >= apix) sl = 0;                                    // unused slots re-read a valid pixel
        const int g = div_small(sl, ct.m_seg_pix, ct.seg_pix), l = sl - g * ct.seg_pix;
        const int ly = div_small(l, ct.m_hw, hw), lx = l - ly * hw;
        a_pos[i] = ((s_seg[g] + ly * a.geom.ppw + lx) * (int32_t)a.lda + gc * 8) * 2;
    }
    if (pro_a) {                                    // halo of chunk 0: in flight during the rest of the set-up
        u32x4* dA = sA + wave * 64;
#pragma unroll
        for (int i = 0; i < A_LD; ++i) PS_LOAD_A(dA, 0, i);
    }
    f32x16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;


    const int fr = lane & 31, fh = lane >> 5;
    // halo slot of each fragment row for tap (0, 0)
    int fa_slot[TM];
#pragma unroll
    for (int i = 0; i < TM; ++i) {
        const int r = wm * WM + i * 32 + fr;
        const int g = div_small(r, ct.m_seg_tokens, ct.seg_tokens), rr = r - g * ct.seg_tokens;
        const int ry = div_small(rr, ct.m_pw, pw), rx = rr - ry * pw;
        fa_slot[i] = g * ct.seg_pix + ry * hw + rx;
    }
    // weight fragment j: row wn*WN + 32*j + fr; the chunk swizzle (row >> 1) & 7 is the same for every j
    const int fb_base0 = (wn * WN + fr) * CH, fb_sw0 = ((wn * WN + fr) >> 1) & 7;

    // fragment registers: two sets, filled one sub-step ahead.  With the K split (256 registers per wavefront) the
    // weight fragments have one set: fb[j] is refilled right behind the last MFMA of the sub-step that reads it.
    constexpr int FBS = KS == 1 ? 2 : 1;
    bf16x8 fa[2][TM], fb[FBS][TN];
    // one fragment read (16 bytes per lane) of K sub-step ks_ into register set dst; r_ = 0: A tile 0, 1 .. TN: B tiles,
    // TN+1 ..: the remaining A tiles (the order in which the MFMAs of a sub-step first need them)
#define PS_READ_ONE(dst, stA_, stB_, cur_, sw_, ks_, r_)                                                          \
    {                                                                                                             \
        const int c_ = ((ks_) + koff) * 2 + fh;                                                                   \
        const int jb_ = ((r_) >= 1 && (r_) <= TN) ? (r_) - 1 : 0;                                             \
        const int ia_ = ((r_) > TN && (r_) < TM + TN) ? (r_) - TN : 0;                                        \
        if ((r_) == 0) fa[dst][0] = __builtin_bit_cast(bf16x8, (stA_)[cur_[0] * CH + (c_ ^ sw_[0])]);             \
        else if ((r_) <= TN) fb[(dst) & (FBS - 1)][jb_] = __builtin_bit_cast(bf16x8, (stB_)[fb_base0 + jb_ * 32 * CH + (c_ ^ fb_sw0)]); \
        else if ((r_) < TM + TN) fa[dst][ia_] = __builtin_bit_cast(bf16x8, (stA_)[cur_[ia_] * CH + (c_ ^ sw_[ia_])]); \
    }

    constexpr int NM = TM * TN;                     // MFMAs per 16-wide sub-step
    constexpr int NR = TM + TN;                     // fragment reads per sub-step
    constexpr int R_PER = (NR + NM - 1) / NM;       // fragment reads slipped in behind one MFMA
    constexpr int SUB = BK / 16 / KS;               // sub-steps of a step one wavefront computes
    constexpr int A_PER = (A_LD + (SUB - 1) * NM - 1) / ((SUB - 1) * NM);   // halo loads slipped in per MFMA before the last sub-step
    static_assert(B_LD <= NM, "weight loads are interleaved one per MFMA");
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    // The loop comes in three forms, chosen per wavefront: 0 = no K split (all sub-steps, both kinds of loads),
    // 1 = first half of every step + the weight loads, 2 = second half + the halo loads.
    auto main_loop = [&](auto role_c) {
        constexpr int ROLE = decltype(role_c)::value;
        constexpr bool issue_b = ROLE != 2, issue_a = ROLE != 1;
        constexpr int koff = ROLE == 2 ? SUB : 0;       // first sub-step of this wavefront
        // MFMAs of a step's last sub-step that a wavefront issues IN FRONT of the block barrier (K split only).  With the
        // barrier at the head of the sub-step a wavefront reaches it right behind its last fragment reads and waits out
        // their LDS latency there.  A few MFMAs later the reads have landed: those MFMAs take fragments read a
        // sub-step earlier, and everything that must follow the barrier (the next step's first fragments, the refill
        // of this step's weight stage) moves behind the remaining MFMAs.  Different slots for the two K groups keep the
        // two wavefronts of a SIMD from reaching their sub-step boundaries together.  Worth 3 % while every wait for a
        // fragment was a wait for all reads in flight (see the loads above), about 1 % since.
        constexpr int QB = KS == 1 ? 0 : (ROLE == 1 ? 2 : 5);
        static_assert(QB + B_LD <= NM && QB + TM <= NM && QB <= NM - TN, "barrier slot");
        int fa_cur[TM], fa_sw[TM];
#pragma unroll
        for (int i = 0; i < TM; ++i) { fa_cur[i] = fa_slot[i]; fa_sw[i] = (fa_cur[i] >> 1) & 7; }
#pragma unroll
        for (int r = 0; r < NR; ++r) PS_READ_ONE(0, sA, sB, fa_cur, fa_sw, 0, r);

        // Step = (chunk kc, tap): 4 sub-steps of NM MFMAs.  Every memory instruction rides behind an MFMA: during
        // sub-steps 0..2 the fragment reads of the next sub-step (and, in tap 0, the halo of the next chunk), during
        // sub-step 3 the first fragments of the NEXT step and the refill of this step's weight stage.  The block barrier
        // sits in sub-step 3 (at its head, or QB MFMAs into it): by then every wavefront has read all of this step's
        // fragments (its stage is free) and has seen its own loads of the next step's weights land.
        int bst = 0;                                    // weight stage of the current step
        // The two wavefronts of a SIMD compete for the matrix pipe, and the older one (the first K group) wins every
        // time both have an MFMA ready: it runs ahead to the barrier and waits there a third of the loop's time
        // (timestamps of a work build) while the second group finishes the step on its own.  With the second group
        // at the higher priority the first one fills the gaps instead: 1-2 % (347 -> 339 us at C = 1280).
        if (ROLE == 2) asm volatile("s_setprio 2" ::: "memory");
        for (int kc = 0; kc < kchunks; ++kc) {
            const u32x4* curA = sA + (kc & 1) * ASTAGE;
            const int nkc_a = kc + 1 < kchunks ? kc + 1 : kc;   // halo chunk fetched during tap 0 (last: itself, never read)
            u32x4* dA = sA + ((kc & 1) ^ 1) * ASTAGE + wave * 64;
            const int a_off = nkc_a * BK;
#pragma unroll 1
            for (int tap = 0; tap < 9; ++tap) {
                const u32x4* curB = sB + bst * BSTAGE;
                const int nst = bst + 1 == NSB ? 0 : bst + 1;
                const u32x4* nxtB = sB + nst * BSTAGE;
                const int ntap = tap == 8 ? 0 : tap + 1;
                const u32x4* nxtA = tap == 8 ? sA + ((kc & 1) ^ 1) * ASTAGE : curA;
                const int nty = ntap / 3, ntx = ntap - nty * 3;
                int nfa_cur[TM], nfa_sw[TM];
#pragma unroll
                for (int i = 0; i < TM; ++i) { nfa_cur[i] = fa_slot[i] + nty * hw + ntx; nfa_sw[i] = (nfa_cur[i] >> 1) & 7; }
                const int64_t b_off = itap * b_tap_stride + ikc * BK;
                if (!(itap == 8 && ikc == kchunks - 1)) { if (++itap == 9) { itap = 0; ++ikc; } }
                u32x4* dB = sB + bst * BSTAGE + wave * 64;
#pragma unroll
                for (int ks = 0; ks < SUB; ++ks) {
                    auto step_barrier = [&] {
                        // own fragment reads of this step are complete; own loads of the next step's weights have landed.
                        // Still allowed in flight: the NSB-2 later weight stages and a halo issued in this or a recent tap 0.
                        // A bare s_barrier: __syncthreads() carries a fence that waits for ALL loads in flight (vmcnt(0)),
                        // which would cut the weight ring down to one step ahead whatever its depth.
                        // With the K split a wavefront waits for the kind it fetches: weights as above, or the halo (needed
                        // from tap 8 on, issued in tap 0).
                        if (KS == 1 ? tap < NSB - 1 : (!issue_b && tap == 0))
                            asm volatile("s_waitcnt lgkmcnt(0)\n\ts_waitcnt vmcnt(%0)\n\ts_barrier" ::"n"((KS == 1 ? (NSB - 2) * B_LD : 0) + A_LD) : "memory");
                        else if (KS == 1 || issue_b)
                            asm volatile("s_waitcnt lgkmcnt(0)\n\ts_waitcnt vmcnt(%0)\n\ts_barrier" ::"n"((NSB - 2) * B_LD) : "memory");
                        else
                            asm volatile("s_waitcnt lgkmcnt(0)\n\ts_waitcnt vmcnt(0)\n\ts_barrier" ::: "memory");
                    };
#pragma unroll
                    for (int i = 0; i < TM; ++i)
#pragma unroll
                        for (int j = 0; j < TN; ++j) {
                            const int q = i * TN + j;
                            if (ks == SUB - 1 && q == QB) step_barrier();
                            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[ks & 1][i], fb[ks & (FBS - 1)][j], acc[i][j], 0, 0, 0);
                            if (KS == 1) {
#pragma unroll
                                for (int u = 0; u < R_PER; ++u) {
                                    if (ks < SUB - 1) { PS_READ_ONE((ks + 1) & 1, curA, curB, fa_cur, fa_sw, ks + 1, q * R_PER + u); }
                                    else { PS_READ_ONE(0, nxtA, nxtB, nfa_cur, nfa_sw, 0, q * R_PER + u); }
                                }
                            } else {
                                // A fragments of the next sub-step behind the first TM MFMAs (other register set), B fragment j
                                // behind the last MFMA that reads the current one (i == TM - 1)
                                const int r = q < TM ? (q == 0 ? 0 : TN + q) : (i == TM - 1 ? 1 + j : NR);
                                if (ks < SUB - 1) { PS_READ_ONE((ks + 1) & 1, curA, curB, fa_cur, fa_sw, ks + 1, r); }
                                else {
                                    // behind the barrier only: the A fragments from slot QB on, B fragment j where it was
                                    const int qa = q - QB;
                                    const int ra = (qa >= 0 && qa < TM) ? (qa == 0 ? 0 : TN + qa) : NR;
                                    const int rb = i == TM - 1 ? 1 + j : NR;
                                    PS_READ_ONE(0, nxtA, nxtB, nfa_cur, nfa_sw, 0, ra);
                                    PS_READ_ONE(0, nxtA, nxtB, nfa_cur, nfa_sw, 0, rb);
                                }
                            }
                            if (ks == SUB - 1) {
                                if (q >= QB && q < QB + B_LD && issue_b) PS_LOAD_B(dB, b_off, q - QB);
                            } else {
#pragma unroll
                                for (int u = 0; u < A_PER; ++u) {
                                    const int qa = (ks * NM + q) * A_PER + u;
                                    if (qa < A_LD && tap == 0 && issue_a) PS_LOAD_A(dA, a_off, qa);
                                }
                            }
                            __builtin_amdgcn_sched_barrier(0);
                        }
                }
#pragma unroll
                for (int i = 0; i < TM; ++i) { fa_cur[i] = nfa_cur[i]; fa_sw[i] = nfa_sw[i]; }
                bst = nst;
            }
        }
    };
    if (KS == 1) main_loop(std::integral_constant<int, 0>{});
    else if (kg == 0) main_loop(std::integral_constant<int, 1>{});
    else main_loop(std::integral_constant<int, 2>{});
#undef PS_READ_ONE
#undef PS_LOAD_A
#undef PS_LOAD_B
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    // The lane's bias of each tile column, loaded here in one batch: inside the epilogue the load of a column sits
    // behind the staging of the previous one (a memory round trip per column); here it hides behind the exchange
    // (1.5 us of a 60 us kernel).
    float bias_t[TN];
#pragma unroll
    for (int j = 0; j < TN; ++j) bias_t[j] = a.bias ? a.bias[n0 + wn * WN + j * 32 + fr] : 0.f;
    if (KS == 2) {
        // the partial sums of wavefront w + 4 go to wavefront w through the drained ring, half the tile columns at a
        // time; the first four wavefronts then run the epilogue
        constexpr int JH = (TN + 1) / 2;
        static_assert(KS == 1 || 4 * JH * TM * 16 * 64 * 4 <= (NSB * BSTAGE + 2 * ASTAGE) * 16, "exchange does not fit the ring");
        f32x4* xch = reinterpret_cast<f32x4*>(smem) + wave * (JH * TM * 4 * 64) + lane;
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const int j0 = h * JH, j1 = h ? TN : JH;
            if (kg == 1) {
#pragma unroll
                for (int j = j0; j < j1; ++j)
#pragma unroll
                    for (int i = 0; i < TM; ++i)
#pragma unroll
                        for (int q = 0; q < 4; ++q) {
                            const f32x4 v = {acc[i][j][4 * q], acc[i][j][4 * q + 1], acc[i][j][4 * q + 2], acc[i][j][4 * q + 3]};
                            xch[(((j - j0) * TM + i) * 4 + q) * 64] = v;
                        }
            }
            __syncthreads();
            if (kg == 0) {
#pragma unroll
                for (int j = j0; j < j1; ++j)
#pragma unroll
                    for (int i = 0; i < TM; ++i)
#pragma unroll
                        for (int q = 0; q < 4; ++q) {
                            const f32x4 v = xch[(((j - j0) * TM + i) * 4 + q) * 64];
#pragma unroll
                            for (int e = 0; e < 4; ++e) acc[i][j][4 * q + e] += v[e];
                        }
            }
            __syncthreads();
        }
        if (kg == 1) return;
    }
    // the launch conditions of these kernels rule the other paths out (conv_select)
    gemm_epilogue<BM, BN, false, WGM, WGN, true, 0>(a, acc, smem, s_tok, n0, bias_t);
}

template <int BM, int BN, int WGM, int WGN, int APIX, int NSB, int KS = 1>
static int launch_conv(const GemmArgs& a, const ConvTile& ct, hipStream_t st) {
    constexpr size_t lds = (size_t)(NSB * BN + 2 * APIX) * 128 + BM * sizeof(int32_t) + 64 * sizeof(int32_t);
    static_assert(lds <= 160 * 1024, "conv LDS budget");
    PS_SET_LDS_ONCE((conv_mfma_kernel<BM, BN, WGM, WGN, APIX, NSB, KS>), lds);
    const unsigned grid = (unsigned)(8 * cdiv(cdiv(a.M, BM), 8) * (a.N / BN));
    conv_mfma_kernel<BM, BN, WGM, WGN, APIX, NSB, KS><<<grid, 256 * KS, lds, st>>>(a, ct);
    return check_launch("conv_mfma_kernel");
}

// Tile geometry of the halo-in-LDS convolution; false if the patch shape does not fit it.
static bool conv_tile(const GemmArgs& a, int BM, int apix_max, ConvTile* ct) {
    const int pw = a.geom.pw, ph = a.geom.ph;
    if (!a.conv || !a.tokens_are_rows || a.taps != 9 || BM % pw != 0) return false;
    int R = BM / pw;
    if (R > ph) R = ph;
    if (ph % R != 0 || BM % (R * pw) != 0) return false;
    ct->seg_rows = R;
    ct->seg_tokens = R * pw;
    ct->nseg = BM / ct->seg_tokens;
    ct->seg_pix = (R + 2) * (pw + 2);
    auto magic = [](int d) { return (uint32_t)((((uint64_t)1 << 32) + d - 1) / d); };      // d == 1 is handled apart
    ct->m_seg_pix = magic(ct->seg_pix);
    ct->m_hw = magic(pw + 2);
    ct->m_seg_tokens = magic(ct->seg_tokens);
    ct->m_pw = magic(pw);
    return ct->nseg * ct->seg_pix <= apix_max && ct->nseg <= 64;
}

template <int BM, int BN, bool GEGLU, int WGM, int WGN, int NS, bool OVERLAP>
static int launch(const GemmArgs& a, hipStream_t st) {
    constexpr size_t lds = GemmCfg<BM, BN, NS, OVERLAP>::LDS;
    PS_SET_LDS_ONCE((gemm_mfma_kernel<BM, BN, GEGLU, WGM, WGN, NS, OVERLAP>), lds);
    // all tiles, or as many blocks as run at once (256 CUs x the blocks of this LDS size per CU): each block then
    // walks over several tiles
    const int64_t all = 8 * cdiv(cdiv(a.M, BM), 8) * (a.N / BN);
    const int64_t resident = 256 * (int64_t)std::max<size_t>(1, std::min<size_t>(2, (160 * 1024) / lds));
    const unsigned grid = (unsigned)std::min(all, resident);
    gemm_mfma_kernel<BM, BN, GEGLU, WGM, WGN, NS, OVERLAP><<<grid, 256, lds, st>>>(a);
    return check_launch("gemm_mfma_kernel");
}

// shapes the MFMA kernels take at all
static bool mfma_eligible(const GemmArgs& a) {
    // the kernels stage both operands by buffer loads with 32-bit byte offsets from the tensors' bases
    const int64_t a_rows = a.conv ? (int64_t)a.geom.P * a.geom.pS : (int64_t)a.M;
    const bool fits = a_rows * a.lda < ((int64_t)1 << 30) && (int64_t)a.taps * a.N * a.K < ((int64_t)1 << 30);
    return a.K % 64 == 0 && a.lda % 8 == 0 && !((uintptr_t)a.A & 15) && !((uintptr_t)a.B & 15) && fits;
}

// Which halo-in-LDS convolution kernel a problem takes (0: none) and the columns one wavefront of it covers.
// Preferred: 256 x 160 tiles, four wavefronts stacked along M (each 64 x 160), three weight stages: half the weight
// bytes per MFMA of the 128 x 320 tile at the same accumulator shape.  That tile runs with the K split (eight
// wavefronts): 66 instead of 70 us at C = 320 / 29,696 tokens, 541 instead of 576 us at C = 640 / about 79,000 tokens.
static int conv_select(const GemmArgs& a, ConvTile* ct, int* wave_cols = nullptr) {
    int wc = 0, sel = 0;
    const bool plain3x3 = a.taps == 9 && (a.tap_w == 0 || a.tap_w == 3) && a.a_mul <= 1 && !a.a_dy && !a.a_dx && !a.o_mul;
    // the kernels address the padded patch buffer and the weights with 32-bit byte offsets below 2^31
    const bool fits32 = (int64_t)a.geom.P * a.geom.pS * a.lda < ((int64_t)1 << 30) &&
                        (int64_t)a.taps * a.N * a.K < ((int64_t)1 << 30);
    // no gate, no GELU, no transposed segment; a per-request bias only where a wavefront's 64 rows lie in one patch (the
    // kernels compile the epilogue without those paths)
    const bool lean = a.seg[0].scale == 1.f && !a.rowscale && !a.act_gelu && (!a.rowbias || (a.geom.S % 64 == 0 && a.geom.pw <= 64 && 64 % a.geom.pw == 0));
    if (plain3x3 && fits32 && lean && a.epi == EPI_ROUTE && a.seg_cols % 32 == 0 && a.seg_cols == a.N && !a.seg[0].transposed) {
        if (a.N % 160 == 0 && conv_tile(a, 256, 384, ct)) { sel = 1; wc = 160; }
        // small patches (8 x 8: four segments of 10 x 10 pixels per 256 rows) need more halo slots than that tile's LDS
        // has beside three weight stages; with two weight stages 416 slots fit
        else if (a.N % 160 == 0 && conv_tile(a, 256, 416, ct)) { sel = 6; wc = 160; }
        else if (conv_tile(a, 128, 256, ct)) {
            if (a.N % 320 == 0) { sel = 2; wc = 160; }
            else if (a.N % 256 == 0) { sel = 3; wc = 128; }
            else if (a.N % 128 == 0) { sel = 4; wc = 64; }
            else if (a.N % 64 == 0) { sel = 5; wc = 32; }
        }
    }
    if (wave_cols) *wave_cols = wc;
    return sel;
}

bool gemm_emits_stats(const GemmArgs& a, int dtype, int mode) {
    if (mode != 0 || dtype != PSERVE_BF16 || !a.stats || a.stats_G <= 0 || !mfma_eligible(a)) return false;
    ConvTile ct;
    int wc = 0;
    if (!conv_select(a, &ct, &wc)) return false;
    // a wavefront's 64 rows must lie in one patch, and its columns must hold whole groups
    return a.geom.S % 64 == 0 && a.stats_slots == a.geom.S / 64 && !a.act.active && a.N % a.stats_G == 0 &&
           wc % (a.N / a.stats_G) == 0;
}

int gemm_mfma_bf16(const GemmArgs& a, hipStream_t st, bool* handled) {
    *handled = false;
    if (!mfma_eligible(a)) return PSERVE_OK;
    if (a.epi == EPI_GEGLU) {
        if (a.N % 128 != 0) return PSERVE_OK;
        *handled = true;
        // The epilogue (GELU of every gate) is as long as the main loop at K = 640: with at least a round of 128-row
        // tiles, two blocks per CU, one block's epilogue runs beside the other's main loop (163 -> 142 us at
        // 13,312 x 5,120 x 640); the wavefront tile is then 32 x 128 = [64 values | 64 gates]
        if (cdiv(a.M, 128) * (a.N / 128) >= 512) return launch<128, 128, true, 4, 1, 2, false>(a, st);
        return launch<256, 128, true, 4, 1, 2, true>(a, st);
    }
    if (a.seg_cols % 32 != 0) return PSERVE_OK;      // a 32-column tile must not straddle output segments
    ConvTile ct;
    switch (conv_select(a, &ct)) {
    case 1: *handled = true; return launch_conv<256, 160, 4, 1, 384, 3, 2>(a, ct, st);
    case 2: *handled = true; return launch_conv<128, 320, 2, 2, 256, 2>(a, ct, st);
    case 3: *handled = true; return launch_conv<128, 256, 2, 2, 256, 2>(a, ct, st);
    case 4: *handled = true; return launch_conv<128, 128, 2, 2, 256, 2>(a, ct, st);
    case 5: *handled = true; return launch_conv<128, 64, 2, 2, 256, 2>(a, ct, st);
    case 6: *handled = true; return launch_conv<256, 160, 4, 1, 416, 2, 2>(a, ct, st);
    default: break;
    }
    // Tile choice.  Two blocks of 128 rows per CU where they fit (one block's prologue and epilogue run beside the
    // other's main loop), 256-row tiles with one block per CU (two stages, the next tile's first loads issued before
    // the epilogue) where the rounds of tiles come out better, and for few rows altogether (the text-token
    // projections) the narrowest tile.
    const int64_t m256 = cdiv(a.M, 256), m128 = cdiv(a.M, 128);
    *handled = true;
    const bool has_t = a.seg[0].transposed || a.seg[1].transposed || a.seg[2].transposed;
    // N a multiple of 160: 128 x 160 tiles, two blocks per CU (wavefront tile 32 x 160).  Against the 256 x 160 tile
    // the rounds are the same: 34 -> 28 us (13,312 x 640 x 640), 68 -> 63 us (K = 2560), 80 -> 72 us
    // (13.4 k x 1280 x 1280), 165 -> 137 us (79 k x 640 x 640).  The fused q/k/v projections (N = 1920, 3840, with the
    // transposed V^T segment and its long epilogue of 8-byte stores) gain 6-11 % over 128 x 128 tiles as well.
    if (a.N % 160 == 0 && m128 * (a.N / 160) >= 256) return launch<128, 160, false, 4, 1, 2, false>(a, st);
    const int64_t tiles128 = a.N % 128 == 0 ? m128 * (a.N / 128) : 0;
    // a transposed segment otherwise: 128 x 128, two blocks per CU (70 -> 62 us and 212 -> 184 us against 256-row tiles)
    if (has_t && tiles128 >= 512) return launch<128, 128, false, 2, 2, 2, false>(a, st);
    // Tile-count quantisation decides between the 256-row tiles (one block per CU: a started round of 256 tiles costs a
    // whole round) and 128 x 128 with two blocks per CU (512 per round; a last round that is at most half full leaves
    // one block per CU, which runs faster alone: about 0.65 of a round).  A full round of either does the same work
    // in about the same time (measured at K = 1536 and 6144), so the cost is rounds x outputs per CU and round.
    int bn_a = 0;
    if (a.N % 160 == 0 && m256 * (a.N / 160) >= 160) bn_a = 160;
    else if (a.N % 128 == 0 && m256 * (a.N / 128) >= 160) bn_a = 128;
    if (bn_a) {
        const int64_t tiles_a = m256 * (a.N / bn_a);
        if (tiles128 >= 512) {
            const double cost_a = (double)cdiv(tiles_a, 256) * 256 * bn_a;
            const int64_t full = tiles128 / 512, rest = tiles128 % 512;
            const double cost_b = ((double)full + (rest == 0 ? 0.0 : (rest <= 256 ? 0.65 : 1.0))) * 2 * 128 * 128;
            if (cost_b < cost_a) return launch<128, 128, false, 2, 2, 2, false>(a, st);
        }
        if (bn_a == 160) return launch<256, 160, false, 4, 1, 2, true>(a, st);
        return launch<256, 128, false, 4, 1, 2, true>(a, st);
    }
    const bool small = a.N % 64 == 0 && m128 * cdiv(a.N, 320) < 128;
    if (!small) {
        if (a.N % 320 == 0) return launch<128, 320, false, 2, 2, 2, true>(a, st);
        if (a.N % 256 == 0) return launch<128, 256, false, 2, 2, 2, true>(a, st);
        if (a.N % 128 == 0) return launch<128, 128, false, 2, 2, 3, true>(a, st);
    }
    if (a.N % 64 == 0) return launch<128, 64, false, 2, 2, 3, false>(a, st);
    *handled = false;
    return PSERVE_OK;
}

}  // namespace pserve
