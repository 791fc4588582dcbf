// bf16 MFMA flash attention over the patch batch (head dim 64), gfx950.
//
// Every query token attends to all tokens of its own image ("Patch-based Self-Attention
// Module"); the key range of request slot s is cu_seqlens[s] .. cu_seqlens[s+1] of the
// patch-major token matrix (RequestOffset of the CSP format times the tokens per patch), so
// no image is reassembled.  Cross-attention uses the request's own text tokens as keys.
//
// Work item = (query tile of 256 compact rows of ONE image, head).  4 wavefronts x 64 queries.
// Scores are formed transposed, S^T = K Q^T, so that a lane owns one query column of each
// 32x32 MFMA tile: the softmax row reductions are in-lane plus one exchange between the two
// lane halves, and the probabilities leave the accumulators already in the layout of the
// B operand of O^T = V^T P^T (the MFMA rows are assigned to keys so that a lane's eight scores
// of a 16-wide MFMA step are eight consecutive keys; V^T is read from LDS in the same order).  V is kept transposed in
// memory ([C][tokens]) by the projection GEMM, so both K and V^T tiles are plain 128-byte
// rows.  Online softmax in base 2 (logits pre-scaled by log2(e)/sqrt(d)), fp32 statistics.
//
// Blocks are numbered so that the blocks resident on one XCD (block id mod 8) walk
// consecutive query tiles of the same head: the K / V^T tiles they stream are then shared
// through that XCD's L2.  Within a head the largest images come first.
#include "kernels.h"

namespace pserve {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;

// queries per block = 4 wavefronts x 32 * QT queries.  QT = 2 (256 queries, 222 registers, two blocks per CU): half the
// K / V^T fragment reads per MFMA, best for long sequences.  QT = 1 (128 queries, 150 registers, three blocks per CU):
// twice the blocks, which wins when a call has too few of them to fill the chip twice (short sequences, text keys).
constexpr int ATT_BKV = 64;      // keys per step
constexpr int ATT_D = 64;        // head dim

// value of lane l^32 (v_permlane32_swap: upper half of the first operand <-> lower half of the second)
__device__ __forceinline__ float other_half(float v) {
    const uint32_t u = __float_as_uint(v);
    const auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
    // r[0]: lanes 0-31 own low value, lanes 32-63 the low half's value; r[1]: lanes 0-31 the high half's value
    return __uint_as_float((threadIdx.x & 32) ? r[0] : r[1]);
}
__device__ __forceinline__ float half_swap_max(float v) { return fmaxf(v, other_half(v)); }

typedef __attribute__((address_space(3))) void lds_void;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(2))) float f32x2;
constexpr int ATT_NS = 3;        // K / V^T ring depth in 64-key tiles
constexpr float ATT_SUM_MAX = 4096.f;   // a lane's 16-key partial row sum above this moves the softmax reference

// MFMA tile row r of a score tile holds key kperm(r) (bits 2 and 3 swapped): with this order the eight scores a lane
// owns for a 16-key MFMA step are eight CONSECUTIVE keys, so the matching V^T fragment is one 16-byte LDS read.
__device__ __forceinline__ int kperm(int r) { return (r & ~12) | ((r & 4) << 1) | ((r & 8) >> 1); }

// The vector ALU shares its issue slot with the matrix pipe, so the softmax is written for the fewest instructions
// per score: one exp2, half a bf16 pack and half a packed dot-product for the row sum.
//   * the scores come out of the MFMAs already shifted: the first MFMA of a 32-key half tile accumulates onto a
//     register tile holding -m_ref of the lane's query (no reset, no subtraction);
//   * no running maximum: the reference m_ref (log2 domain) is fixed by the first half tile and moves only when a
//     lane's partial row sum shows that a shifted score got large (rare; the exact maximum is then taken, the
//     accumulators are rescaled and the probabilities recomputed);
//   * the row sum is taken over the bf16-rounded probabilities, i.e. of exactly what multiplies V.
// K / V^T tiles of 64 keys are staged by direct global->LDS loads into a ring of three stages, two tiles ahead.
template <int ATT_QT>
__global__ void __launch_bounds__(256, ATT_QT == 1 ? 3 : 2)
attn_mfma_kernel(AttnArgs a) {
    constexpr int ATT_BQ = 4 * 32 * ATT_QT;
    extern __shared__ __attribute__((aligned(16))) uint8_t att_smem[];
    u32x4* sK = reinterpret_cast<u32x4*>(att_smem);            // [ATT_NS][64 keys][8 chunks], chunk ^ ((key>>1)&7)
    u32x4* sV = sK + ATT_NS * 512;                             // [ATT_NS][64 d][8 chunks of 8 keys], chunk ^ ((d>>1)&7)

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int fr = lane & 31, fh = lane >> 5;

    // ---- which (head, query tile) ----------------------------------------------------------------
    const int total_tiles = a.tile_off[a.n];
    const int64_t items = (int64_t)total_tiles * a.heads;
    const int64_t chunk = (items + 7) >> 3;
    const int64_t j = blockIdx.x >> 3;
    const int64_t k = (int64_t)(blockIdx.x & 7) * chunk + j;
    if (j >= chunk || k >= items) return;
    const int head = (int)(k / total_tiles);
    const int tile = total_tiles - 1 - (int)(k - (int64_t)head * total_tiles);
    int lo = 0, hi = a.n;                     // largest s with tile_off[s] <= tile
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (a.tile_off[mid] <= tile) lo = mid; else hi = mid;
    }
    const int s = lo;
    const int S = a.geom.S;
    const int rows_s = (a.act_off[s + 1] - a.act_off[s]) * S;            // computed query rows of this image
    const int r0 = (tile - a.tile_off[s]) * ATT_BQ;
    int64_t k0;
    int nk;
    if (a.cross_len) { k0 = (int64_t)a.perm[s] * a.cross_ld; nk = a.cross_len; }
    else { k0 = a.cu_seqlens[s]; nk = a.seq_len ? a.seq_len[s] : a.cu_seqlens[s + 1] - a.cu_seqlens[s]; }

    const uint16_t* Q = (const uint16_t*)a.Q;
    const uint16_t* K = (const uint16_t*)a.K;
    const uint16_t* V = (const uint16_t*)a.V;
    const int C = a.C;

    // ---- query fragments: lane holds Q[q][16*ks + 8*fh .. +8] of its query column, both query sub-tiles
    int64_t q_tok[ATT_QT];
    bool q_ok[ATT_QT];
    bf16x8 fq[ATT_QT][4];
#pragma unroll
    for (int qt = 0; qt < ATT_QT; ++qt) {
        int r = r0 + wave * (32 * ATT_QT) + qt * 32 + fr;
        q_ok[qt] = r < rows_s;
        if (!q_ok[qt]) r = rows_s - 1;
        const int pi = a.act_off[s] + r / S;
        const int p = a.act.active ? a.act.active[pi] : pi;
        q_tok[qt] = (int64_t)p * S + (r - (r / S) * S);
        const uint16_t* qp = Q + q_tok[qt] * C + head * ATT_D + fh * 8;
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) fq[qt][ks] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(qp + ks * 16));
    }

    // ---- staging by direct loads: a wavefront instruction fills 8 rows x 8 chunk positions; rows lr and lr + 32
    const int lc = lane & 7, lr = 8 * wave + (lane >> 3);
    const int gc = lc ^ ((lr >> 1) & 7);                     // global chunk fetched into position lc (same for both rows)
    const uint16_t* k_base = K + k0 * C + head * ATT_D + gc * 8;
    const uint16_t* v_base = V + (int64_t)(head * ATT_D + lr) * a.ldv + k0;
    const int64_t v_row32 = (int64_t)32 * a.ldv;
    const int steps = (nk + ATT_BKV - 1) / ATT_BKV;
    // A tile that lies inside the sequence is addressed as (uniform base of the tile) + (32-bit byte offset of the lane,
    // the same for every tile), so that its four loads cost no vector arithmetic (a 64-bit multiply per load before:
    // ~30 vector instructions per tile, two of them quarter-rate).  The launch checks that the offsets fit 32 bits.
    const uint8_t* k_uni = reinterpret_cast<const uint8_t*>(K + k0 * C + head * ATT_D);
    const uint8_t* v_uni = reinterpret_cast<const uint8_t*>(V + (int64_t)(head * ATT_D) * a.ldv + k0);
    uint32_t k_lane[2], v_lane[2];
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        k_lane[i] = (uint32_t)(((lr + 32 * i) * C + gc * 8) * 2);
        v_lane[i] = (uint32_t)(((int64_t)(lr + 32 * i) * a.ldv + gc * 8) * 2);
    }
    // keys / chunks past the image are clamped to valid ones: their scores are masked, their P is zero
#define PS_ISSUE_TILE(t_, st_)                                                                                   \
    {                                                                                                            \
        u32x4* dk_ = sK + (st_) * 512 + wave * 64;                                                               \
        u32x4* dv_ = sV + (st_) * 512 + wave * 64;                                                               \
        if ((t_) < steps - 1) {                                                                                  \
            const uint8_t* kt_ = k_uni + (int64_t)(t_) * (ATT_BKV * 2) * C;                                      \
            const uint8_t* vt_ = v_uni + (int64_t)(t_) * (ATT_BKV * 2);                                          \
            _Pragma("unroll") for (int i = 0; i < 2; ++i)                                                        \
                __builtin_amdgcn_global_load_lds((const void*)(kt_ + k_lane[i]), (lds_void*)(dk_ + i * 256), 16, 0, 0); \
            _Pragma("unroll") for (int i = 0; i < 2; ++i)                                                        \
                __builtin_amdgcn_global_load_lds((const void*)(vt_ + v_lane[i]), (lds_void*)(dv_ + i * 256), 16, 0, 0); \
        } else {                                                                                                 \
            const int kv_ = (steps - 1) * ATT_BKV;                                                               \
            _Pragma("unroll") for (int i = 0; i < 2; ++i) {                                                      \
                const int key_ = min(kv_ + lr + 32 * i, nk - 1);                                                 \
                __builtin_amdgcn_global_load_lds((const void*)(k_base + (int64_t)key_ * C), (lds_void*)(dk_ + i * 256), 16, 0, 0); \
            }                                                                                                    \
            const int vc_ = kv_ + gc * 8 < nk ? kv_ + gc * 8 : 0;                                                \
            _Pragma("unroll") for (int i = 0; i < 2; ++i)                                                        \
                __builtin_amdgcn_global_load_lds((const void*)(v_base + i * v_row32 + vc_), (lds_void*)(dv_ + i * 256), 16, 0, 0); \
        }                                                                                                        \
    }

    f32x16 acc_o[ATT_QT][2];
#pragma unroll
    for (int qt = 0; qt < ATT_QT; ++qt)
#pragma unroll
        for (int dt = 0; dt < 2; ++dt)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc_o[qt][dt][e] = 0.f;
    float m_ref[ATT_QT] = {}, l_run[ATT_QT] = {};   // reference maximum (log2 domain) and partial row sums
    f32x16 cinit[ATT_QT];                                       // -m_ref of the lane's query in every element
    f32x16 acc_s[ATT_QT];                                       // shifted scores of one 32-key half tile, per query sub-tile
    bf16x8 fp[ATT_QT][2];                                       // [query sub-tile][16-key step]: probabilities (B operand)
#pragma unroll
    for (int qt = 0; qt < ATT_QT; ++qt)
#pragma unroll
        for (int e = 0; e < 16; ++e) cinit[qt][e] = 0.f;

    // LDS rows of this lane's fragments
    const int krow[2] = {kperm(fr), kperm(fr) + 32};        // key row of MFMA tile row fr in half 0 / 1
    int ksw[2], vsw[2];
#pragma unroll
    for (int i = 0; i < 2; ++i) { ksw[i] = (krow[i] >> 1) & 7; vsw[i] = ((fr + 32 * i) >> 1) & 7; }

    PS_ISSUE_TILE(0, 0);
    PS_ISSUE_TILE(1, 1);

    // probabilities of query sub-tile QT from its shifted scores minus SH_: exp2, bf16 pack, row sum of the packed values
#define PS_PROBS(QT, SH_)                                                                                        \
    {                                                                                                            \
        sum_ = 0.f;                                                                                              \
        _Pragma("unroll") for (int k2 = 0; k2 < 2; ++k2) {                                                       \
            uint32_t pk_[4];                                                                                     \
            _Pragma("unroll") for (int i = 0; i < 4; ++i) {                                                      \
                const f32x2 pf_ = {__builtin_amdgcn_exp2f(acc_s[QT][8 * k2 + 2 * i] - (SH_)),                    \
                                   __builtin_amdgcn_exp2f(acc_s[QT][8 * k2 + 2 * i + 1] - (SH_))};               \
                const bf16x2 pb_ = __builtin_convertvector(pf_, bf16x2);                                         \
                sum_ = __builtin_amdgcn_fdot2_f32_bf16(pb_, bf16x2{(__bf16)1.f, (__bf16)1.f}, sum_, false);      \
                pk_[i] = __builtin_bit_cast(uint32_t, pb_);                                                      \
            }                                                                                                    \
            fp[QT][k2] = __builtin_bit_cast(bf16x8, u32x4{pk_[0], pk_[1], pk_[2], pk_[3]});                      \
        }                                                                                                        \
    }
    // one 32-key half tile (KT = 0 / 1 of the tile in stage ST): S^T = K Q^T - m_ref, P = 2^S, O^T += V^T P
#define PS_HALF(ST, KT, KV0, FIRST)                                                                              \
    {                                                                                                            \
        __builtin_amdgcn_sched_barrier(0);                                                                       \
        bf16x8 fk_[4], fv_[2][2];                                                                                \
        if ((KT) == 0) {                                                                                         \
            _Pragma("unroll") for (int ks = 0; ks < 4; ++ks)                                                     \
                fk_[ks] = __builtin_bit_cast(bf16x8, sK[(ST) * 512 + krow[0] * 8 + ((2 * ks + fh) ^ ksw[0])]);   \
        } else {                                /* read during the first half (behind its S MFMAs) */            \
            _Pragma("unroll") for (int ks = 0; ks < 4; ++ks) fk_[ks] = fkn_[ks];                                 \
        }                                                                                                        \
        /* first step: D = K Q^T + (-m_ref) written as the three-address instruction, so that the -m_ref tile is */    \
        /* read in place (the builtin form made the compiler copy it back and forth: 64 moves per key tile)      */    \
        _Pragma("unroll") for (int qt = 0; qt < ATT_QT; ++qt)                                                         \
            asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %3"                                               \
                         : "=&v"(acc_s[qt]) : "v"(fk_[0]), "v"(fq[qt][0]), "v"(cinit[qt]));                      \
        _Pragma("unroll") for (int ks = 1; ks < 4; ++ks)                                                         \
            _Pragma("unroll") for (int qt = 0; qt < ATT_QT; ++qt)                                                     \
                acc_s[qt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fk_[ks], fq[qt][ks], acc_s[qt], 0, 0, 0);    \
        __builtin_amdgcn_sched_barrier(0);                                                                       \
        _Pragma("unroll") for (int k2 = 0; k2 < 2; ++k2)                                                         \
            _Pragma("unroll") for (int dt = 0; dt < 2; ++dt)                                                     \
                fv_[k2][dt] = __builtin_bit_cast(bf16x8, sV[(ST) * 512 + (fr + 32 * dt) * 8 + ((4 * (KT) + 2 * k2 + fh) ^ vsw[dt])]); \
        if ((KT) == 0) {                        /* the key fragments of the second half: their LDS latency hides here */ \
            _Pragma("unroll") for (int ks = 0; ks < 4; ++ks)                                                     \
                fkn_[ks] = __builtin_bit_cast(bf16x8, sK[(ST) * 512 + krow[1] * 8 + ((2 * ks + fh) ^ ksw[1])]);  \
        }                                                                                                        \
        __builtin_amdgcn_sched_barrier(0);                                                                       \
        if ((KV0) + ATT_BKV > nk) {                                                                              \
            _Pragma("unroll") for (int e = 0; e < 16; ++e) {                                                     \
                const int key_ = (KV0) + 32 * (KT) + 16 * (e >> 3) + 8 * fh + (e & 7);                           \
                if (key_ >= nk) { _Pragma("unroll") for (int qt = 0; qt < ATT_QT; ++qt) acc_s[qt][e] = -INFINITY; }                            \
            }                                                                                                    \
        }                                                                                                        \
        _Pragma("unroll") for (int qt = 0; qt < ATT_QT; ++qt) {                                                       \
            float sum_;                                                                                          \
            PS_PROBS(qt, 0.f);                                                                                   \
            if ((FIRST) || __any(!(sum_ <= ATT_SUM_MAX))) {                                                      \
                float m_ = -INFINITY;                                                                            \
                _Pragma("unroll") for (int e = 0; e < 16; ++e) m_ = fmaxf(m_, acc_s[qt][e]);                     \
                m_ = half_swap_max(m_);                                                                          \
                const float d_ = ((FIRST) || m_ > 4.f) ? m_ : 0.f;                                               \
                const float corr_ = (FIRST) ? 1.f : __builtin_amdgcn_exp2f(-d_);                                 \
                m_ref[qt] += d_;                                                                                 \
                l_run[qt] *= corr_;                                                                              \
                _Pragma("unroll") for (int dt = 0; dt < 2; ++dt)                                                 \
                    _Pragma("unroll") for (int e = 0; e < 16; ++e) acc_o[qt][dt][e] *= corr_;                    \
                _Pragma("unroll") for (int e = 0; e < 16; ++e) cinit[qt][e] -= d_;    /* == -m_ref, in place */  \
                PS_PROBS(qt, d_);                                                                                \
            }                                                                                                    \
            l_run[qt] += sum_;                                                                                   \
            _Pragma("unroll") for (int k2 = 0; k2 < 2; ++k2)                                                     \
                _Pragma("unroll") for (int dt = 0; dt < 2; ++dt)                                                 \
                    acc_o[qt][dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fv_[k2][dt], fp[qt][k2], acc_o[qt][dt], 0, 0, 0); \
        }                                                                                                        \
    }

    bf16x8 fkn_[4];                                             // key fragments of the second half tile, read ahead
    int st = 0;
    for (int t = 0; t < steps; ++t) {
        // own loads of tile t have landed (tile t+1 may be in flight); then tile t is visible to all and the stage of
        // tile t-1 is free.  A bare s_barrier: __syncthreads() carries a fence that waits for ALL loads in flight.
        asm volatile("s_waitcnt lgkmcnt(0)\n\ts_waitcnt vmcnt(4)\n\ts_barrier" ::: "memory");
        const int st2 = st == 0 ? ATT_NS - 1 : st - 1;          // stage of tile t-1 == stage of tile t+2
        PS_ISSUE_TILE(t + 2, st2);
        const int kv0 = t * ATT_BKV;
        const bool first = t == 0;
        PS_HALF(st, 0, kv0, first);
        PS_HALF(st, 1, kv0, false);
        st = st + 1 == ATT_NS ? 0 : st + 1;
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");        // no load may still target LDS when the block retires
#undef PS_HALF
#undef PS_PROBS
#undef PS_ISSUE_TILE

    // ---- O[q][head*64 + d] = O^T / l ; lane holds d = 32*dt + 8*(e/4) + 4*fh + e%4 of query fr
    uint16_t* O = (uint16_t*)a.O;
#pragma unroll
    for (int qt = 0; qt < ATT_QT; ++qt) {
        const float l = l_run[qt] + other_half(l_run[qt]);
        const float inv = 1.f / l;
        if (!q_ok[qt]) continue;
        // A lane holds four consecutive d (8 bytes) of its query per (dt, eg), lane ^ 32 the next four.  The two halves
        // trade them so that the lower half owns the even eg chunks and the upper half the odd ones: 16-byte stores,
        // two adjacent chunks of a row per instruction (half the stores of the 8-byte form).
        uint16_t* op = O + q_tok[qt] * C + head * ATT_D + 8 * fh;
#pragma unroll
        for (int dt = 0; dt < 2; ++dt)
#pragma unroll
            for (int eg = 0; eg < 4; eg += 2) {
                uint32_t w[2][2];               // [eg parity][dword]
#pragma unroll
                for (int q = 0; q < 2; ++q) {
                    w[q][0] = pack_bf16x2(acc_o[qt][dt][4 * (eg + q)] * inv, acc_o[qt][dt][4 * (eg + q) + 1] * inv);
                    w[q][1] = pack_bf16x2(acc_o[qt][dt][4 * (eg + q) + 2] * inv, acc_o[qt][dt][4 * (eg + q) + 3] * inv);
                }
                // swap(x = even chunk, y = odd chunk): r[0] = {lower: own even, upper: the lower half's odd},
                // r[1] = {lower: the upper half's even, upper: own odd}
                const auto r0 = __builtin_amdgcn_permlane32_swap(w[0][0], w[1][0], false, false);
                const auto r1 = __builtin_amdgcn_permlane32_swap(w[0][1], w[1][1], false, false);
                *reinterpret_cast<u32x4*>(op + dt * 32 + eg * 8) = u32x4{r0[0], r1[0], r0[1], r1[1]};
            }
    }
}

// One block: per request slot, number of computed patches and of query tiles (exclusive prefixes).
__global__ void attn_tiles_kernel(const int32_t* __restrict__ request_offset, const uint8_t* __restrict__ mask, int32_t n,
                                  int32_t S, int32_t ATT_BQ, int32_t* __restrict__ act_off, int32_t* __restrict__ tile_off) {
    __shared__ int32_t s_cnt[1024], s_til[1024];
    __shared__ int32_t c_cnt, c_til;
    const int tid = threadIdx.x;
    if (tid == 0) { c_cnt = 0; c_til = 0; act_off[0] = 0; tile_off[0] = 0; }
    __syncthreads();
    for (int base = 0; base < n; base += 1024) {
        const int s = base + tid;
        int cnt = 0, til = 0;
        if (s < n) {
            const int p0 = request_offset[s], p1 = request_offset[s + 1];
            if (mask) { for (int p = p0; p < p1; ++p) cnt += mask[p] == 0; }
            else cnt = p1 - p0;
            til = (cnt * S + ATT_BQ - 1) / ATT_BQ;
        }
        s_cnt[tid] = cnt;
        s_til[tid] = til;
        __syncthreads();
        for (int off = 1; off < 1024; off <<= 1) {
            int x = 0, y = 0;
            if (tid >= off) { x = s_cnt[tid - off]; y = s_til[tid - off]; }
            __syncthreads();
            s_cnt[tid] += x;
            s_til[tid] += y;
            __syncthreads();
        }
        if (s < n) { act_off[s + 1] = c_cnt + s_cnt[tid]; tile_off[s + 1] = c_til + s_til[tid]; }
        __syncthreads();
        if (tid == 1023) { c_cnt += s_cnt[tid]; c_til += s_til[tid]; }
        __syncthreads();
    }
}

int attention_tiles(const int32_t* request_offset, const uint8_t* mask, int32_t n, int32_t S, int32_t qt, int32_t* act_off,
                    int32_t* tile_off, hipStream_t st) {
    attn_tiles_kernel<<<1, 1024, 0, st>>>(request_offset, mask, n, S, 128 * qt, act_off, tile_off);
    return check_launch("attn_tiles_kernel");
}

int attention_max_tiles(const pserve_plan_t* plan, int32_t qt) {
    int64_t t = 0;
    const auto& ro = plan->h_tab[PSERVE_TAB_REQUEST_OFFSET];
    for (int s = 0; s < plan->n; ++s) t += cdiv((int64_t)(ro[s + 1] - ro[s]) * plan->S, 128 * qt);
    return (int)t;
}

int attention_mfma_bf16(const AttnArgs& a, hipStream_t st, bool* handled) {
    *handled = false;
    if (a.d != ATT_D || !a.v_transposed || !a.tile_off || !a.act_off || (a.qt != 1 && a.qt != 2)) return PSERVE_OK;
    if (a.C % 8 != 0 || a.ldv % 8 != 0) return PSERVE_OK;
    if ((int64_t)64 * a.ldv * 2 + 128 >= ((int64_t)1 << 32) || (int64_t)64 * a.C * 2 + 128 >= ((int64_t)1 << 32)) return PSERVE_OK;
    if (a.cross_len) {
        if (a.cross_ld % 8 != 0) return PSERVE_OK;
    } else if (a.geom.S % 8 != 0) {
        return PSERVE_OK;              // image token ranges must start on 16-byte boundaries of the V^T rows
    }
    *handled = true;
    const int64_t items = (int64_t)a.max_tiles * a.heads;
    const unsigned grid = (unsigned)(8 * cdiv(items, 8));
    constexpr int lds = ATT_NS * 2 * 512 * 16;
    static bool attr_set = false;
    if (!attr_set) {
        PS_CHECK_HIP(hipFuncSetAttribute((const void*)attn_mfma_kernel<1>, hipFuncAttributeMaxDynamicSharedMemorySize, lds));
        PS_CHECK_HIP(hipFuncSetAttribute((const void*)attn_mfma_kernel<2>, hipFuncAttributeMaxDynamicSharedMemorySize, lds));
        attr_set = true;
    }
    if (a.qt == 1) attn_mfma_kernel<1><<<grid, 256, lds, st>>>(a);
    else attn_mfma_kernel<2><<<grid, 256, lds, st>>>(a);
    return check_launch("attn_mfma_kernel");
}

}  // namespace pserve
