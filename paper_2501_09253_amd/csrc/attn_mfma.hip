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
// through that XCD's L2.  The largest images come first (attn_item).
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
extern __shared__ __attribute__((aligned(16))) uint8_t att_smem[];

// Work item of a block: (request slot, head, query tile of that request).  A block's run time goes with the number of
// keys of its request, so the items are ordered longest first: request slots from the last (the plan sorts requests by
// size, largest last) to the first, head-major inside a slot, so that consecutive items are consecutive query tiles of
// one head.  Groups of ATT_GROUP consecutive items are dealt to the XCDs in turn (block b runs on XCD b mod 8 and an XCD
// starts its blocks in order): the blocks resident on an XCD stream the K / V^T tiles of the same head through that
// XCD's L2, every XCD gets the same share of the long items, and the short ones fill the last round.
constexpr int ATT_GROUP = 64;
__device__ __forceinline__ bool attn_item(const AttnArgs& a, int& s, int& head, int& tile_in_s) {
    const int total_tiles = a.tile_off[a.n];
    const int64_t items = (int64_t)total_tiles * a.heads;
    const int64_t seq = blockIdx.x >> 3;
    const int64_t k = ((seq / ATT_GROUP) * 8 + (blockIdx.x & 7)) * ATT_GROUP + seq % ATT_GROUP;
    if (k >= items) return false;
    const int64_t q = items - 1 - k;                 // position in ascending slot order
    const int qt = (int)(q / a.heads);
    int lo = 0, hi = a.n;                            // largest s with tile_off[s] <= qt
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (a.tile_off[mid] <= qt) lo = mid; else hi = mid;
    }
    s = lo;
    const int tiles_s = a.tile_off[s + 1] - a.tile_off[s];
    const int r = tiles_s * a.heads - 1 - (int)(q - (int64_t)a.tile_off[s] * a.heads);
    head = r / tiles_s;
    tile_in_s = r - head * tiles_s;
    return true;
}

template <int ATT_QT>
__device__ __forceinline__ void attn_body(const AttnArgs& a, const int tid) {
    constexpr int ATT_BQ = 4 * 32 * ATT_QT;
    u32x4* sK = reinterpret_cast<u32x4*>(att_smem);            // [ATT_NS][64 keys][8 chunks], chunk ^ ((key>>1)&7)
    u32x4* sV = sK + ATT_NS * 512;                             // [ATT_NS][64 d][8 chunks of 8 keys], chunk ^ ((d>>1)&7)

    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int fr = lane & 31, fh = lane >> 5;

    // ---- which (request slot, head, query tile) ---------------------------------------------------
    int s, head, tile_in_s;
    if (!attn_item(a, s, head, tile_in_s)) return;
    const int S = a.geom.S;
    const int rows_s = (a.act_off[s + 1] - a.act_off[s]) * S;            // computed query rows of this image
    const int r0 = tile_in_s * ATT_BQ;
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

template <int ATT_QT>
__global__ void __launch_bounds__(256, ATT_QT == 1 ? 3 : 2)
attn_mfma_kernel(AttnArgs a) {
    attn_body<ATT_QT>(a, threadIdx.x);
}

// ---- the software-pipelined form (256 queries per block) ------------------------------------------------------
// What the chip does with ONE wavefront's instruction stream (probe kernels: a stream of v_mfma_f32_32x32x16_bf16 with
// K vector instructions between consecutive MFMAs): the MFMA occupies the matrix pipe for 32 clocks, and up to four
// full-rate vector instructions or two v_exp_f32 issue behind it for free (more cost 4.2 resp. 7.3 clocks each); a
// second wavefront on the SIMD adds no issue slots, it only fills stalls; v_dot2c_f32_bf16 next to an MFMA costs about
// 20 clocks.  So the softmax has to ride behind the MFMAs of the SAME wavefront.  The work of a wavefront is cut into
// units of (32 keys, 32 queries), and in every step the 4 score MFMAs of the NEXT unit and the 4 output MFMAs of the
// PREVIOUS unit are issued alternately, with the 16 exponentials and 8 packs of the CURRENT unit spread over the eight
// MFMA slots (the three are independent of each other); the row sums are two running fp32 additions per pair of exponentials.  The two query sub-tiles of a wavefront
// alternate as units, so their score tiles and probability fragments are the double buffers.  Key fragments of the next
// half tile and value fragments of the current one are refilled from LDS right behind the MFMA that last read the
// register, eight MFMA slots before they are needed.  Because the scores of a tile's first unit are formed during the
// previous tile, the key ring runs one tile ahead of the value ring: both have four stages of 64 keys (64 KB per block,
// two blocks per CU), filled two tiles ahead by direct global->LDS loads, one barrier per tile.
//
// No softmax reference: P = 2^score as it is (the scores arrive pre-scaled by log2 e / sqrt d).  bf16 and fp32 share
// the exponent range, and O / l does not depend on a common factor, so this is exact as long as nothing overflows or
// underflows: the largest score of every query row within +-100 (logits of +-69 before the log2 e factor).  A block
// that sees a row sum outside [2^-100, 2^100] (or not a number) at the end runs again through attn_body<2>, which
// tracks a reference and takes any range.
constexpr int ATT_PNS = 4;       // ring depth of the pipelined kernel
constexpr float ATT_L_MAX = 1.2676506e30f, ATT_L_MIN = 7.8886091e-31f;      // 2^100, 2^-100

__global__ void __launch_bounds__(256, 2)
attn_pipe_kernel(AttnArgs a) {
    constexpr int ATT_BQ = 256;
    // sK: [ATT_PNS][64 keys][8 chunks of 8 d], chunk ^ ((key>>1)&7); sV behind it: [ATT_PNS][64 d][8 chunks of 8 keys],
    // chunk ^ ((d>>1)&7).  A stage is 8 KB.
    constexpr uint32_t STAGE = 8192, SV_OFF = ATT_PNS * STAGE;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int fr = lane & 31, fh = lane >> 5;

    // ---- which (request slot, head, query tile) ---------------------------------------------------
    int s, head, tile_in_s;
    if (!attn_item(a, s, head, tile_in_s)) return;
    const int S = a.geom.S;
    const int rows_s = (a.act_off[s + 1] - a.act_off[s]) * S;            // computed query rows of this image
    const int r0 = tile_in_s * ATT_BQ;
    int64_t k0;
    int nk;
    if (a.cross_len) { k0 = (int64_t)a.perm[s] * a.cross_ld; nk = a.cross_len; }
    else { k0 = a.cu_seqlens[s]; nk = a.seq_len ? a.seq_len[s] : a.cu_seqlens[s + 1] - a.cu_seqlens[s]; }

    const uint16_t* Q = (const uint16_t*)a.Q;
    const uint16_t* K = (const uint16_t*)a.K;
    const uint16_t* V = (const uint16_t*)a.V;
    const int C = a.C;

    // token of query row (sub-tile qt, lane's column); rows past the image's computed rows repeat its last row
#define PS_QTOK(qt_, tok_, ok_)                                                                                  \
    {                                                                                                            \
        int r_ = r0 + wave * 64 + (qt_) * 32 + fr;                                                               \
        ok_ = r_ < rows_s;                                                                                       \
        if (!ok_) r_ = rows_s - 1;                                                                               \
        const int pi_ = a.act_off[s] + r_ / S;                                                                   \
        const int p_ = a.act.active ? a.act.active[pi_] : pi_;                                                   \
        tok_ = (int64_t)p_ * S + (r_ - (r_ / S) * S);                                                            \
    }
    // ---- query fragments: lane holds Q[q][16*ks + 8*fh .. +8] of its query column, both query sub-tiles
    bf16x8 fq[2][4];
#pragma unroll
    for (int qt = 0; qt < 2; ++qt) {
        int64_t tok;
        bool ok;
        PS_QTOK(qt, tok, ok);
        const uint16_t* qp = Q + tok * C + head * ATT_D + fh * 8;
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) fq[qt][ks] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(qp + ks * 16));
    }

    // ---- staging by direct loads: a wavefront instruction fills 8 rows x 8 chunk positions; rows lr and lr + 32
    const int lc = lane & 7, lr = 8 * wave + (lane >> 3);
    const int gc = lc ^ ((lr >> 1) & 7);                     // global chunk fetched into position lc (same for both rows)
    const int steps = (nk + ATT_BKV - 1) / ATT_BKV;
    const uint8_t* k_uni = reinterpret_cast<const uint8_t*>(K + k0 * C + head * ATT_D);
    const uint8_t* v_uni = reinterpret_cast<const uint8_t*>(V + (int64_t)(head * ATT_D) * a.ldv + k0);
    uint32_t k_lane[2], v_lane[2];
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        k_lane[i] = (uint32_t)(((lr + 32 * i) * C + gc * 8) * 2);
        v_lane[i] = (uint32_t)(((int64_t)(lr + 32 * i) * a.ldv + gc * 8) * 2);
    }
    typedef __attribute__((address_space(3))) uint8_t lds_u8;
    // Two load instructions per tile and operand.  Tiles past the sequence re-load the last tile (into a stage nobody
    // reads), so that every wavefront always has the same number of loads in flight; inside the last tile, keys /
    // chunks past the image are clamped to valid ones: their scores are masked, their P is zero.  The clamped
    // addresses are formed from the tile index on the spot (rare path; nothing of it is kept in registers).
#define PS_ISSUE_K(t_)                                                                                           \
    {                                                                                                            \
        const int tt_ = min((t_), steps - 1);                                                                    \
        lds_u8* dk_ = (lds_u8*)(att_smem + ((t_) & (ATT_PNS - 1)) * STAGE + wave * 1024);                        \
        const uint8_t* kt_ = k_uni + (int64_t)tt_ * (ATT_BKV * 2) * C;                                           \
        if ((tt_ + 1) * ATT_BKV <= nk) {                                                                         \
            _Pragma("unroll") for (int i = 0; i < 2; ++i) {                                                      \
                uint32_t off_ = k_lane[i];                                                                       \
                asm volatile("" : "+v"(off_));                  /* stays a 32-bit offset beside the uniform base */ \
                __builtin_amdgcn_global_load_lds((const void*)(kt_ + off_), (lds_void*)(dk_ + i * 4096), 16, 0, 0); \
            }                                                                                                    \
        } else {                                                                                                 \
            int ln_ = lane;                                                                                      \
            asm volatile("" : "+v"(ln_));                       /* formed here, not ahead of the loop */         \
            const int lr_ = 8 * wave + (ln_ >> 3), gc_ = (ln_ & 7) ^ ((lr_ >> 1) & 7);                           \
            _Pragma("unroll") for (int i = 0; i < 2; ++i) {                                                      \
                const int row_ = min(lr_ + 32 * i, nk - 1 - tt_ * ATT_BKV);                                      \
                __builtin_amdgcn_global_load_lds((const void*)(kt_ + (uint32_t)((row_ * C + gc_ * 8) * 2)), (lds_void*)(dk_ + i * 4096), 16, 0, 0); \
            }                                                                                                    \
        }                                                                                                        \
    }
#define PS_ISSUE_V(t_)                                                                                           \
    {                                                                                                            \
        const int tt_ = min((t_), steps - 1);                                                                    \
        lds_u8* dv_ = (lds_u8*)(att_smem + SV_OFF + ((t_) & (ATT_PNS - 1)) * STAGE + wave * 1024);               \
        const uint8_t* vt_ = v_uni + (int64_t)tt_ * (ATT_BKV * 2);                                               \
        if ((tt_ + 1) * ATT_BKV <= nk) {                                                                         \
            _Pragma("unroll") for (int i = 0; i < 2; ++i) {                                                      \
                uint32_t off_ = v_lane[i];                                                                       \
                asm volatile("" : "+v"(off_));                                                                   \
                __builtin_amdgcn_global_load_lds((const void*)(vt_ + off_), (lds_void*)(dv_ + i * 4096), 16, 0, 0); \
            }                                                                                                    \
        } else {                                                                                                 \
            int ln_ = lane;                                                                                      \
            asm volatile("" : "+v"(ln_));                                                                        \
            const int lr_ = 8 * wave + (ln_ >> 3), gc_ = (ln_ & 7) ^ ((lr_ >> 1) & 7);                           \
            const int col_ = tt_ * ATT_BKV + gc_ * 8 < nk ? gc_ * 8 : -tt_ * ATT_BKV;                            \
            _Pragma("unroll") for (int i = 0; i < 2; ++i)                                                        \
                __builtin_amdgcn_global_load_lds((const void*)(vt_ + ((int64_t)(lr_ + 32 * i) * a.ldv + col_) * 2), (lds_void*)(dv_ + i * 4096), 16, 0, 0); \
        }                                                                                                        \
    }

    f32x16 acc_o[2][2];
    f32x16 acc_s[2];                                            // scores of the unit in flight, per query sub-tile
    u32x4 fp[2][2];                                             // [query sub-tile][16-key step]: probabilities (B operand), packed bf16
    bf16x8 fk[4], fv[4];                                        // key fragments [ks], value fragments [2*k2 + dt]
    const f32x16 zero16 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int qt = 0; qt < 2; ++qt) {
        acc_o[qt][0] = zero16;
        acc_o[qt][1] = zero16;
#pragma unroll
        for (int k2 = 0; k2 < 2; ++k2) fp[qt][k2] = u32x4{0u, 0u, 0u, 0u};
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) fv[i] = __builtin_bit_cast(bf16x8, u32x4{0u, 0u, 0u, 0u});   // the first step's output MFMAs add 0 * 0
    // Row sums on the vector unit: every exponential is added to one of two running sums per query sub-tile (fp32, before
    // the rounding to bf16; the rounding errors of the probabilities that multiply V are unbiased).  Four
    // v_mfma_f32_4x4x4_16b_bf16 per unit with an all-ones operand did the same on the matrix pipe; a register-resident
    // stream with this loop's instruction mix is 5 % faster with the additions (the small MFMAs hold the pipe for two
    // passes each), the kernel 2.7 %.
    float lsum[2][2] = {{0.f, 0.f}, {0.f, 0.f}};

    // LDS byte addresses of this lane's fragments in stage 0.  Key fragment ks of half H: row kperm(fr) + 32 H (half 1 is
    // 4 KB further), chunk (2 ks + fh) ^ swizzle.  Value fragment (H, k2, dt): row fr + 32 dt (dt = 1 is 4 KB further),
    // chunk (4 H + 2 k2 + fh) ^ swizzle.  The registers follow the ring: they advance by one stage per tile.
    uint32_t ka[4], va[4];
    {
        const int krow = kperm(fr), ksw = (krow >> 1) & 7, vsw = (fr >> 1) & 7;
        const uint32_t smem_base = (uint32_t)(uintptr_t)(lds_u8*)att_smem;
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) ka[ks] = smem_base + (uint32_t)(krow * 128 + 16 * ((2 * ks + fh) ^ ksw));
#pragma unroll
        for (int i = 0; i < 4; ++i) va[i] = smem_base + SV_OFF + (uint32_t)(fr * 128 + 16 * ((2 * i + fh) ^ vsw));
    }
    // the fragment addresses are absolute LDS addresses (no base to add per read)
    typedef const __attribute__((address_space(3))) u32x4* lds_frag;
#define PS_LDS(addr_) __builtin_bit_cast(bf16x8, *(lds_frag)(uintptr_t)(addr_))

    // One MFMA slot's share of the softmax of the unit whose scores are acc_s[QT]: the two exponentials of pair G, and
    // the bf16 pack and the two row-sum additions of pair G-1 (one slot later, so that nothing waits for an
    // exponential).  Pack and additions are one block of assembly: as separate instructions the compiler's scheduler no
    // longer keeps the slot order (with 16 more vector instructions per step it falls back into clumps of
    // exponentials), and a block that nothing ties down sinks to the end of the step.  Two operands that pass through
    // the block untouched tie it down: PIN, an accumulator element that this slot's MFMA has just written (the block
    // follows that MFMA), and the first score of pair G (the block precedes that pair's exponentials).  The pack comes
    // LAST in the block: its result may be given the register of one of the block's inputs (an output that is not
    // marked early-clobber), and the additions read those inputs.  The s_nop is the wait state a vector instruction
    // needs behind the transcendental whose result it reads, should the two ever end up next to each other; nothing
    // else in the block can meet a hazard the compiler does not see: it writes only its own results (never a register
    // an MFMA in flight reads as its addend or writes) and reads only exponentials of an earlier slot.
#define PS_SOFT(QT, G, PIN)                                                                                      \
    {                                                                                                            \
        if ((G) > 0) {                                                                                           \
            uint32_t pk_;                                                                                        \
            asm("s_nop 0\n\tv_add_f32 %[l0], %[l0], %[e0]\n\tv_add_f32 %[l1], %[l1], %[e1]\n\tv_cvt_pk_bf16_f32 %[pk], %[e0], %[e1]" \
                : [pk] "=v"(pk_), [l0] "+v"(lsum[QT][0]), [l1] "+v"(lsum[QT][1]), "+v"(acc_s[QT][(G) < 8 ? 2 * (G) : 0]), "+v"(PIN) \
                : [e0] "v"(e0_), [e1] "v"(e1_));                                                                 \
            fp[QT][((G) - 1) >> 2][((G) - 1) & 3] = pk_;                                                         \
        }                                                                                                        \
        if ((G) < 8) {                                                                                           \
            e0_ = __builtin_amdgcn_exp2f(acc_s[QT][2 * (G)]);                                                    \
            e1_ = __builtin_amdgcn_exp2f(acc_s[QT][2 * (G) + 1]);                                                \
        }                                                                                                        \
    }
#define PS_MFMA_O(QT, J) acc_o[QT][(J) & 1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fv[J], __builtin_bit_cast(bf16x8, fp[QT][(J) >> 1]), acc_o[QT][(J) & 1], 0, 0, 0)
#define PS_MFMA_S(QT, J) acc_s[QT] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fk[J], fq[QT][J], (J) == 0 ? zero16 : acc_s[QT], 0, 0, 0)
    // keys past the end of the sequence (last tile only): their scores become -inf
#define PS_MASK(QT, KEY0)                                                                                        \
    if ((KEY0) + 32 > nk) {                                                                                      \
        int ln_ = lane;                                                                                          \
        asm volatile("" : "+v"(ln_));                           /* formed here, not ahead of the loop */         \
        _Pragma("unroll") for (int e = 0; e < 16; ++e) {                                                         \
            const int key_ = (KEY0) + 16 * (e >> 3) + 8 * (ln_ >> 5) + (e & 7);                                  \
            if (key_ >= nk) acc_s[QT][e] = -INFINITY;                                                            \
        }                                                                                                        \
    }
#define PS_FENCE __builtin_amdgcn_sched_barrier(0)
    // Step of unit (half H, sub-tile 0) of a tile (PS_STEP0): the score MFMAs of (H, sub-tile 1) alternate with the output
    // MFMAs of the previous unit (sub-tile 1 of the previous half, whose value fragments are still in fv); behind its last
    // reader each key fragment is refilled for the next half (KOFF: 4096 = second half of the stage ka points at, 0 =
    // first half of the next stage, to which ka has then advanced) and each value fragment for half H.  Step of unit
    // (H, sub-tile 1) (PS_STEP1): the score MFMAs of (next half, sub-tile 0) alternate with the output MFMAs of
    // (H, sub-tile 0); no fragment is refilled (both sets are read again by the next step).
    // A step is one basic block, and the order inside it is prescribed slot by slot (sched_group_barrier: 0x8 matrix,
    // 0x400 transcendental, 0x2 other vector, 0x100 LDS read).  Left to itself the compiler gathers the 16 exponentials
    // of a step in front of its MFMAs: fences between the slots do not hold instructions without side effects in place.
#define PS_SGB(mask_, n_) __builtin_amdgcn_sched_group_barrier((mask_), (n_), 0)
#define PS_LOADS_K(t_)                                                                                           \
    {                                                                                                            \
        lds_u8* dk_ = (lds_u8*)(att_smem + ((t_) & (ATT_PNS - 1)) * STAGE + wave * 1024);                        \
        const uint8_t* kt_ = k_uni + (int64_t)min((t_), steps - 1) * (ATT_BKV * 2) * C;                          \
        _Pragma("unroll") for (int i = 0; i < 2; ++i) {                                                          \
            uint32_t off_ = k_lane[i];                                                                           \
            asm volatile("" : "+v"(off_));                                                                       \
            __builtin_amdgcn_global_load_lds((const void*)(kt_ + off_), (lds_void*)(dk_ + i * 4096), 16, 0, 0);  \
        }                                                                                                        \
    }
#define PS_LOADS_V(t_)                                                                                           \
    {                                                                                                            \
        lds_u8* dv_ = (lds_u8*)(att_smem + SV_OFF + ((t_) & (ATT_PNS - 1)) * STAGE + wave * 1024);               \
        const uint8_t* vt_ = v_uni + (int64_t)min((t_), steps - 1) * (ATT_BKV * 2);                              \
        _Pragma("unroll") for (int i = 0; i < 2; ++i) {                                                          \
            uint32_t off_ = v_lane[i];                                                                           \
            asm volatile("" : "+v"(off_));                                                                       \
            __builtin_amdgcn_global_load_lds((const void*)(vt_ + off_), (lds_void*)(dv_ + i * 4096), 16, 0, 0);  \
        }                                                                                                        \
    }
#define PS_STEP0(H, KOFF, LEAD)                                                                                  \
    {                                                                                                            \
        float e0_, e1_;                                                                                          \
        LEAD;                                                                                                    \
        _Pragma("unroll") for (int j_ = 0; j_ < 4; ++j_) {                                                       \
            PS_MFMA_S(1, j_);                                                                                    \
            PS_SOFT(0, 2 * j_, acc_s[1][0])                                                                                   \
            fk[j_] = PS_LDS(ka[j_] + (KOFF));                                                                    \
            PS_MFMA_O(1, j_);                                                                                    \
            PS_SOFT(0, 2 * j_ + 1, acc_o[1][j_ & 1][0])                                                                               \
            fv[j_] = PS_LDS(va[2 * (H) + (j_ >> 1)] + (j_ & 1) * 4096);                                          \
        }                                                                                                        \
        PS_SOFT(0, 8, acc_o[1][1][1])                                                                                            \
        _Pragma("unroll") for (int j_ = 0; j_ < 4; ++j_) {                                                       \
            PS_SGB(0x008, 1);                                                                                    \
            PS_SGB(0x100, 1);                                                                                    \
            PS_SGB(0x400, 2);                                                                                    \
            PS_SGB(0x008, 1);                                                                                    \
            PS_SGB(0x100, 1);                                                                                    \
            PS_SGB(0x400, 2);                                                                                    \
        }                                                                                                        \
        PS_FENCE;                                                                                                \
    }
#define PS_STEP1(LEAD)                                                                                           \
    {                                                                                                            \
        float e0_, e1_;                                                                                          \
        LEAD;                                                                                                    \
        _Pragma("unroll") for (int j_ = 0; j_ < 4; ++j_) {                                                       \
            PS_MFMA_S(0, j_);                                                                                    \
            PS_SOFT(1, 2 * j_, acc_s[0][0])                                                                                   \
            PS_MFMA_O(0, j_);                                                                                    \
            PS_SOFT(1, 2 * j_ + 1, acc_o[0][j_ & 1][0])                                                                               \
        }                                                                                                        \
        PS_SOFT(1, 8, acc_o[0][1][1])                                                                                            \
        _Pragma("unroll") for (int j_ = 0; j_ < 4; ++j_) {                                                       \
            PS_SGB(0x008, 1);                                                                                    \
            PS_SGB(0x400, 2);                                                                                    \
            PS_SGB(0x008, 1);                                                                                    \
            PS_SGB(0x400, 2);                                                                                    \
        }                                                                                                        \
        PS_FENCE;                                                                                                \
    }

    // ---- prologue: K tiles 0..2 and V tiles 0..1 in flight (three groups, oldest first), scores of the first unit
    PS_ISSUE_K(0);
    PS_ISSUE_K(1);
    PS_ISSUE_V(0);
    PS_ISSUE_K(2);
    PS_ISSUE_V(1);
    asm volatile("s_waitcnt vmcnt(8)\n\ts_barrier" ::: "memory");          // K tile 0 has landed everywhere
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) fk[ks] = PS_LDS(ka[ks]);
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) PS_MFMA_S(0, ks);

    // K tile t+1 and V tile t have landed at the barrier of iteration t (the loads of the previous iteration may be in
    // flight) and every wavefront has left iteration t-1: the stages of K tile t-1 and V tile t-2 are free.  The loads
    // of an iteration are issued behind MFMAs of its first two steps, not in front of them: right after the barrier all
    // wavefronts of the block would queue at the memory pipeline at once, each with idle matrix pipe behind it.
    int t = 0;
    // Interior iterations: tile t whole (nothing to mask) and the tiles loaded (t + 2, t + 3, or the last tile again
    // once past the end) whole (nothing to clamp): every iteration of a sequence that is a multiple of the tile.
    const int interior = (nk & (ATT_BKV - 1)) == 0 ? steps : steps - 4;
    for (; t < interior; ++t) {
        asm volatile("s_waitcnt vmcnt(4)\n\ts_barrier" ::: "memory");
        const uint32_t adv = ((t & (ATT_PNS - 1)) == ATT_PNS - 1) ? (uint32_t)(-(int)((ATT_PNS - 1) * STAGE)) : STAGE;
        PS_STEP0(0, 4096, PS_FENCE);
        PS_LOADS_K(t + 3);
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) ka[ks] += adv;           // the key fragments now come from the next tile's stage
        PS_STEP1(PS_FENCE);
        PS_LOADS_V(t + 2);
        PS_STEP0(1, 0, PS_FENCE);
        PS_STEP1(PS_FENCE);
#pragma unroll
        for (int i = 0; i < 4; ++i) va[i] += adv;
    }
    for (; t < steps; ++t) {
        asm volatile("s_waitcnt vmcnt(4)\n\ts_barrier" ::: "memory");
        const int kv0 = t * ATT_BKV;
        const uint32_t adv = ((t & (ATT_PNS - 1)) == ATT_PNS - 1) ? (uint32_t)(-(int)((ATT_PNS - 1) * STAGE)) : STAGE;
        PS_MASK(0, kv0)
        PS_STEP0(0, 4096, );
        PS_ISSUE_K(t + 3);
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) ka[ks] += adv;
        PS_MASK(1, kv0)
        PS_STEP1();
        PS_ISSUE_V(t + 2);
        PS_MASK(0, kv0 + 32)
        PS_STEP0(1, 0, );
        PS_MASK(1, kv0 + 32)
        PS_STEP1();
#pragma unroll
        for (int i = 0; i < 4; ++i) va[i] += adv;
    }
    // ---- epilogue: output MFMAs of the last unit
#pragma unroll
    for (int j_ = 0; j_ < 4; ++j_) {
        PS_MFMA_O(1, j_);
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");        // no load may still target LDS when the block moves on
#undef PS_STEP0
#undef PS_STEP1
#undef PS_LOADS_K
#undef PS_LOADS_V
#undef PS_SGB
#undef PS_FENCE
#undef PS_MASK
#undef PS_MFMA_S
#undef PS_MFMA_O
#undef PS_SOFT
#undef PS_LDS
#undef PS_ISSUE_K
#undef PS_ISSUE_V

    // ---- row sums; a row sum out of range (or not a number) anywhere in the block: the whole block again, with a
    // softmax reference (the vote goes through LDS, which nobody reads any more after the barrier)
    float inv[2];
    bool fine = true;
#pragma unroll
    for (int qt = 0; qt < 2; ++qt) {
        const float lown = lsum[qt][0] + lsum[qt][1];
        const float l = lown + other_half(lown);
        fine = fine && l >= ATT_L_MIN && l <= ATT_L_MAX;
        inv[qt] = 1.f / l;
    }
    __syncthreads();
    int32_t* vote = reinterpret_cast<int32_t*>(att_smem);
    if (tid < 4) vote[tid] = 0;
    __syncthreads();
    if (lane == 0 && __any(!fine)) vote[wave] = 1;
    __syncthreads();
    const bool redo = (vote[0] | vote[1] | vote[2] | vote[3]) != 0;
    __syncthreads();
    if (redo) {
        // the thread index through an opaque move: nothing of the second pass is computed (and kept in registers)
        // ahead of the loop above
        int tid2 = threadIdx.x;
        asm volatile("" : "+v"(tid2));
        attn_body<2>(a, tid2);
        return;
    }

    // ---- O[q][head*64 + d] = O^T / l ; lane holds d = 32*dt + 8*(e/4) + 4*fh + e%4 of query fr
    uint16_t* O = (uint16_t*)a.O;
#pragma unroll
    for (int qt = 0; qt < 2; ++qt) {
        int64_t tok;
        bool ok;
        PS_QTOK(qt, tok, ok);
        if (!ok) continue;
        // A lane holds four consecutive d (8 bytes) of its query per (dt, eg), lane ^ 32 the next four.  The two halves
        // trade them so that the lower half owns the even eg chunks and the upper half the odd ones: 16-byte stores.
        uint16_t* op = O + tok * C + head * ATT_D + 8 * fh;
#pragma unroll
        for (int dt = 0; dt < 2; ++dt)
#pragma unroll
            for (int eg = 0; eg < 4; eg += 2) {
                uint32_t w[2][2];               // [eg parity][dword]
#pragma unroll
                for (int q = 0; q < 2; ++q) {
                    w[q][0] = pack_bf16x2(acc_o[qt][dt][4 * (eg + q)] * inv[qt], acc_o[qt][dt][4 * (eg + q) + 1] * inv[qt]);
                    w[q][1] = pack_bf16x2(acc_o[qt][dt][4 * (eg + q) + 2] * inv[qt], acc_o[qt][dt][4 * (eg + q) + 3] * inv[qt]);
                }
                const auto r0_ = __builtin_amdgcn_permlane32_swap(w[0][0], w[1][0], false, false);
                const auto r1_ = __builtin_amdgcn_permlane32_swap(w[0][1], w[1][1], false, false);
                *reinterpret_cast<u32x4*>(op + dt * 32 + eg * 8) = u32x4{r0_[0], r1_[0], r0_[1], r1_[1]};
            }
    }
#undef PS_QTOK
}

// ---- few keys (the text tokens of cross-attention: at most 128 per request) ------------------------------------
// With 77 keys a query tile is two key tiles of work behind a full prologue (query fragments, K / V^T staging), and
// every 128 queries pay it again.  Here a block belongs to one (request, head): it stages that pair's keys and values in
// LDS ONCE and then walks over query tiles of 128 rows (tile c, c + chunks, ...), the query fragments of the next tile
// in flight while the current one is computed.  All scores of a query fit the registers (128 keys x 32 queries per
// wavefront = 64 per lane), so the softmax is the plain three-pass form: exact row maximum, exponentials, sum.
constexpr int ATT_XK = 128;      // keys the kernel takes at most

__global__ void __launch_bounds__(256, 3)
attn_cross_kernel(AttnArgs a, int chunks) {
    u32x4* sK = reinterpret_cast<u32x4*>(att_smem);            // [2 tiles][64 keys][8 chunks], chunk ^ ((key>>1)&7)
    u32x4* sV = sK + 2 * 512;                                  // [2 tiles][64 d][8 chunks of 8 keys], chunk ^ ((d>>1)&7)
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int fr = lane & 31, fh = lane >> 5;
    // head fastest: the blocks that run at the same time read and write the same token rows (all heads of a row
    // are one contiguous piece of memory), which keeps the DRAM pages they touch few
    const int head = blockIdx.x % a.heads;
    const int sc_ = blockIdx.x / a.heads;
    const int c0 = sc_ % chunks, s = sc_ / chunks;
    const int S = a.geom.S;
    const int rows_s = (a.act_off[s + 1] - a.act_off[s]) * S;            // computed query rows of this request
    const int tiles_s = (rows_s + 127) >> 7;
    if (c0 >= tiles_s) return;
    const int nk = a.cross_len;
    const int64_t k0 = (int64_t)a.perm[s] * a.cross_ld;
    const uint16_t* Q = (const uint16_t*)a.Q;
    const uint16_t* K = (const uint16_t*)a.K;
    const uint16_t* V = (const uint16_t*)a.V;
    const int C = a.C;

    // ---- keys and values of the pair: rows / chunks past the last key are clamped to valid ones (masked below)
    {
        const int lc = lane & 7, lr = 8 * wave + (lane >> 3);
        const int gc = lc ^ ((lr >> 1) & 7);
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                const int key = min(t * 64 + lr + 32 * i, nk - 1);
                __builtin_amdgcn_global_load_lds((const void*)(K + (k0 + key) * C + head * ATT_D + gc * 8),
                                                 (lds_void*)(sK + t * 512 + wave * 64 + i * 256), 16, 0, 0);
                const int vc = t * 64 + gc * 8 < nk ? t * 64 + gc * 8 : 0;
                __builtin_amdgcn_global_load_lds((const void*)(V + (int64_t)(head * ATT_D + lr + 32 * i) * a.ldv + k0 + vc),
                                                 (lds_void*)(sV + t * 512 + wave * 64 + i * 256), 16, 0, 0);
            }
    }
    // query fragments of a tile: lane holds Q[q][16*ks + 8*fh .. +8] of its query column
    auto query = [&](int tile, bf16x8 (&fq)[4], int64_t& tok, bool& ok) {
        int r = tile * 128 + wave * 32 + fr;
        ok = r < rows_s;
        if (!ok) r = rows_s - 1;
        const int pi = a.act_off[s] + r / S;
        const int p = a.act.active ? a.act.active[pi] : pi;
        tok = (int64_t)p * S + (r - (r / S) * S);
        const uint16_t* qp = Q + tok * C + head * ATT_D + fh * 8;
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) fq[ks] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(qp + ks * 16));
    };
    bf16x8 fq[4];
    int64_t tok;
    bool ok;
    query(c0, fq, tok, ok);
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();                                        // keys and values are in LDS for the rest of the block's life

    const int krow[2] = {kperm(fr), kperm(fr) + 32};
    const int ksw = (krow[0] >> 1) & 7, vsw = (fr >> 1) & 7;
    const int nunit = (nk + 31) >> 5;                       // 32-key units that hold keys at all (1 .. 4)
    uint16_t* O = (uint16_t*)a.O;
    for (int tile = c0; tile < tiles_s; tile += chunks) {
        // the next tile's query fragments travel while this tile is computed
        bf16x8 fq_n[4];
        int64_t tok_n = tok;
        bool ok_n = false;
        const bool more = tile + chunks < tiles_s;
        if (more) query(tile + chunks, fq_n, tok_n, ok_n);
        // scores: unit u = 2*t + h holds keys 64 t + 32 h + 16 (e >> 3) + 8 fh + (e & 7)
        f32x16 sc[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
#pragma unroll
            for (int e = 0; e < 16; ++e) sc[u][e] = 0.f;
            if (u < nunit) {
#pragma unroll
                for (int ks = 0; ks < 4; ++ks) {
                    const bf16x8 fk = __builtin_bit_cast(bf16x8, sK[(u >> 1) * 512 + krow[u & 1] * 8 + ((2 * ks + fh) ^ ksw)]);
                    sc[u] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fk, fq[ks], sc[u], 0, 0, 0);
                }
            }
        }
        float m = -INFINITY;
#pragma unroll
        for (int u = 0; u < 4; ++u)
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int key = 32 * u + 16 * (e >> 3) + 8 * fh + (e & 7);
                if (key >= nk) sc[u][e] = -INFINITY;
                m = fmaxf(m, sc[u][e]);
            }
        m = half_swap_max(m);
        float l = 0.f;
        u32x4 fp[4][2];
#pragma unroll
        for (int u = 0; u < 4; ++u)
#pragma unroll
            for (int g = 0; g < 8; ++g) {
                const float p0 = __builtin_amdgcn_exp2f(sc[u][2 * g] - m), p1 = __builtin_amdgcn_exp2f(sc[u][2 * g + 1] - m);
                l += p0 + p1;
                fp[u][g >> 2][g & 3] = pack_bf16x2(p0, p1);
            }
        l += other_half(l);
        f32x16 acc_o[2];
#pragma unroll
        for (int dt = 0; dt < 2; ++dt)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc_o[dt][e] = 0.f;
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            if (u < nunit) {
#pragma unroll
                for (int k2 = 0; k2 < 2; ++k2)
#pragma unroll
                    for (int dt = 0; dt < 2; ++dt) {
                        const bf16x8 fv = __builtin_bit_cast(bf16x8, sV[(u >> 1) * 512 + (fr + 32 * dt) * 8 + ((4 * (u & 1) + 2 * k2 + fh) ^ vsw)]);
                        acc_o[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fv, __builtin_bit_cast(bf16x8, fp[u][k2]), acc_o[dt], 0, 0, 0);
                    }
            }
        }
        // O[q][head*64 + d] = O^T / l; the lane halves trade pieces so that every store is 16 bytes (as in attn_body;
        // the two lanes of an exchange hold the same query row, so they are in or out together)
        if (ok) {
            const float inv = 1.f / l;
            uint16_t* op = O + tok * C + head * ATT_D + 8 * fh;
#pragma unroll
            for (int dt = 0; dt < 2; ++dt)
#pragma unroll
                for (int eg = 0; eg < 4; eg += 2) {
                    uint32_t w[2][2];
#pragma unroll
                    for (int q = 0; q < 2; ++q) {
                        w[q][0] = pack_bf16x2(acc_o[dt][4 * (eg + q)] * inv, acc_o[dt][4 * (eg + q) + 1] * inv);
                        w[q][1] = pack_bf16x2(acc_o[dt][4 * (eg + q) + 2] * inv, acc_o[dt][4 * (eg + q) + 3] * inv);
                    }
                    const auto r0_ = __builtin_amdgcn_permlane32_swap(w[0][0], w[1][0], false, false);
                    const auto r1_ = __builtin_amdgcn_permlane32_swap(w[0][1], w[1][1], false, false);
                    *reinterpret_cast<u32x4*>(op + dt * 32 + eg * 8) = u32x4{r0_[0], r1_[0], r0_[1], r1_[1]};
                }
        }
        if (more) {
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) fq[ks] = fq_n[ks];
            tok = tok_n;
            ok = ok_n;
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
    if (a.cross_len && a.cross_len <= ATT_XK) {
        // one block per (request, head, chunk of its query tiles): about six blocks per CU in all (three run at once)
        const int64_t pairs = (int64_t)a.n * a.heads;
        const int tiles_max = (int)cdiv(a.max_rows, 128);
        const int chunks = (int)std::max<int64_t>(1, std::min<int64_t>(tiles_max, cdiv(1536, pairs)));
        attn_cross_kernel<<<(unsigned)(pairs * chunks), 256, 4 * 512 * 16, st>>>(a, chunks);
        return check_launch("attn_cross_kernel");
    }
    const int64_t items = (int64_t)a.max_tiles * a.heads;
    const unsigned grid = (unsigned)(8 * ATT_GROUP * cdiv(items, 8 * ATT_GROUP));
    constexpr int lds = ATT_NS * 2 * 512 * 16;
    constexpr int lds_pipe = ATT_PNS * 2 * 512 * 16;
    PS_SET_LDS_ONCE(attn_mfma_kernel<1>, lds);
    PS_SET_LDS_ONCE(attn_pipe_kernel, lds_pipe);
    if (a.qt == 1) attn_mfma_kernel<1><<<grid, 256, lds, st>>>(a);
    else attn_pipe_kernel<<<grid, 256, lds_pipe, st>>>(a);
    return check_launch("attn_mfma_kernel");
}

}  // namespace pserve
