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
// B operand of O^T = V^T P^T (keys of a 16-wide MFMA step are taken in the order the
// accumulator holds them; V^T is read from LDS in the same order).  V is kept transposed in
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

constexpr int ATT_BQ = 256;      // queries per block
constexpr int ATT_BKV = 64;      // keys per step
constexpr int ATT_D = 64;        // head dim
constexpr float ATT_TAU = 8.f;   // the softmax reference moves when a shifted score exceeds this (p <= 2^8)

// value of lane l^32 (v_permlane32_swap: upper half of the first operand <-> lower half of the second)
__device__ __forceinline__ float other_half(float v) {
    const uint32_t u = __float_as_uint(v);
    const auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
    // r[0]: lanes 0-31 own low value, lanes 32-63 the low half's value; r[1]: lanes 0-31 the high half's value
    return __uint_as_float((threadIdx.x & 32) ? r[0] : r[1]);
}
__device__ __forceinline__ float half_swap_max(float v) { return fmaxf(v, other_half(v)); }

__global__ void __launch_bounds__(256, 2)
attn_mfma_kernel(AttnArgs a) {
    __shared__ __attribute__((aligned(16))) u32x4 sK[2][ATT_BKV * 8];      // [key][8 chunks of 16 B], chunk ^ ((key>>1)&7)
    __shared__ __attribute__((aligned(16))) u32x2 sV[2][ATT_D * 16];       // [d][16 chunks of 8 B], chunk ^ g(d)

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
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
    else { k0 = a.cu_seqlens[s]; nk = a.cu_seqlens[s + 1] - a.cu_seqlens[s]; }

    const uint16_t* Q = (const uint16_t*)a.Q;
    const uint16_t* K = (const uint16_t*)a.K;
    const uint16_t* V = (const uint16_t*)a.V;
    const int C = a.C;

    // ---- query fragments: lane holds Q[q][16*ks + 8*fh .. +8] of its query column, both query sub-tiles
    int64_t q_tok[2];
    bool q_ok[2];
    bf16x8 fq[2][4];
#pragma unroll
    for (int qt = 0; qt < 2; ++qt) {
        int r = r0 + wave * 64 + qt * 32 + fr;
        q_ok[qt] = r < rows_s;
        if (!q_ok[qt]) r = rows_s - 1;
        const int pi = a.act_off[s] + r / S;
        const int p = a.act.active ? a.act.active[pi] : pi;
        q_tok[qt] = (int64_t)p * S + (r - (r / S) * S);
        const uint16_t* qp = Q + q_tok[qt] * C + head * ATT_D + fh * 8;
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) fq[qt][ks] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(qp + ks * 16));
    }

    // ---- staging: thread loads 2 chunks of K and 2 chunks of V^T per step
    const int lrow = tid >> 3, lc = tid & 7;                 // rows lrow and lrow + 32, 16-byte chunk lc
    const uint16_t* kp = K + (k0 + lrow) * C + head * ATT_D + lc * 8;
    const uint16_t* vp = V + (int64_t)(head * ATT_D + lrow) * a.ldv + k0 + lc * 8;
    const int64_t k_row32 = (int64_t)32 * C, v_row32 = (int64_t)32 * a.ldv;
    int sk_slot[2], sv_slot[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int row = lrow + 32 * i;
        sk_slot[i] = row * 8 + (lc ^ ((row >> 1) & 7));
        const int g = ((row & 7) << 1) | ((row >> 3) & 1);
        sv_slot[i][0] = row * 16 + ((2 * lc) ^ g);
        sv_slot[i][1] = row * 16 + ((2 * lc + 1) ^ g);
    }
    u32x4 rk[2], rv[2];
    const u32x4 zero4 = {0, 0, 0, 0};

    f32x16 acc_o[2][2];
#pragma unroll
    for (int qt = 0; qt < 2; ++qt)
#pragma unroll
        for (int dt = 0; dt < 2; ++dt)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc_o[qt][dt][e] = 0.f;
    float m_ref[2] = {0.f, 0.f}, l_run[2] = {0.f, 0.f};   // reference maximum (log2 domain) and partial row sums

    // step 0 into LDS
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const bool kin = lrow + 32 * i < nk;
        rk[i] = kin ? *reinterpret_cast<const u32x4*>(kp + i * k_row32) : zero4;
        const bool vin = lc * 8 < nk;
        rv[i] = vin ? *reinterpret_cast<const u32x4*>(vp + i * v_row32) : zero4;
    }
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        sK[0][sk_slot[i]] = rk[i];
        sV[0][sv_slot[i][0]] = u32x2{rv[i][0], rv[i][1]};
        sV[0][sv_slot[i][1]] = u32x2{rv[i][2], rv[i][3]};
    }
    __syncthreads();

    const int steps = (nk + ATT_BKV - 1) / ATT_BKV;
    for (int st = 0; st < steps; ++st) {
        const int buf = st & 1;
        const int kv0 = st * ATT_BKV;
        // prefetch the next step (the last iteration loads nothing)
        const int kvn = kv0 + ATT_BKV;
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const bool kin = kvn + lrow + 32 * i < nk;
            rk[i] = kin ? *reinterpret_cast<const u32x4*>(kp + (int64_t)kvn * C + i * k_row32) : zero4;
            const bool vin = kvn + lc * 8 < nk;
            rv[i] = vin ? *reinterpret_cast<const u32x4*>(vp + kvn + i * v_row32) : zero4;
        }

        // ---- S^T = K Q^T - m_ref : the accumulators start at minus the reference maximum of their query column,
        // so the products come out already shifted.  lane: query fr, keys 32*kt + 8*(e/4) + 4*fh + e%4
        f32x16 acc_s[2][2];
#pragma unroll
        for (int qt = 0; qt < 2; ++qt)
#pragma unroll
            for (int kt = 0; kt < 2; ++kt)
#pragma unroll
                for (int e = 0; e < 16; ++e) acc_s[qt][kt][e] = -m_ref[qt];
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            bf16x8 fk[2];
#pragma unroll
            for (int kt = 0; kt < 2; ++kt) {
                const int row = kt * 32 + fr;
                fk[kt] = __builtin_bit_cast(bf16x8, sK[buf][row * 8 + ((2 * ks + fh) ^ ((row >> 1) & 7))]);
            }
#pragma unroll
            for (int qt = 0; qt < 2; ++qt)
#pragma unroll
                for (int kt = 0; kt < 2; ++kt)
                    acc_s[qt][kt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fk[kt], fq[qt][ks], acc_s[qt][kt], 0, 0, 0);
        }
        if (kv0 + ATT_BKV > nk) {                  // ragged last step: keys past the image get -inf
#pragma unroll
            for (int kt = 0; kt < 2; ++kt)
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    const int key = kv0 + 32 * kt + 8 * (e >> 2) + 4 * fh + (e & 3);
                    if (key >= nk) { acc_s[0][kt][e] = -INFINITY; acc_s[1][kt][e] = -INFINITY; }
                }
        }

        // ---- online softmax with a lazily updated reference maximum.  p = 2^(s - m_ref) is exact softmax
        // numerator up to the common factor 2^(-m_ref); the reference only moves (and O, l are rescaled) when a
        // column's shifted maximum exceeds ATT_TAU, i.e. before p could grow past 2^ATT_TAU.  The first step
        // always anchors the reference at the true maximum.  The decision is wavefront-uniform.
        float mx[2];
#pragma unroll
        for (int qt = 0; qt < 2; ++qt) {
            float m = -INFINITY;
#pragma unroll
            for (int kt = 0; kt < 2; ++kt)
#pragma unroll
                for (int e = 0; e < 16; ++e) m = fmaxf(m, acc_s[qt][kt][e]);
            mx[qt] = half_swap_max(m);
        }
        if (st == 0 || __any(mx[0] > ATT_TAU || mx[1] > ATT_TAU)) {
#pragma unroll
            for (int qt = 0; qt < 2; ++qt) {
                const float d = (st == 0 || mx[qt] > ATT_TAU) ? mx[qt] : 0.f;    // shift of this column's reference
                const float corr = st == 0 ? 1.f : __builtin_amdgcn_exp2f(-d);   // O and l are still zero in step 0
                m_ref[qt] += d;
                l_run[qt] *= corr;
#pragma unroll
                for (int kt = 0; kt < 2; ++kt)
#pragma unroll
                    for (int e = 0; e < 16; ++e) acc_s[qt][kt][e] -= d;
#pragma unroll
                for (int dt = 0; dt < 2; ++dt)
#pragma unroll
                    for (int e = 0; e < 16; ++e) acc_o[qt][dt][e] *= corr;
            }
        }
        bf16x8 fp[2][4];                           // P leaves as the B operand of the PV product
#pragma unroll
        for (int qt = 0; qt < 2; ++qt) {
            float sum = 0.f;
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) {
                float pv[8];
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    pv[i] = __builtin_amdgcn_exp2f(acc_s[qt][ks >> 1][8 * (ks & 1) + i]);
                    sum += pv[i];
                }
                u32x4 pk;
#pragma unroll
                for (int i = 0; i < 4; ++i) pk[i] = pack_bf16x2(pv[2 * i], pv[2 * i + 1]);
                fp[qt][ks] = __builtin_bit_cast(bf16x8, pk);
            }
            l_run[qt] += sum;
        }

        // ---- O^T += V^T P^T : A operand = V^T rows (d), keys 16*ks + 8*(i/4) + 4*fh + i%4
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            bf16x8 fv[2];
#pragma unroll
            for (int dt = 0; dt < 2; ++dt) {
                const int row = dt * 32 + fr;
                const int g = ((row & 7) << 1) | ((row >> 3) & 1);
                const u32x2 lo2 = sV[buf][row * 16 + ((4 * ks + fh) ^ g)];
                const u32x2 hi2 = sV[buf][row * 16 + ((4 * ks + fh + 2) ^ g)];
                fv[dt] = __builtin_bit_cast(bf16x8, u32x4{lo2[0], lo2[1], hi2[0], hi2[1]});
            }
#pragma unroll
            for (int qt = 0; qt < 2; ++qt)
#pragma unroll
                for (int dt = 0; dt < 2; ++dt)
                    acc_o[qt][dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fv[dt], fp[qt][ks], acc_o[qt][dt], 0, 0, 0);
        }

        // ---- stage the prefetched step
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            sK[buf ^ 1][sk_slot[i]] = rk[i];
            sV[buf ^ 1][sv_slot[i][0]] = u32x2{rv[i][0], rv[i][1]};
            sV[buf ^ 1][sv_slot[i][1]] = u32x2{rv[i][2], rv[i][3]};
        }
        __syncthreads();
    }

    // ---- O[q][head*64 + d] = O^T / l ; lane holds d = 32*dt + 8*(e/4) + 4*fh + e%4 of query fr
    uint16_t* O = (uint16_t*)a.O;
#pragma unroll
    for (int qt = 0; qt < 2; ++qt) {
        const float l = l_run[qt] + other_half(l_run[qt]);
        const float inv = 1.f / l;
        if (!q_ok[qt]) continue;
        uint16_t* op = O + q_tok[qt] * C + head * ATT_D + 4 * fh;
#pragma unroll
        for (int dt = 0; dt < 2; ++dt)
#pragma unroll
            for (int eg = 0; eg < 4; ++eg) {
                const uint32_t w0 = pack_bf16x2(acc_o[qt][dt][4 * eg] * inv, acc_o[qt][dt][4 * eg + 1] * inv);
                const uint32_t w1 = pack_bf16x2(acc_o[qt][dt][4 * eg + 2] * inv, acc_o[qt][dt][4 * eg + 3] * inv);
                *reinterpret_cast<u32x2*>(op + dt * 32 + eg * 8) = u32x2{w0, w1};
            }
    }
}

// One block: per request slot, number of computed patches and of query tiles (exclusive prefixes).
__global__ void attn_tiles_kernel(const int32_t* __restrict__ request_offset, const uint8_t* __restrict__ mask, int32_t n,
                                  int32_t S, int32_t* __restrict__ act_off, int32_t* __restrict__ tile_off) {
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

int attention_tiles(const int32_t* request_offset, const uint8_t* mask, int32_t n, int32_t S, int32_t* act_off,
                    int32_t* tile_off, hipStream_t st) {
    attn_tiles_kernel<<<1, 1024, 0, st>>>(request_offset, mask, n, S, act_off, tile_off);
    return check_launch("attn_tiles_kernel");
}

int attention_max_tiles(const pserve_plan_t* plan) {
    int64_t t = 0;
    const auto& ro = plan->h_tab[PSERVE_TAB_REQUEST_OFFSET];
    for (int s = 0; s < plan->n; ++s) t += cdiv((int64_t)(ro[s + 1] - ro[s]) * plan->S, ATT_BQ);
    return (int)t;
}

int attention_mfma_bf16(const AttnArgs& a, hipStream_t st, bool* handled) {
    *handled = false;
    if (a.d != ATT_D || !a.v_transposed || !a.tile_off || !a.act_off) return PSERVE_OK;
    if (a.C % 8 != 0 || a.ldv % 8 != 0) return PSERVE_OK;
    if (a.cross_len) {
        if (a.cross_ld % 8 != 0) return PSERVE_OK;
    } else if (a.geom.S % 8 != 0) {
        return PSERVE_OK;              // image token ranges must start on 16-byte boundaries of the V^T rows
    }
    *handled = true;
    const int64_t items = (int64_t)a.max_tiles * a.heads;
    const unsigned grid = (unsigned)(8 * cdiv(items, 8));
    attn_mfma_kernel<<<grid, 256, 0, st>>>(a);
    return check_launch("attn_mfma_kernel");
}

}  // namespace pserve
