/*
 * pserve — one denoising block over a batch of mixed-resolution latents cut into
 * equal patches (PatchedServe, arXiv 2501.09253, section "Patched Inference with
 * Batching" and section "Exploiting Patch-Level Locality").
 *
 * C ABI of libpserve.so.  Every entry point is extern "C", takes plain pointers and
 * sizes, returns an int status (0 = PSERVE_OK, negative = error) and never throws or
 * aborts.  pserve_last_error() gives a thread-local description of the last failure.
 *
 * Conventions
 *   - "device" pointers are HIP device memory of the current device; "host" pointers
 *     are ordinary process memory.  `stream` is a hipStream_t passed as void*
 *     (NULL = the default stream).  All device work is enqueued on `stream` and is
 *     asynchronous; errors detectable on the host are returned synchronously.
 *   - Per-request arrays (resolutions, images, text context) are in CALLER order.
 *     Per-patch arrays (reuse mask, tables) are in PLAN order (requests sorted by
 *     resolution; use the PERM / PATCH_OWNER / PATCH_RC tables to map).
 *   - Activations are token-major, channels-last, patch-major: x[T][C] with token id
 *     t = patch*ph*pw + y*pw + x.  dtype is PSERVE_F32 (float) or PSERVE_BF16
 *     (bfloat16 storage, float accumulation); every tensor of a block, parameters
 *     included, has the block's dtype.
 *   - The caller owns x, y, images, parameters, ctx and masks.  The library owns plan
 *     tables, packed weights and cache / scratch buffers; pserve_block_forward
 *     allocates nothing.
 */
#ifndef PSERVE_H
#define PSERVE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define PSERVE_OK       0
#define PSERVE_EINVAL  (-1)   /* bad argument (shape, divisibility, NULL, unsupported dtype/stage) */
#define PSERVE_ENOMEM  (-2)   /* host or device allocation failed */
#define PSERVE_EHIP    (-3)   /* a HIP runtime call failed */
#define PSERVE_ESTATE  (-4)   /* object used in a state that does not allow the call */

#define PSERVE_F32   0
#define PSERVE_BF16  1

/* stage kinds of the block grammar */
#define PSERVE_RES1   1   /* x + conv3(SiLU(GN(x)))                                    params: gn_g gn_b conv_w conv_b */
#define PSERVE_RES2   2   /* x + conv3_b(SiLU(GN_b(conv3_a(SiLU(GN_a(x))))))            params: gn_a_g gn_a_b conv_a_w conv_a_b gn_b_g gn_b_b conv_b_w conv_b_b */
#define PSERVE_SATTN  3   /* x + MHA(GN(x))W_o + b_o, keys = all tokens of the own image params: gn_g gn_b wq wk wv wo bo */
#define PSERVE_XATTN  4   /* x + MHA(x W_q; ctx W_k, ctx W_v)W_o + b_o                  params: wq wk wv wo bo */
#define PSERVE_FFN    5   /* x + (a * GELU(g))W_2 + b_2, [a|g] = x W_1 + b_1            params: w1 b1 w2 b2 */
/* The three token stages with a per-token LayerNorm over the C channels in front (biased variance, desc.eps, affine):
 * the transformer layer of an SDXL level.  A per-pixel operator needs nothing from other patches ("Patch-Tailored
 * Diffusion Operators"), so LSATTN caches K and V only (no PSERVE_SLOT_R). */
#define PSERVE_LSATTN 6   /* x + MHA(LN(x))W_o + b_o, keys = all tokens of the own image params: ln_g ln_b wq wk wv wo bo */
#define PSERVE_LXATTN 7   /* x + MHA(LN(x) W_q; ctx W_k, ctx W_v)W_o + b_o              params: ln_g ln_b wq wk wv wo bo */
#define PSERVE_LFFN   8   /* x + (a * GELU(g))W_2 + b_2, [a|g] = LN(x) W_1 + b_1        params: ln_g ln_b w1 b1 w2 b2 */
/* RES2 with the time embedding of the residual block of an SDXL level: the request's embedding vector goes through
 * SiLU and a linear layer and the C results are added to every pixel of the first convolution's output (a per-pixel
 * operator with a per-request operand): h1 = conv3_a(SiLU(GN_a(x))) + SiLU(temb) W_t + b_t.  Needs desc.temb_dim and
 * pserve_block_forward_temb.  params: the eight of RES2, then wt [temb_dim][C], bt [C] */
#define PSERVE_RES2T  9
/* Sub-layers of a block of the second model family (a diffusion transformer): the request's conditioning vector c (the
 * `temb` argument of pserve_block_forward_temb, desc.temb_dim wide) gives (shift, scale, gate) = thirds of
 * SiLU(c) W_m + b_m; the sub-layer sees h = LN0(x) * (1 + scale) + shift (LN0: LayerNorm over the channels without
 * affine) and its output is multiplied by gate before the residual add.  Per-pixel operators with per-request
 * operands; ASATTN caches K and V like LSATTN.  The joint text-image attention of that model is not part of them. */
#define PSERVE_ASATTN 10  /* x + gate * (MHA(h) W_o + b_o)                              params: wm [temb_dim][3C] bm [3C] wq wk wv wo bo */
#define PSERVE_AMLP   11  /* x + gate * (GELU_tanh(h W_1 + b_1) W_2 + b_2), W_1 [C][ffn_mult*C]  params: wm bm w1 b1 w2 b2 */
/* One whole joint block of that model on a joint plan (pserve_plan_text; x holds image AND text patches).  Each of
 * the two streams (image tokens, text tokens) has its own weights; (sh1, sc1, g1, sh2, sc2, g2) = sixths of
 * SiLU(c) W_m + b_m per stream; q, k, v from h = LN0(x)(1 + sc1) + sh1; ONE attention per request over its image and
 * text tokens together; x += g1 * (o W_o + b_o); x += g2 * (GELU_tanh(h2 W_1 + b_1) W_2 + b_2), h2 = LN0(x)(1 + sc2) + sh2.
 * A block with a PSERVE_MMDIT stage holds only such stages, needs a joint plan, and has no cache slots (no reuse mask).
 * params: image stream wm [temb_dim][6C] bm [6C] wq wk wv wo [C][C] bo [C] w1 [C][F] b1 [F] w2 [F][C] b2 [C]
 * (F = ffn_mult*C), then the same eleven for the text stream. */
#define PSERVE_MMDIT  12

#define PSERVE_MAX_STAGES 8
#define PSERVE_MAX_PARAMS 24

/* plan tables (int32) for pserve_plan_table */
#define PSERVE_TAB_PERM            0   /* [n]      caller index of sorted slot s */
#define PSERVE_TAB_REQUEST_OFFSET  1   /* [n+1]    first patch of sorted slot s (RequestOffset of the CSP format) */
#define PSERVE_TAB_RES_OFFSET      2   /* [R+1]    first sorted slot of each distinct resolution */
#define PSERVE_TAB_RES_HW          3   /* [R][2]   the distinct resolutions (H, W), ascending */
#define PSERVE_TAB_PATCH_OWNER     4   /* [P]      sorted slot owning patch p (the per-patch request index) */
#define PSERVE_TAB_PATCH_RC        5   /* [P][2]   (row, col) of patch p in its image's patch grid */
#define PSERVE_TAB_NEIGHBOUR       6   /* [P][8]   patch ids NW N NE W E SW S SE, -1 = absent (zero fill) */
#define PSERVE_TAB_HALO_SRC        7   /* [P][2(pw+2)+2ph] global token id of each ring pixel, -1 = outside the image;
                                          ring order: top row x=-1..pw, bottom row x=-1..pw, left col y=0..ph-1, right col y=0..ph-1 */
#define PSERVE_TAB_CU_SEQLENS      8   /* [n+1]    first token of sorted slot s */
#define PSERVE_TAB_SEQ_LEN         9   /* [n]      valid tokens of sorted slot s: H*W, plus text_len in a joint plan */
#define PSERVE_TAB_COUNT           10

/* cache slots of a stage (pserve_cache_load / pserve_cache_read); stage = -1 addresses the block output slot */
#define PSERVE_SLOT_H1  0   /* RES2, RES2T: output of the first convolution (RES2T: time embedding included) */
#define PSERVE_SLOT_R   1   /* SATTN: stage input */
#define PSERVE_SLOT_K   2   /* SATTN, LSATTN, ASATTN: keys */
#define PSERVE_SLOT_V   3   /* SATTN, LSATTN, ASATTN: values */
#define PSERVE_SLOT_Y   4   /* block output (use stage = -1) */

typedef struct pserve_plan_s pserve_plan_t;    /* CSP tables of one batch composition (host + device copies) */
typedef struct pserve_block_s pserve_block_t;   /* block description + packed weights */
typedef struct pserve_cache_s pserve_cache_t;   /* per (plan, block): cached operand tensors + scratch */

typedef struct {
    int32_t n;        /* requests */
    int32_t R;        /* distinct resolutions */
    int32_t P;        /* patches */
    int32_t ph, pw;   /* patch height / width (latent pixels) */
    int32_t ring;     /* 2(pw+2)+2ph, entries of HALO_SRC per patch */
    int64_t T;        /* tokens = P*ph*pw */
    int32_t text_len;      /* text tokens per request (pserve_plan_text), else 0 */
    int32_t text_patches;  /* ceil(text_len / (ph*pw)): extra patches per request, counted in P and T */
} pserve_plan_info_t;

typedef struct {
    int32_t n_stages;
    int32_t stages[PSERVE_MAX_STAGES];   /* PSERVE_RES1 .. PSERVE_MMDIT, in execution order */
    int32_t C;          /* channels */
    int32_t G;          /* GroupNorm groups (C % G == 0) */
    int32_t heads;      /* attention heads (C % heads == 0) */
    int32_t dtype;      /* PSERVE_F32 | PSERVE_BF16 */
    float   eps;        /* GroupNorm / LayerNorm epsilon */
    int32_t ctx_len;    /* text tokens per request (XATTN), else 0 */
    int32_t ctx_dim;    /* width of a text token (XATTN), else 0 */
    int32_t ffn_mult;   /* FFN hidden width = ffn_mult*C (W_1 is C x 2*ffn_mult*C) */
    int32_t temb_dim;   /* width of the per-request vector (RES2T: time embedding; ASATTN / AMLP: conditioning), else 0 */
} pserve_block_desc;

/* Device pointers of the parameters of every stage, in the order listed beside the
 * stage kinds above.  Layouts: conv weights W[Cout][Cin][3][3] (cross-correlation,
 * zero padding 1); linear weights W[Cin][Cout] (y = x W); vectors [C]. */
typedef struct {
    const void* p[PSERVE_MAX_STAGES][PSERVE_MAX_PARAMS];
} pserve_block_params;

const char* pserve_last_error(void);

/* ---- planner: Compressed Sparse Patch tables ("Compressed Sparse Patch Format") and
 * per-patch neighbour metadata ("Patch-Tailored Diffusion Operators", patch-based
 * convolution).  resolutions_hw: HOST int32 [n][2] = (H, W) in latent pixels, caller
 * order.  ph = pw = 0 selects the greatest common divisor of all heights resp. widths
 * (the paper's patch-size rule).  Requests are sorted ascending by (H, W), stable.
 * The tables are built by device kernels on `stream`; the call returns after they are
 * complete (it synchronises the stream once to mirror them on the host).
 * Errors: EINVAL for n <= 0, non-positive sizes, H % ph != 0, W % pw != 0, or more
 * than 2^31-1 tokens; ENOMEM; EHIP.  *out is owned by the caller until pserve_plan_free. */
int  pserve_plan(const int32_t* resolutions_hw, int32_t n, int32_t ph, int32_t pw,
                 void* stream, pserve_plan_t** out);
/* The same for the joint text-image attention of the paper's second model ("Patch-based Self-Attention Module":
 * every token attends to the tokens of its own request): the text_len text tokens of a request ride along as
 * ceil(text_len / (ph*pw)) extra patches behind its image patches (grid position (-1, k), no neighbours, no halo), so
 * that per-token operators and the per-request attention take them in without a second code path.  SEQ_LEN[s] = H*W +
 * text_len counts the valid tokens of slot s: its key set is the token range [CU_SEQLENS[s], CU_SEQLENS[s] +
 * SEQ_LEN[s]); the padding rows of the last text patch lie behind it.  split / reassemble move image patches only;
 * pserve_text_scatter copies text DEVICE [n][text_len][C] (caller order) into the text patches of x (padding rows
 * zeroed), pserve_text_gather copies them back out.  text_len = 0 gives pserve_plan. */
int  pserve_plan_text(const int32_t* resolutions_hw, int32_t n, int32_t ph, int32_t pw, int32_t text_len,
                      void* stream, pserve_plan_t** out);
int  pserve_text_scatter(const pserve_plan_t* plan, const void* text, int32_t C, int dtype, void* x, void* stream);
int  pserve_text_gather(const pserve_plan_t* plan, const void* x, int32_t C, int dtype, void* text, void* stream);
void pserve_plan_free(pserve_plan_t* plan);
int  pserve_plan_info(const pserve_plan_t* plan, pserve_plan_info_t* out);
/* Borrowed pointer to a table (valid until pserve_plan_free): on_device != 0 gives the
 * device copy, else the host mirror.  *count = number of int32 entries. */
int  pserve_plan_table(const pserve_plan_t* plan, int which, int on_device,
                       const int32_t** ptr, int64_t* count);

/* ---- split / reassembly (patch splitting of "Compressed Sparse Patch Format";
 * rebuilding full images from patches, "Patch-based Self-Attention Module").
 * images: HOST array of n DEVICE pointers, image i is NCHW [C][H_i][W_i] in caller
 * order; x / y: DEVICE [T][C].  Pure copies: bit-exact.  dtype as above. */
int  pserve_split(const pserve_plan_t* plan, const void* const* images, int32_t C, int dtype,
                  void* x, void* stream);
int  pserve_reassemble(const pserve_plan_t* plan, const void* y, int32_t C, int dtype,
                       void* const* images, void* stream);
/* pserve_split that also takes the statistics of the block's first normalisation while the
 * data passes through ("Patch-Tailored Diffusion Operators": the group statistics of a
 * request are those of all its patches): same x, bit for bit; per (patch, token chunk,
 * channel) the mean and the sum of squared deviations go into scratch of `cache` (a cache
 * of this plan), and the NEXT pserve_block_forward call of that cache on this x merges them
 * instead of reading x once more.  Single use: any other forward call, or a later change of
 * x, needs a new split.  Call it on the stream of that forward call (or order the two).
 * Where the fast path does not apply (fp32, channel counts or patch shapes it does not
 * cover, reference kernel mode, joint plans) it is pserve_split and the forward call takes
 * its own statistics.  Errors: EINVAL for NULL arguments or a cache of another plan. */
int  pserve_split_stats(const pserve_plan_t* plan, const void* const* images, int32_t C, int dtype,
                        void* x, pserve_cache_t* cache, void* stream);

/* ---- block: description + weights.  Packs the weights into the layouts the kernels
 * read (device copies owned by the block); the caller's parameter buffers are not
 * referenced after the call returns (it synchronises `stream`).
 * Errors: EINVAL for unknown stage kinds, C % G, C % heads, XATTN without ctx sizes,
 * a NULL parameter; ENOMEM; EHIP. */
int  pserve_block_create(const pserve_block_desc* desc, const pserve_block_params* params,
                         void* stream, pserve_block_t** out);
void pserve_block_free(pserve_block_t* block);

/* ---- per (plan, block) activation store: the cached operand tensors of the patch-level
 * cache ("Patch-aware Caching Strategy": operands of context operators and the block
 * output of the previous step, per patch) plus all scratch the forward pass needs.
 * with_slots = 0 allocates scratch only (then reuse_mask must be NULL). */
int  pserve_cache_create(const pserve_plan_t* plan, const pserve_block_t* block, int with_slots,
                         pserve_cache_t** out);
void pserve_cache_free(pserve_cache_t* cache);
/* Test / warm-start hooks: copy a [T][C] tensor (block dtype, token-major) into or out
 * of a slot.  stage = index into desc.stages (or -1 with PSERVE_SLOT_Y). */
int  pserve_cache_load(pserve_cache_t* cache, int stage, int slot, const void* src, void* stream);
int  pserve_cache_read(const pserve_cache_t* cache, int stage, int slot, void* dst, void* stream);

/* ---- the hot path: run the block on the patch batch.
 *   x    DEVICE [T][C]   input tokens (fresh for every patch)
 *   ctx  DEVICE [n][ctx_len][ctx_dim] text tokens per request, caller order (NULL if no XATTN)
 *   reuse_mask DEVICE uint8 [P], plan order, 1 = reuse the cached patch (skip compute),
 *        0 = compute; NULL = compute everything.
 *   y    DEVICE [T][C]   output; must not alias x.
 * Result: equal (up to rounding order) to running the block on every image on its own,
 * unpatched ("Patched Inference with Batching").  With a mask (steps 3-5 of
 * "Patch-aware Caching Strategy"): pixel-wise operators run on computed patches only;
 * at every operator that needs context (GroupNorm statistics, convolution halos,
 * attention keys/values) reused patches contribute their cached operand; afterwards
 * y of reused patches is the cached output bit for bit, and every slot holds the fresh
 * value on computed patches and keeps the old one on reused patches.
 * Errors: EINVAL (NULL arguments, plan/block/cache mismatch, missing ctx), ESTATE (mask
 * given but the cache has no slots or was never filled), EHIP. */
int  pserve_block_forward(const pserve_plan_t* plan, const void* x, const void* ctx,
                          const pserve_block_t* weights, pserve_cache_t* cache,
                          const uint8_t* reuse_mask, void* y, void* stream);
/* The same with the time embedding of the RES2T stages: temb DEVICE [n][temb_dim] (block dtype), one vector per
 * request, caller order (also the conditioning vector of ASATTN / AMLP); NULL if the block has no such stage (then identical to pserve_block_forward, which is
 * this call with temb = NULL).  Errors as above, EINVAL for a RES2T block without temb. */
int  pserve_block_forward_temb(const pserve_plan_t* plan, const void* x, const void* ctx, const void* temb,
                               const pserve_block_t* weights, pserve_cache_t* cache,
                               const uint8_t* reuse_mask, void* y, void* stream);

/* ---- cache manager pieces around the block ("Patch-aware Caching Strategy", "Batching Patches in Cache").
 *
 * pserve_patch_mse: the feature the cache reuse predictor compares per patch (step 1 of "Patch-aware
 * Caching Strategy": the new input against the cache of the previous step; the similarity metric named
 * in the implementation section is the mean squared error).  a, b: DEVICE [T][C] patch batches of the
 * plan (dtype as above); out: DEVICE float [P], out[p] = mean over the S*C elements of patch p of
 * (a - b)^2, accumulated in fp32 per thread and in a fixed order across threads (deterministic).
 * The partial sums live in scratch owned by the plan: calls on the same plan must not overlap (one stream, or
 * serialised by the caller); calls on different plans are independent.
 * Errors: EINVAL (NULL, C not a multiple of 8 (bf16) / 4 (fp32), C > 8192), EHIP.
 *
 * pserve_cache_sets: id bookkeeping when the batch composition changes between steps.  Every patch has
 * the unique id (request id, patch row, patch column); comparing the ids of the new batch with the ids
 * the cache holds gives the Common Set (in both), the New Set (only in the new batch) and the Expired
 * Set (only in the cache).  old_ids / new_ids: HOST int64 [n], unique per batch, CALLER order of the
 * respective plan.  Outputs: req_src HOST int32 [n_new] = caller index of the same request in the old
 * batch or -1 (New Set); expired HOST uint8 [n_old] = 1 for the Expired Set; patch_src DEVICE int32
 * [P_new] (plan order) = old plan's patch with the same id or -1.  Either host output may be NULL.
 * The call synchronises `stream` (one small host->device copy).
 * Errors: EINVAL (NULL, duplicate ids, different patch sizes, a common request with another resolution).
 *
 * pserve_cache_migrate: the coalesced insert of the Common Set into the cache of the new batch: every
 * slot of new_cache takes, for each new patch p with patch_src[p] >= 0, the rows of old patch
 * patch_src[p] of the same slot of old_cache (bit-exact copies, one launch per slot); other patches are
 * left as they are and must be computed (mask 0) in the next pserve_block_forward.  valid: DEVICE uint8
 * [P_new] or NULL, set to patch_src[p] >= 0.  Both caches must have slots and belong to the same block.
 * Errors: EINVAL, ESTATE (old cache never filled). */
int  pserve_patch_mse(const pserve_plan_t* plan, const void* a, const void* b, int32_t C, int dtype,
                      float* out, void* stream);
/* pserve_patch_mse for callers that cannot allocate device memory or own a plan-side scratch: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same kernels and the same result bit
 * for bit; the partial sums go to a fixed array inside the library's device image (PSERVE_MSE_STATIC_MAX_PATCHES * 16
 * floats = 1 MiB per GPU, held until the process ends) instead of the plan's scratch.  The call allocates nothing and
 * frees nothing.  Every call on one GPU shares that array: calls that overlap on the same GPU (two streams, two
 * threads) race; calls on different GPUs do not.  Nothing needs clearing between calls (every entry read is written
 * first by the same call).
 * Errors: as pserve_patch_mse, and EINVAL when the plan has more than PSERVE_MSE_STATIC_MAX_PATCHES patches. */
#define PSERVE_MSE_STATIC_MAX_PATCHES 16384
int  pserve_patch_mse_static(const pserve_plan_t* plan, const void* a, const void* b, int32_t C, int dtype,
                             float* out, void* stream);
int  pserve_cache_sets(const pserve_plan_t* old_plan, const int64_t* old_ids, const pserve_plan_t* new_plan,
                       const int64_t* new_ids, int32_t* req_src, uint8_t* expired, int32_t* patch_src,
                       void* stream);
int  pserve_cache_migrate(const pserve_cache_t* old_cache, pserve_cache_t* new_cache, const int32_t* patch_src,
                          uint8_t* valid, void* stream);

/* ---- resolution changes between two levels of the network (not part of the paper's block; its patch-size rule, the
 * greatest common divisor of the resolutions, is what makes them keep the patch grid: a ph x pw patch becomes
 * ph/2 x pw/2 resp. 2ph x 2pw, halos come from the neighbour patches as in "Patch-Tailored Diffusion Operators").
 *   PSERVE_DOWN2  3x3 convolution, stride 2, zero padding 1: image [C_in][H][W] -> [C_out][H/2][W/2]; the taps of
 *                 output pixel (oy, ox) are centred on input pixel (2oy, 2ox)
 *   PSERVE_UP2    every pixel repeated 2 x 2 (nearest neighbour), then 3x3 convolution, zero padding 1:
 *                 -> [C_out][2H][2W]
 * pserve_resample_create: w DEVICE [C_out][C_in][3][3], b DEVICE [C_out] (dtype as given); packs them (for UP2 the nine
 * taps are merged, in fp32, into four taps for each of the four output parities) and synchronises `stream`.
 * pserve_resample_forward: x DEVICE [T_in][C_in] on plan_in, y DEVICE [T_out][C_out] on plan_out, where plan_out is
 * the pserve_plan of the halved (doubled) resolutions, same caller order, with the halved (doubled) patch size;
 * workspace DEVICE, at least pserve_resample_workspace bytes (the padded copy of x), owned by the caller; nothing is
 * allocated.  Result: equal (up to rounding order) to the operator applied to every image on its own.
 * Errors: EINVAL (NULL, widths not multiples of 16 bytes, plans that are not such a pair, odd patch size for DOWN2,
 * workspace too small), ENOMEM, EHIP. */
#define PSERVE_DOWN2 1
#define PSERVE_UP2   2
typedef struct pserve_resample_s pserve_resample_t;
int  pserve_resample_create(int kind, int32_t C_in, int32_t C_out, int dtype, const void* w, const void* b,
                            void* stream, pserve_resample_t** out);
void pserve_resample_free(pserve_resample_t* op);
int  pserve_resample_workspace(const pserve_resample_t* op, const pserve_plan_t* plan_in, size_t* bytes);
int  pserve_resample_forward(const pserve_resample_t* op, const pserve_plan_t* plan_in, const pserve_plan_t* plan_out,
                             const void* x, void* workspace, size_t workspace_bytes, void* y, void* stream);

/* ---- host-side scheduler pieces (section "SLO-Aware Scheduler").  All pointers HOST; no GPU work; times in ms.
 *
 * pserve_task: a request as the scheduler sees it.  ddl = its SLO budget counted from arrival (DDL_i), standalone =
 * its latency when run alone (SA_i), steps_left = denoising steps still to run.
 * pserve_slack: the slack score of "SLO-based Scheduling Algorithm": (DDL_i - C_i - P_i) / SA_i with C_i = now -
 * arrival and P_i = steps_left * latency (the predicted per-step latency of the batch the task runs in).
 * pserve_latency_model: stands in for the MLP of "Mixed-Resolution Throughput Analyzer" (which needs the authors'
 * measurements); same inputs, reduced to three features of a batch at patch size ph x pw: per-step latency =
 * w[0] + w[1] * total patches + w[2] * distinct resolutions + w[3] * 1e-6 * sum_i (H_i W_i)^2.
 * pserve_latency_fit: ordinary least squares on m >= 4 samples, X [m][3] = the three features, y [m] = measured
 * latency.  EINVAL if the samples do not determine the four coefficients.
 * pserve_schedule: the scheduling loop of the section's algorithm.  Repeats: take the least-slack waiting task (slack
 * with the latency of the batch it would join) and the least-slack active task; if the candidate would miss its
 * deadline even so (now + steps_left * latency > arrival + ddl) it is discarded; if its slack exceeds relaxed_slack
 * the candidate becomes the waiting task with the most batch tokens per predicted millisecond (among those that
 * would meet their deadline); if the least-slack active task would miss its deadline with the candidate on board the
 * loop stops, else the candidate is admitted and counts as active from then on.  Ties go to queue order.
 * admitted / discarded: HOST int32 [n_wait] each, indices into `wait` in the order decided.
 * Errors: EINVAL (NULL, resolutions that are not multiples of the patch, standalone <= 0). */
typedef struct {
    int64_t id;
    int32_t H, W;
    int32_t steps_left;
    double  arrival, ddl, standalone;
} pserve_task;
typedef struct { double w[4]; } pserve_latency_model;
int  pserve_latency_predict(const pserve_latency_model* model, const pserve_task* batch, int32_t n, int32_t ph,
                            int32_t pw, double* latency);
int  pserve_latency_fit(const double* X, const double* y, int32_t m, pserve_latency_model* model);
int  pserve_slack(const pserve_task* task, double now, double latency, double* slack);
int  pserve_schedule(const pserve_task* wait, int32_t n_wait, const pserve_task* active, int32_t n_active, double now,
                     const pserve_latency_model* model, int32_t ph, int32_t pw, double relaxed_slack,
                     int32_t* admitted, int32_t* n_admitted, int32_t* discarded, int32_t* n_discarded);

/* Kernel selection for measurements and tests: 0 = fastest path available for the
 * shapes (MFMA kernels where they apply; edge stitching pushed by the normalisation pass, the
 * paper's "Patch Edge Stitcher"), 1 = plain reference kernels only (stitching as a separate gather),
 * 2 = as 0 but with the separate gather (the two stitching forms side by side). */
int  pserve_set_kernel_mode(int mode);

/* ---- per-kernel timing for measurements.  While enabled, pserve_block_forward brackets every
 * kernel it launches with a pair of HIP events recorded on the call's stream (no host
 * synchronisation).  pserve_profile_read waits for the recorded events, sums the elapsed time per
 * kernel label, fills up to `max` entries, sets *count to the number of labels and clears the
 * records.  Not thread-safe; meant for benchmarks. */
typedef struct {
    char    name[32];     /* kernel label, e.g. "conv3x3", "gn_stats", "attn_self" */
    int32_t calls;        /* launches recorded */
    float   total_ms;     /* summed device time of those launches */
} pserve_prof_entry;
int  pserve_profile_enable(int on);
/* Restrict the timing to the kernels with this label (NULL or "": all kernels again).  Every event
 * pair costs a few microseconds of stream time, so a throughput measurement that also wants one
 * kernel's duration times only that kernel.  Errors: EINVAL (label of 32 characters or more). */
int  pserve_profile_select(const char* label);
/* Time only every n-th pserve_block_forward call counted from this call (1 = every call): the sampled
 * launches are bracketed exactly as above, the others run without events.  Errors: EINVAL (every < 1). */
int  pserve_profile_sample(int every);
int  pserve_profile_read(pserve_prof_entry* out, int32_t max, int32_t* count);

/* ---- peak probes for measurements (no operation of the paper; they give the roofline figures a second reference
 * beside the datasheet).  All time their own launches with a pair of events on `stream` and wait for them.
 * pserve_probe_mfma_bf16: 512 blocks of four wavefronts, each wavefront issuing 8 * iters independent
 * v_mfma_f32_32x32x16_bf16 on register-resident operands: all 1.0 (random_operands = 0) or standard normals rounded to
 * bf16 (random_operands = 1).  *tflops = dense bf16 rate reached; *mhz (may be NULL) = shader clock inside the timed
 * loop (core cycles per tick of the 100 MHz wall clock).  The chip lowers its clock with the bit activity of the
 * operands, so the second form is the rate a real workload's matrix products can reach.
 * pserve_probe_mfma_mix: the same stream on standard-normal operands with the other instructions of a kernel's inner
 * loop between the MFMAs, everything in registers or LDS (no global memory, no barriers): the rate a kernel with that
 * instruction mix can reach at best on this chip.  `mix` is a sum of 1 (two v_exp_f32 and one v_cvt_pk_bf16_f32 per
 * MFMA: a softmax), 2 (one 16-byte LDS fragment read per two MFMAs), 4 (one v_mfma_f32_4x4x4_16b_bf16 per two MFMAs:
 * row sums on the matrix pipe), 16 (two v_add_f32 per MFMA: row sums on the vector unit), so 19 is the inner loop of the
 * self-attention kernel; or 8 alone (seven fragment reads per ten MFMAs: a 64 x 160 wavefront tile of the convolution /
 * GEMM).  *tflops counts the 32 x 32 x 16 MFMAs only.
 * pserve_probe_copy: a plain 16-byte-per-lane copy of `bytes` bytes from src to dst (DEVICE, 16-byte aligned, not
 * overlapping), `reps` launches; *gbs = (bytes read + bytes written) per second.  A buffer well beyond the 256 MB
 * last-level cache gives the HBM figure; the same launch is the known-size reference for memory counters.
 * Errors: EINVAL, EHIP. */
int  pserve_probe_mfma_bf16(int iters, int random_operands, double* tflops, double* mhz, void* stream);
int  pserve_probe_mfma_mix(int iters, int mix, double* tflops, double* mhz, void* stream);
int  pserve_probe_copy(void* dst, const void* src, size_t bytes, int reps, double* gbs, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* PSERVE_H */
