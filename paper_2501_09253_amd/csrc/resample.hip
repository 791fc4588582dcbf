// Resolution changes between two levels on the patch batch: stride-2 3x3 convolution (DOWN2) and nearest-neighbour
// 2x followed by a 3x3 convolution (UP2).  Both keep the patch grid (a ph x pw patch becomes ph/2 x pw/2 resp.
// 2ph x 2pw), so the output plan is the plan of the halved / doubled resolutions with the halved / doubled patch and
// has the same patch order, owners and neighbours.
//   1. the input is copied into the padded patch layout and its rims are pushed to the neighbours (the apply pass
//      of the GroupNorm without a scale table: the "Patch Edge Stitcher" of the paper as a plain copy);
//   2. DOWN2: one implicit GEMM whose rows are OUTPUT tokens (p, y, x) reading the padded pixels (2y + ty, 2x + tx);
//      UP2:   four implicit GEMMs, one per output parity (a, b), whose rows are INPUT tokens (p, y, x): the nine taps
//             of output pixel (2y + a, 2x + b) fall on 2 x 2 input pixels, so the weights are merged into four taps per
//             class when the operator is created (4/9 of the multiply-adds of the plain form).
#include "kernels.h"

using namespace pserve;

struct pserve_resample_s {
    int kind = 0, dtype = 0;
    int32_t C_in = 0, C_out = 0;
    void* w = nullptr;          // DOWN2: [9][C_out][C_in]; UP2: [4 classes][4 taps][C_out][C_in]
    float* b = nullptr;
    DevicePool pool;
};

static int check_pair(const pserve_resample_t* op, const pserve_plan_t* in, const pserve_plan_t* out, const char* who) {
    PS_REQUIRE(op && in && out, "%s: NULL argument", who);
    const int num = op->kind == PSERVE_DOWN2 ? 1 : 2, den = op->kind == PSERVE_DOWN2 ? 2 : 1;   // out = in * num / den
    PS_REQUIRE(in->P == out->P && in->n == out->n, "%s: the two plans have different patch grids (%d / %d patches)", who, in->P, out->P);
    PS_REQUIRE(in->ph * num == out->ph * den && in->pw * num == out->pw * den,
               "%s: patch %dx%d does not go to %dx%d", who, in->ph, in->pw, out->ph, out->pw);
    for (int s = 0; s < in->n; ++s)
        PS_REQUIRE(in->h_sorted_hw[2 * s] * num == out->h_sorted_hw[2 * s] * den &&
                   in->h_sorted_hw[2 * s + 1] * num == out->h_sorted_hw[2 * s + 1] * den &&
                   in->h_tab[PSERVE_TAB_PERM][s] == out->h_tab[PSERVE_TAB_PERM][s],
                   "%s: request slot %d of the output plan is not the resampled request of the input plan", who, s);
    return PSERVE_OK;
}

extern "C" {

static int resample_create_impl(int kind, int32_t C_in, int32_t C_out, int dtype, const void* w, const void* b, void* stream,
                           pserve_resample_t** out) {
    PS_REQUIRE(out, "pserve_resample_create: out is NULL");
    *out = nullptr;
    PS_REQUIRE(kind == PSERVE_DOWN2 || kind == PSERVE_UP2, "pserve_resample_create: unknown kind %d", kind);
    PS_REQUIRE(dtype == PSERVE_F32 || dtype == PSERVE_BF16, "pserve_resample_create: unknown dtype %d", dtype);
    PS_REQUIRE(w && b && C_in > 0 && C_out > 0, "pserve_resample_create: NULL parameter or non-positive width");
    const int vn = dtype == PSERVE_BF16 ? 8 : 4;
    PS_REQUIRE(C_in % vn == 0 && C_out % vn == 0, "pserve_resample_create: C_in=%d and C_out=%d must be multiples of 16 bytes", C_in, C_out);
    pserve_resample_t* r = new (std::nothrow) pserve_resample_t();
    if (!r) { set_error("pserve_resample_create: out of host memory"); return PSERVE_ENOMEM; }
    struct Guard { pserve_resample_t* p; ~Guard() { delete p; } } guard{r};
    r->kind = kind; r->dtype = dtype; r->C_in = C_in; r->C_out = C_out;
    hipStream_t st = (hipStream_t)stream;
    const size_t es = dtype_size(dtype);
    if (kind == PSERVE_DOWN2) {
        PS_TRY(r->pool.alloc(&r->w, es * 9 * C_out * C_in));
        PS_TRY(pack_conv(w, r->w, C_out, C_in, dtype, st));
    } else {
        PS_TRY(r->pool.alloc(&r->w, es * 16 * C_out * C_in));
        PS_TRY(pack_conv_up2(w, r->w, C_out, C_in, dtype, st));
    }
    PS_TRY(r->pool.alloc_t(&r->b, C_out));
    PS_TRY(pack_bias(b, r->b, C_out, dtype, st));
    PS_CHECK_HIP(hipStreamSynchronize(st));
    guard.p = nullptr;
    *out = r;
    return PSERVE_OK;
}

int pserve_resample_create(int kind, int32_t C_in, int32_t C_out, int dtype, const void* w, const void* b, void* stream,
                           pserve_resample_t** out) {
    return guarded("pserve_resample_create", [&] { return resample_create_impl(kind, C_in, C_out, dtype, w, b, stream, out); });
}

void pserve_resample_free(pserve_resample_t* op) { delete op; }

int pserve_resample_workspace(const pserve_resample_t* op, const pserve_plan_t* plan_in, size_t* bytes) {
    PS_REQUIRE(op && plan_in && bytes, "pserve_resample_workspace: NULL argument");
    *bytes = (size_t)plan_in->P * (plan_in->ph + 2) * (plan_in->pw + 2) * op->C_in * dtype_size(op->dtype);
    return PSERVE_OK;
}

int pserve_resample_forward(const pserve_resample_t* op, const pserve_plan_t* plan_in, const pserve_plan_t* plan_out,
                            const void* x, void* workspace, size_t workspace_bytes, void* y, void* stream) {
    PS_TRY(check_pair(op, plan_in, plan_out, "pserve_resample_forward"));
    PS_REQUIRE(x && y && workspace, "pserve_resample_forward: NULL buffer");
    PS_REQUIRE(op->kind != PSERVE_DOWN2 || (plan_in->ph % 2 == 0 && plan_in->pw % 2 == 0),
               "pserve_resample_forward: DOWN2 needs an even patch size (got %dx%d)", plan_in->ph, plan_in->pw);
    size_t need = 0;
    PS_TRY(pserve_resample_workspace(op, plan_in, &need));
    PS_REQUIRE(workspace_bytes >= need, "pserve_resample_forward: workspace of %zu bytes, %zu needed", workspace_bytes, need);
    hipStream_t st = (hipStream_t)stream;
    const int dt = op->dtype;
    PatchGeom gin;
    gin.P = plan_in->P; gin.S = plan_in->S; gin.ph = plan_in->ph; gin.pw = plan_in->pw;
    gin.ppw = plan_in->pw + 2; gin.pS = (plan_in->ph + 2) * (plan_in->pw + 2);
    const ActiveList all{nullptr, nullptr};
    {   // padded copy with the rims of the neighbours (and zeros at the image border)
        GroupNormArgs ga{};
        ga.x = x; ga.C = op->C_in; ga.G = 1; ga.n = plan_in->n; ga.nsplit = 1;
        ga.scale_shift = nullptr;
        ga.owner = plan_in->d_tab[PSERVE_TAB_PATCH_OWNER];
        ga.neighbour = plan_in->d_tab[PSERVE_TAB_NEIGHBOUR];
        ga.request_offset = plan_in->d_tab[PSERVE_TAB_REQUEST_OFFSET];
        PS_TRY(gn_apply(ga, gin, dt, /*silu=*/false, /*padded=*/true, /*stitch=*/true, workspace, all, st));
    }
    GemmArgs g{};
    g.A = workspace; g.lda = op->C_in; g.conv = 1; g.act = all; g.tokens_are_rows = 1;
    g.N = op->C_out; g.K = op->C_in; g.bias = op->b; g.epi = EPI_ROUTE; g.seg_cols = op->C_out;
    for (auto& s : g.seg) { s.ptr = nullptr; s.ld = 0; s.transposed = 0; s.scale = 1.f; }
    g.seg[0].ptr = y; g.seg[0].ld = op->C_out;
    g.geom = gin;
    if (op->kind == PSERVE_DOWN2) {
        g.geom.S = plan_out->S; g.geom.pw = plan_out->pw; g.geom.ph = plan_out->ph;     // rows: output tokens
        g.M = (int32_t)plan_out->T; g.taps = 9; g.tap_w = 3; g.a_mul = 2; g.B = op->w;
        return gemm(g, dt, 0, st);
    }
    const size_t es = dtype_size(dt);
    g.M = (int32_t)plan_in->T; g.taps = 4; g.tap_w = 2; g.a_mul = 1;                     // rows: input tokens
    g.o_mul = 2; g.o_S = plan_out->S; g.o_pw = plan_out->pw;
    for (int cls = 0; cls < 4; ++cls) {
        g.a_dy = g.o_dy = cls >> 1;
        g.a_dx = g.o_dx = cls & 1;
        g.B = (const char*)op->w + (size_t)cls * 4 * op->C_out * op->C_in * es;
        PS_TRY(gemm(g, dt, 0, st));
    }
    return PSERVE_OK;
}

}  // extern "C"
