// Host-side scheduler pieces (section "SLO-Aware Scheduler"): slack score, a linear latency model in place of the
// paper's MLP (fitted on this machine's own measurements), and the scheduling loop of the paper's algorithm.  No GPU
// work: plain C++ behind the C ABI, all pointers HOST.
#include "common.h"

#include <cmath>
#include <set>
#include <utility>

using namespace pserve;

namespace {

struct Feat { double patches, resolutions, attn; };

// batch = active[0 .. na) plus, if extra != nullptr, *extra
Feat features(const pserve_task* active, int na, const pserve_task* extra, int ph, int pw) {
    Feat f{0.0, 0.0, 0.0};
    std::set<std::pair<int32_t, int32_t>> res;
    auto add = [&](const pserve_task& t) {
        f.patches += (double)((t.H / ph) * (t.W / pw));
        res.insert({t.H, t.W});
        const double tok = (double)t.H * (double)t.W;
        f.attn += tok * tok;
    };
    for (int i = 0; i < na; ++i) add(active[i]);
    if (extra) add(*extra);
    f.resolutions = (double)res.size();
    f.attn *= 1e-6;
    return f;
}

double predict(const pserve_latency_model& m, const pserve_task* active, int na, const pserve_task* extra, int ph, int pw) {
    const Feat f = features(active, na, extra, ph, pw);
    return m.w[0] + m.w[1] * f.patches + m.w[2] * f.resolutions + m.w[3] * f.attn;
}

double slack_of(const pserve_task& t, double now, double latency) {
    return (t.ddl - (now - t.arrival) - (double)t.steps_left * latency) / t.standalone;
}

bool time_out(const pserve_task& t, double now, double latency) {
    return now + (double)t.steps_left * latency > t.arrival + t.ddl;
}

int check_tasks(const pserve_task* t, int n, int ph, int pw, const char* who) {
    for (int i = 0; i < n; ++i) {
        PS_REQUIRE(t[i].H > 0 && t[i].W > 0 && t[i].H % ph == 0 && t[i].W % pw == 0,
                   "%s: task %d has resolution %dx%d, not a positive multiple of the %dx%d patch", who, i, t[i].H, t[i].W, ph, pw);
        PS_REQUIRE(t[i].steps_left >= 0 && t[i].standalone > 0.0, "%s: task %d needs steps_left >= 0 and standalone > 0", who, i);
    }
    return PSERVE_OK;
}

}  // namespace

extern "C" {

int pserve_latency_predict(const pserve_latency_model* model, const pserve_task* batch, int32_t n, int32_t ph, int32_t pw,
                           double* latency) {
    PS_REQUIRE(model && latency && (batch || n == 0) && n >= 0 && ph > 0 && pw > 0, "pserve_latency_predict: bad argument");
    PS_TRY(check_tasks(batch, n, ph, pw, "pserve_latency_predict"));
    *latency = predict(*model, batch, n, nullptr, ph, pw);
    return PSERVE_OK;
}

static int latency_fit_impl(const double* X, const double* y, int32_t m, pserve_latency_model* model) {
    PS_REQUIRE(X && y && model && m >= 4, "pserve_latency_fit: needs at least 4 samples");
    // normal equations of y ~ [1, X] (4 unknowns), solved by Gaussian elimination with partial pivoting
    double A[4][5] = {};
    for (int s = 0; s < m; ++s) {
        const double r[4] = {1.0, X[3 * s], X[3 * s + 1], X[3 * s + 2]};
        for (int i = 0; i < 4; ++i) {
            for (int j = 0; j < 4; ++j) A[i][j] += r[i] * r[j];
            A[i][4] += r[i] * y[s];
        }
    }
    for (int c = 0; c < 4; ++c) {
        int piv = c;
        for (int r = c + 1; r < 4; ++r) if (std::fabs(A[r][c]) > std::fabs(A[piv][c])) piv = r;
        PS_REQUIRE(std::fabs(A[piv][c]) > 1e-12 * (1.0 + std::fabs(A[0][0])), "pserve_latency_fit: the samples do not determine the model (rank deficient)");
        if (piv != c) for (int j = 0; j < 5; ++j) std::swap(A[piv][j], A[c][j]);
        for (int r = c + 1; r < 4; ++r) {
            const double f = A[r][c] / A[c][c];
            for (int j = c; j < 5; ++j) A[r][j] -= f * A[c][j];
        }
    }
    for (int c = 3; c >= 0; --c) {
        double v = A[c][4];
        for (int j = c + 1; j < 4; ++j) v -= A[c][j] * model->w[j];
        model->w[c] = v / A[c][c];
    }
    return PSERVE_OK;
}

int pserve_latency_fit(const double* X, const double* y, int32_t m, pserve_latency_model* model) {
    return guarded("pserve_latency_fit", [&] { return latency_fit_impl(X, y, m, model); });
}

int pserve_slack(const pserve_task* task, double now, double latency, double* slack) {
    PS_REQUIRE(task && slack && task->standalone > 0.0, "pserve_slack: bad argument");
    *slack = slack_of(*task, now, latency);
    return PSERVE_OK;
}

static int schedule_impl(const pserve_task* wait, int32_t n_wait, const pserve_task* active, int32_t n_active, double now,
                    const pserve_latency_model* model, int32_t ph, int32_t pw, double relaxed_slack,
                    int32_t* admitted, int32_t* n_admitted, int32_t* discarded, int32_t* n_discarded) {
    PS_REQUIRE(model && admitted && n_admitted && discarded && n_discarded && n_wait >= 0 && n_active >= 0 &&
               (wait || n_wait == 0) && (active || n_active == 0) && ph > 0 && pw > 0, "pserve_schedule: bad argument");
    PS_TRY(check_tasks(wait, n_wait, ph, pw, "pserve_schedule"));
    PS_TRY(check_tasks(active, n_active, ph, pw, "pserve_schedule"));
    std::vector<pserve_task> act(active, active + n_active);
    std::vector<int> waiting(n_wait);
    for (int i = 0; i < n_wait; ++i) waiting[i] = i;
    int na = 0, nd = 0;
    auto drop = [&](int idx) { waiting.erase(std::find(waiting.begin(), waiting.end(), idx)); };
    while (!waiting.empty()) {
        const int n_act = (int)act.size();
        const double lat_now = n_act ? predict(*model, act.data(), n_act, nullptr, ph, pw) : 0.0;
        // least-slack waiting task, scored with the latency of the batch it would join (ties: queue order)
        int cur = -1;
        double cur_s = 0.0;
        for (int i : waiting) {
            const double s = slack_of(wait[i], now, predict(*model, act.data(), n_act, &wait[i], ph, pw));
            if (cur < 0 || s < cur_s) { cur = i; cur_s = s; }
        }
        int act_task = -1;
        double act_s = 0.0;
        for (int k = 0; k < n_act; ++k) {
            const double s = slack_of(act[k], now, lat_now);
            if (act_task < 0 || s < act_s) { act_task = k; act_s = s; }
        }
        double pred = predict(*model, act.data(), n_act, &wait[cur], ph, pw);
        if (time_out(wait[cur], now, pred)) {       // cannot meet its deadline even if run now
            discarded[nd++] = cur;
            drop(cur);
            continue;
        }
        if (cur_s > relaxed_slack) {                // throughput mode: most batch tokens per predicted millisecond
            double tok_act = 0.0;
            for (const pserve_task& t : act) tok_act += (double)(t.H * t.W);
            int top = -1;
            double top_v = 0.0;
            for (int i : waiting) {
                const double lat_i = predict(*model, act.data(), n_act, &wait[i], ph, pw);
                if (time_out(wait[i], now, lat_i)) continue;
                const double v = (tok_act + (double)(wait[i].H * wait[i].W)) / lat_i;
                if (top < 0 || v > top_v) { top = i; top_v = v; }
            }
            cur = top;                              // the first candidate itself qualifies, so top >= 0
            pred = predict(*model, act.data(), n_act, &wait[cur], ph, pw);
        }
        if (act_task >= 0 && time_out(act[act_task], now, pred)) break;    // the most urgent running task would be late
        admitted[na++] = cur;
        drop(cur);
        act.push_back(wait[cur]);
    }
    *n_admitted = na;
    *n_discarded = nd;
    return PSERVE_OK;
}

int pserve_schedule(const pserve_task* wait, int32_t n_wait, const pserve_task* active, int32_t n_active, double now,
                    const pserve_latency_model* model, int32_t ph, int32_t pw, double relaxed_slack,
                    int32_t* admitted, int32_t* n_admitted, int32_t* discarded, int32_t* n_discarded) {
    return guarded("pserve_schedule", [&] { return schedule_impl(wait, n_wait, active, n_active, now, model, ph, pw, relaxed_slack, admitted, n_admitted, discarded, n_discarded); });
}

}  // extern "C"
