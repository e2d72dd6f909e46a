// Loss-aware early exit (paper Sec. 4.1, Algorithm "Loss-Aware Pattern Detection"; Sec. 4.2 warmup selection).
// Host code only: a few floating-point operations per adapter per evaluation step.  It lives in this library because its
// decisions drive the segmentation of the next step: an adapter that exits leaves the batch, and the caller builds the
// next plan without it.
#include <cmath>
#include <algorithm>
#include <limits>
#include <numeric>
#include <vector>

#include "common.h"

using mlora::set_error;

namespace {

struct AdapterState {
    bool have_lhat = false;
    double lhat = 0.0;
    std::vector<double> hist_train, hist_val;     // one entry per evaluation step
    int32_t cnt_div = 0, cnt_ovf = 0;
    int32_t status = MLORA_EXIT_CONTINUE;
    double best_val = std::numeric_limits<double>::infinity();
    int32_t best_eval = -1;
};

// least-squares slope over x = 0 .. w-1: sum (x - xbar)(y - ybar) / sum (x - xbar)^2, sums left to right
double linreg_slope(const double* y, int32_t w) {
    if (w < 2) return 0.0;
    const double xbar = (w - 1) / 2.0;
    double ybar = 0.0;
    for (int32_t x = 0; x < w; ++x) ybar += y[x];
    ybar /= w;
    double num = 0.0, den = 0.0;
    for (int32_t x = 0; x < w; ++x) {
        num += (x - xbar) * (y[x] - ybar);
        den += (x - xbar) * (x - xbar);
    }
    return num / den;
}

}  // namespace

struct mlora_monitor {
    mlora_monitor_params p;
    std::vector<AdapterState> a;
};

extern "C" int multi_lora_monitor_create(mlora_monitor** out, int32_t n_adapters, const mlora_monitor_params* params) {
    if (!out || !params) {
        set_error("out / params is NULL");
        return MLORA_ERR_NULL;
    }
    *out = nullptr;
    if (n_adapters < 0 || n_adapters > MLORA_MAX_ADAPTERS) {
        set_error("n_adapters must be in [0, MLORA_MAX_ADAPTERS]");
        return MLORA_ERR_SHAPE;
    }
    const mlora_monitor_params& p = *params;
    if (!(p.ema_alpha > 0.0 && p.ema_alpha <= 1.0) || p.window < 2 || p.patience_div < 1 || p.patience_ovf < 1 ||
        !std::isfinite(p.tau_slope) || !std::isfinite(p.tau_gap)) {
        set_error("monitor parameters: need 0 < ema_alpha <= 1, window >= 2, patience >= 1, finite thresholds");
        return MLORA_ERR_SHAPE;
    }
    mlora_monitor* m = new mlora_monitor();
    m->p = p;
    m->a.resize(n_adapters);
    *out = m;
    return MLORA_OK;
}

extern "C" int multi_lora_monitor_destroy(mlora_monitor* m) {
    delete m;
    return MLORA_OK;
}

static int check_adapter(const mlora_monitor* m, int32_t adapter) {
    if (!m) {
        set_error("monitor is NULL");
        return MLORA_ERR_NULL;
    }
    if (adapter < 0 || adapter >= (int32_t)m->a.size()) {
        set_error("adapter index out of range");
        return MLORA_ERR_SHAPE;
    }
    return MLORA_OK;
}

extern "C" int multi_lora_monitor_train_loss(mlora_monitor* m, int32_t adapter, double loss) {
    const int rc = check_adapter(m, adapter);
    if (rc != MLORA_OK) return rc;
    AdapterState& a = m->a[adapter];
    if (a.status != MLORA_EXIT_CONTINUE) return MLORA_OK;      // already out
    if (!std::isfinite(loss)) {
        // a loss that is no number any more is the end point of the divergence pattern: decided at once (fed into the
        // moving average it would turn every later comparison false and the job would never be caught)
        a.status = MLORA_EXIT_DIVERGING;
        return MLORA_OK;
    }
    a.lhat = a.have_lhat ? m->p.ema_alpha * loss + (1.0 - m->p.ema_alpha) * a.lhat : loss;
    a.have_lhat = true;
    return MLORA_OK;
}

extern "C" int multi_lora_monitor_val_loss(mlora_monitor* m, int32_t adapter, double val_loss, int32_t* decision) {
    const int rc = check_adapter(m, adapter);
    if (rc != MLORA_OK) return rc;
    if (!decision) {
        set_error("decision is NULL");
        return MLORA_ERR_NULL;
    }
    AdapterState& a = m->a[adapter];
    const mlora_monitor_params& p = m->p;
    if (a.status != MLORA_EXIT_CONTINUE) {   // already out: the decision stands
        *decision = a.status;
        return MLORA_OK;
    }
    if (!a.have_lhat) {
        set_error("validation loss reported before any training loss of this adapter");
        return MLORA_ERR_SHAPE;
    }
    if (!std::isfinite(val_loss)) {      // as for the training loss; the histories keep finite values only
        a.status = MLORA_EXIT_DIVERGING;
        *decision = a.status;
        return MLORA_OK;
    }
    a.hist_train.push_back(a.lhat);
    a.hist_val.push_back(val_loss);
    if (val_loss < a.best_val) {
        a.best_val = val_loss;
        a.best_eval = (int32_t)a.hist_val.size() - 1;
    }
    // Pattern 1: both curves trend upward over the last `window` evaluations, for patience_div evaluations in a row
    const int32_t w = p.window;
    if ((int32_t)a.hist_train.size() >= w) {
        const double s_train = linreg_slope(a.hist_train.data() + a.hist_train.size() - w, w);
        const double s_val = linreg_slope(a.hist_val.data() + a.hist_val.size() - w, w);
        a.cnt_div = (s_train >= p.tau_slope && s_val >= p.tau_slope) ? a.cnt_div + 1 : 0;
        if (a.cnt_div >= p.patience_div) {
            a.status = MLORA_EXIT_DIVERGING;
            *decision = a.status;
            return MLORA_OK;
        }
    }
    // Pattern 2: the gap ratio between raw validation loss and smoothed training loss stays above tau_gap
    const double lt = a.hist_train.back();
    const bool exceeded = lt > 0.0 && (val_loss - lt) / lt > p.tau_gap;
    a.cnt_ovf = exceeded ? a.cnt_ovf + 1 : 0;
    if (a.cnt_ovf >= p.patience_ovf) a.status = MLORA_EXIT_OVERFITTING;
    *decision = a.status;
    return MLORA_OK;
}

// ceil(ratio * n), a product within 1e-9 of an integer counting as that integer
static int32_t keep_count(double ratio, int32_t n) {
    const double x = ratio * n;
    const double r = std::nearbyint(x);
    const double k = std::fabs(x - r) <= 1e-9 ? r : std::ceil(x);
    return (int32_t)std::min<double>(std::max<double>(k, 0.0), n);
}

extern "C" int multi_lora_monitor_warmup_select(mlora_monitor* m, double ratio, int32_t* status) {
    if (!m || !status) {
        set_error("monitor / status is NULL");
        return MLORA_ERR_NULL;
    }
    if (!(ratio >= 0.0 && ratio <= 1.0)) {
        set_error("warmup selection ratio must be in [0, 1]");
        return MLORA_ERR_SHAPE;
    }
    std::vector<int32_t> alive;
    for (int32_t i = 0; i < (int32_t)m->a.size(); ++i)
        if (m->a[i].status == MLORA_EXIT_CONTINUE) alive.push_back(i);
    auto key = [&](int32_t i) {
        return m->a[i].hist_val.empty() ? std::numeric_limits<double>::infinity() : m->a[i].hist_val.back();
    };
    std::stable_sort(alive.begin(), alive.end(), [&](int32_t x, int32_t y) { return key(x) < key(y); });
    const int32_t k = keep_count(ratio, (int32_t)alive.size());
    for (size_t j = (size_t)k; j < alive.size(); ++j) m->a[alive[j]].status = MLORA_EXIT_UNDERPERFORMING;
    for (size_t i = 0; i < m->a.size(); ++i) status[i] = m->a[i].status;
    return MLORA_OK;
}

extern "C" int multi_lora_monitor_state(const mlora_monitor* m, int32_t adapter, mlora_monitor_state* out) {
    const int rc = check_adapter(m, adapter);
    if (rc != MLORA_OK) return rc;
    if (!out) {
        set_error("out is NULL");
        return MLORA_ERR_NULL;
    }
    const AdapterState& a = m->a[adapter];
    out->ema_train_loss = a.have_lhat ? a.lhat : std::numeric_limits<double>::quiet_NaN();
    out->best_val_loss = a.best_val;
    out->best_eval_step = a.best_eval;
    out->evaluations = (int32_t)a.hist_val.size();
    out->count_diverging = a.cnt_div;
    out->count_overfitting = a.cnt_ovf;
    out->status = a.status;
    return MLORA_OK;
}
