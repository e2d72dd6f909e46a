// Online greedy intra-task scheduling (paper Sec. 6.1; App. "Intra-Task Scheduling Details"): the fitted memory model
// Mhat(B) = k0 + k1 B L, greedy admission in decreasing per-adapter batch size, backfill that prefers the batch size
// of the job that left.  Host code only.  The running set it reports, in admission order, is the adapter order of the
// next step's batch: the caller turns it into segment offsets and builds that step's plan.
#include <algorithm>
#include <cmath>
#include <vector>

#include "common.h"

using mlora::set_error;

extern "C" int multi_lora_memory_model_fit(int32_t n_points, const double* batch_times_seq, const double* peak_bytes,
                                           double* k0, double* k1) {
    if (!batch_times_seq || !peak_bytes || !k0 || !k1) {
        set_error("memory model fit: NULL argument");
        return MLORA_ERR_NULL;
    }
    if (n_points < 1) {
        set_error("memory model fit needs at least one profiled point");
        return MLORA_ERR_SHAPE;
    }
    // least squares, sums left to right: k1 = sum (x - xbar)(y - ybar) / sum (x - xbar)^2, k0 = ybar - k1 xbar
    double xbar = 0.0, ybar = 0.0;
    for (int32_t i = 0; i < n_points; ++i) {
        xbar += batch_times_seq[i];
        ybar += peak_bytes[i];
    }
    xbar /= n_points;
    ybar /= n_points;
    double num = 0.0, den = 0.0;
    for (int32_t i = 0; i < n_points; ++i) {
        num += (batch_times_seq[i] - xbar) * (peak_bytes[i] - ybar);
        den += (batch_times_seq[i] - xbar) * (batch_times_seq[i] - xbar);
    }
    *k1 = den > 0.0 ? num / den : 0.0;
    *k0 = ybar - *k1 * xbar;
    return MLORA_OK;
}

struct mlora_admission {
    mlora_admission_params p;
    struct Job { int32_t id, batch; };
    std::vector<Job> pending;   // submission order
    std::vector<Job> running;   // admission order
    int64_t total_batch = 0;

    bool fits(int32_t b) const {
        return p.k0 + p.k1 * (double)(total_batch + b) * (double)p.seq_len <= p.safety_margin * p.capacity_bytes;
    }
    void admit(size_t pending_index, std::vector<int32_t>& out) {
        const Job j = pending[pending_index];
        pending.erase(pending.begin() + (std::ptrdiff_t)pending_index);
        running.push_back(j);
        total_batch += j.batch;
        out.push_back(j.id);
    }
    // greedy pass: decreasing batch size, submission order within a size; a job that does not fit is skipped
    void fill(std::vector<int32_t>& out) {
        std::vector<Job> order = pending;
        std::stable_sort(order.begin(), order.end(), [](const Job& a, const Job& b) { return a.batch > b.batch; });
        for (const Job& j : order) {
            if (!fits(j.batch)) continue;
            for (size_t i = 0; i < pending.size(); ++i)
                if (pending[i].id == j.id) {
                    admit(i, out);
                    break;
                }
        }
    }
};

static int copy_out(const std::vector<int32_t>& v, int32_t* dst, int32_t cap, int32_t* count) {
    if (count) *count = (int32_t)v.size();
    if ((int32_t)v.size() > cap || (!dst && !v.empty())) {
        set_error("output array too small for the admitted jobs (the scheduler state has been updated; see *count)");
        return MLORA_ERR_SHAPE;
    }
    for (size_t i = 0; i < v.size(); ++i) dst[i] = v[i];
    return MLORA_OK;
}

extern "C" int multi_lora_admission_create(mlora_admission** out, const mlora_admission_params* params) {
    if (!out || !params) {
        set_error("out / params is NULL");
        return MLORA_ERR_NULL;
    }
    *out = nullptr;
    const mlora_admission_params& p = *params;
    if (!std::isfinite(p.k0) || !std::isfinite(p.k1) || !(p.capacity_bytes > 0.0) || !(p.safety_margin > 0.0 && p.safety_margin <= 1.0) ||
        p.seq_len < 1) {
        set_error("admission parameters: finite k0, k1; capacity > 0; 0 < safety_margin <= 1; seq_len >= 1");
        return MLORA_ERR_SHAPE;
    }
    mlora_admission* a = new mlora_admission();
    a->p = p;
    *out = a;
    return MLORA_OK;
}

extern "C" int multi_lora_admission_destroy(mlora_admission* a) {
    delete a;
    return MLORA_OK;
}

extern "C" int multi_lora_admission_submit(mlora_admission* a, int32_t job_id, int32_t batch_size) {
    if (!a) {
        set_error("scheduler is NULL");
        return MLORA_ERR_NULL;
    }
    if (batch_size < 1) {
        set_error("batch_size must be >= 1");
        return MLORA_ERR_SHAPE;
    }
    for (const auto& j : a->pending)
        if (j.id == job_id) { set_error("job id already pending"); return MLORA_ERR_SHAPE; }
    for (const auto& j : a->running)
        if (j.id == job_id) { set_error("job id already running"); return MLORA_ERR_SHAPE; }
    a->pending.push_back({job_id, batch_size});
    return MLORA_OK;
}

extern "C" int multi_lora_admission_fill(mlora_admission* a, int32_t* admitted, int32_t cap, int32_t* count) {
    if (!a) {
        set_error("scheduler is NULL");
        return MLORA_ERR_NULL;
    }
    std::vector<int32_t> out;
    a->fill(out);
    return copy_out(out, admitted, cap, count);
}

extern "C" int multi_lora_admission_exit(mlora_admission* a, int32_t job_id, int32_t* admitted, int32_t cap, int32_t* count) {
    if (!a) {
        set_error("scheduler is NULL");
        return MLORA_ERR_NULL;
    }
    size_t at = a->running.size();
    for (size_t i = 0; i < a->running.size(); ++i)
        if (a->running[i].id == job_id) at = i;
    if (at == a->running.size()) {
        set_error("job is not running");
        return MLORA_ERR_SHAPE;
    }
    const int32_t b = a->running[at].batch;
    a->total_batch -= b;
    a->running.erase(a->running.begin() + (std::ptrdiff_t)at);
    std::vector<int32_t> out;
    // the vacated slot goes to the oldest pending job of the same batch size, if there is one and it fits
    for (size_t i = 0; i < a->pending.size(); ++i)
        if (a->pending[i].batch == b) {
            if (a->fits(b)) a->admit(i, out);
            break;
        }
    a->fill(out);
    return copy_out(out, admitted, cap, count);
}

extern "C" int multi_lora_admission_running(const mlora_admission* a, int32_t* job_ids, int32_t* batch_sizes, int32_t cap,
                                            int32_t* count) {
    if (!a || !count) {
        set_error("scheduler / count is NULL");
        return MLORA_ERR_NULL;
    }
    *count = (int32_t)a->running.size();
    if (*count > cap) {
        set_error("output arrays too small for the running set");
        return MLORA_ERR_SHAPE;
    }
    for (size_t i = 0; i < a->running.size(); ++i) {
        if (job_ids) job_ids[i] = a->running[i].id;
        if (batch_sizes) batch_sizes[i] = a->running[i].batch;
    }
    return MLORA_OK;
}
