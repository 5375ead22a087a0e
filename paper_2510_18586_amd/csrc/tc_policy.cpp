// Host-side scheduling arithmetic that consumes the copy path's measurements: the linear
// transfer-cost model (paper Eq. 2), the ShouldOffload gate (Alg. 1), the upload budget (Eq. 3),
// the gradual reservation (Eq. 4), the hard rejections ahead of the offload score (Sec. 4.2), one
// scheduling step of predictive upload (Sec. 4.3), the five-state request lifecycle (Sec. 6.2) and the call-duration
// forecast (Eq. 1).  No GPU work here; tc_calibrate lives in the engine.
#include <algorithm>
#include <cmath>
#include <mutex>
#include <new>
#include <unordered_map>

#include "tokencake_kv.h"

namespace {

// least squares of t = a + b*n; false when the sizes do not span a line
bool fit_line(const uint32_t *n, const double *t, uint32_t m, double *a, double *b)
{
    long double sn = 0, st = 0;
    for (uint32_t i = 0; i < m; ++i) {
        sn += n[i];
        st += t[i];
    }
    const long double mn = sn / m, mt = st / m;
    long double sxx = 0, sxy = 0;
    for (uint32_t i = 0; i < m; ++i) {
        const long double dx = n[i] - mn;
        sxx += dx * dx;
        sxy += dx * (t[i] - mt);
    }
    if (sxx == 0) return false;
    *b = double(sxy / sxx);
    *a = double(mt - (sxy / sxx) * mn);
    return true;
}

}  // namespace

// No exception crosses the C boundary: running out of host memory inside a container is reported,
// anything else unexpected is an invalid call.
#define TC_CATCH_ALL                                              \
    catch (const std::bad_alloc &) { return TC_ERR_HOST_NOMEM; } \
    catch (...) { return TC_ERR_INVAL; }

extern "C" {

int tc_cost_fit(const uint32_t *n_blocks, const double *offload_ms, const double *upload_ms, uint32_t m,
                tc_cost_model *out)
try {
    if (!n_blocks || !offload_ms || !upload_ms || !out || m < 2) return TC_ERR_INVAL;
    tc_cost_model r;
    if (!fit_line(n_blocks, offload_ms, m, &r.off_a_ms, &r.off_b_ms_per_block)) return TC_ERR_INVAL;
    if (!fit_line(n_blocks, upload_ms, m, &r.up_a_ms, &r.up_b_ms_per_block)) return TC_ERR_INVAL;
    *out = r;
    return TC_OK;
} TC_CATCH_ALL

double tc_estimate_transfer_ms(const tc_cost_model *model, uint32_t n_blocks)
{
    if (!model) return std::nan("");
    const double t_offload = model->off_a_ms + model->off_b_ms_per_block * n_blocks;
    const double t_upload = model->up_a_ms + model->up_b_ms_per_block * n_blocks;
    return t_offload + t_upload;
}

int tc_should_offload(const tc_cost_model *model, uint32_t req_blocks, double t_fc_ms,
                      double v_throughput_tokens_per_ms, const tc_waiting_req *queue, uint32_t n_queue,
                      int32_t *chosen)
try {
    if (!model || (n_queue && !queue)) return TC_ERR_INVAL;
    if (chosen) *chosen = -1;
    const double t_transfer = tc_estimate_transfer_ms(model, req_blocks);
    if (t_fc_ms <= t_transfer) return 0;  // the stall does not even cover the round trip
    const double n_capacity = (t_fc_ms - t_transfer) * v_throughput_tokens_per_ms;
    for (uint32_t k = 0; k < n_queue; ++k) {
        if (queue[k].kv_blocks <= req_blocks && queue[k].work_tokens <= n_capacity) {
            if (chosen) *chosen = int32_t(k);
            return 1;
        }
    }
    return 0;
} TC_CATCH_ALL

uint32_t tc_upload_budget(uint32_t gpu_free, uint32_t d_critical, uint32_t shared_free)
{
    const uint32_t held_back = d_critical > shared_free ? d_critical - shared_free : 0;
    return gpu_free > held_back ? gpu_free - held_back : 0;
}

uint32_t tc_gradual_reserve(uint32_t remain, uint32_t deficit, uint32_t budget)
{
    uint32_t r = deficit / 2 + (deficit & 1u);
    if (remain < r) r = remain;
    if (budget < r) r = budget;
    return r;
}

int tc_offload_gate(const tc_cost_model *model, const tc_gate_input *in, const tc_waiting_req *queue,
                    uint32_t n_queue, int32_t *chosen, int *reason)
try {
    if (!model || !in || !reason || (n_queue && !queue) || in->gpu_total_blocks == 0) return TC_ERR_INVAL;
    if (std::isnan(in->pressure_threshold) || std::isnan(in->t_fc_ms) || std::isnan(in->v_throughput_tokens_per_ms))
        return TC_ERR_INVAL;
    if (chosen) *chosen = -1;
    // the four hard rejections, tested in the order Sec. 4.2 lists them
    if (in->cpu_free_blocks < in->req_blocks) {
        *reason = TC_GATE_CPU_FULL;
        return 0;
    }
    if (in->t_fc_ms <= tc_estimate_transfer_ms(model, in->req_blocks)) {
        *reason = TC_GATE_STALL_SHORT;
        return 0;
    }
    int32_t k = -1;
    if (tc_should_offload(model, in->req_blocks, in->t_fc_ms, in->v_throughput_tokens_per_ms, queue, n_queue, &k) != 1) {
        *reason = TC_GATE_NO_FIT;
        return 0;
    }
    if (double(in->gpu_used_blocks) / double(in->gpu_total_blocks) < in->pressure_threshold) {
        *reason = TC_GATE_LOW_PRESSURE;
        return 0;
    }
    *reason = TC_GATE_PASS;
    if (chosen) *chosen = k;
    return 1;
} TC_CATCH_ALL

int tc_upload_plan(const tc_upload_cand *cands, uint32_t n, uint32_t gpu_free, uint32_t d_critical,
                   uint32_t shared_free, uint32_t *order, uint32_t *reserve)
try {
    if (n && (!cands || !order || !reserve)) return TC_ERR_INVAL;
    for (uint32_t i = 0; i < n; ++i)
        if (std::isnan(cands[i].importance) || std::isnan(cands[i].urgency)) return TC_ERR_INVAL;
    for (uint32_t i = 0; i < n; ++i) order[i] = i;
    // falling P_upload = I + U; equal P: the more urgent first, then the one named first
    std::sort(order, order + n, [cands](uint32_t a, uint32_t b) {
        const double pa = cands[a].importance + cands[a].urgency, pb = cands[b].importance + cands[b].urgency;
        if (pa != pb) return pa > pb;
        if (cands[a].urgency != cands[b].urgency) return cands[a].urgency > cands[b].urgency;
        return a < b;
    });
    const uint32_t budget = tc_upload_budget(gpu_free, d_critical, shared_free);
    uint32_t remain = budget;
    for (uint32_t r = 0; r < n; ++r) {
        const uint32_t i = order[r];
        reserve[i] = tc_gradual_reserve(remain, cands[i].deficit, budget);
        remain -= reserve[i];
    }
    return TC_OK;
} TC_CATCH_ALL

int tc_lifecycle_step(tc_req_state *req, int event, int *action)
try {
    if (!req || req->state > TC_UPLOADED) return TC_ERR_INVAL;
    tc_req_state r = *req;
    int act = TC_ACT_NONE;
    bool ok = false;
    const bool fin = r.finish_seen != 0, fly = r.copy_in_flight != 0;
    switch (event) {
    case TC_EV_CALL_START:
        if (r.state == TC_RUNNING && !fin && !fly) {
            r.state = TC_PENDING_OFFLOAD;
            ok = true;
        }
        break;
    case TC_EV_OFFLOAD_ISSUED:
        if (r.state == TC_PENDING_OFFLOAD && !fin && !fly) {
            r.copy_in_flight = 1;
            ok = true;
        }
        break;
    case TC_EV_OFFLOAD_DONE:
        if (r.state == TC_PENDING_OFFLOAD && fly) {
            r.state = TC_OFFLOADED;
            r.copy_in_flight = 0;
            if (fin) act = TC_ACT_UPLOAD_NOW;  // the tool came back while the copy ran
            ok = true;
        }
        break;
    case TC_EV_UPLOAD_ISSUED:
        if (r.state == TC_OFFLOADED) {
            r.state = TC_PENDING_UPLOAD;
            r.copy_in_flight = 1;
            ok = true;
        }
        break;
    case TC_EV_UPLOAD_DONE:
        if (r.state == TC_PENDING_UPLOAD && fly) {
            r.copy_in_flight = 0;
            if (fin) {
                r.state = TC_RUNNING;
                r.finish_seen = 0;
                act = TC_ACT_RESUME;
            } else {
                r.state = TC_UPLOADED;
            }
            ok = true;
        }
        break;
    case TC_EV_CALL_FINISH:
        if (fin) break;
        if (r.state == TC_UPLOADED) {
            r.state = TC_RUNNING;
            r.copy_in_flight = 0;
            act = TC_ACT_RESUME;
            ok = true;
        } else if (r.state == TC_OFFLOADED) {
            r.finish_seen = 1;
            r.copy_in_flight = 0;
            act = TC_ACT_UPLOAD_NOW;
            ok = true;
        } else if (r.state == TC_PENDING_UPLOAD) {
            r.finish_seen = 1;
            act = TC_ACT_WAIT;
            ok = true;
        } else if (r.state == TC_PENDING_OFFLOAD) {
            if (fly) {
                r.finish_seen = 1;
                act = TC_ACT_WAIT;
            } else {
                r.state = TC_RUNNING;  // the KV never left the GPU
                act = TC_ACT_RESUME;
            }
            ok = true;
        }
        break;
    default: break;
    }
    if (!ok) return TC_ERR_INVAL;
    *req = r;
    if (action) *action = act;
    return TC_OK;
} TC_CATCH_ALL

}  // extern "C"

struct tc_forecaster {
    double alpha, gamma, default_ms;
    mutable std::mutex mu;
    std::unordered_map<uint32_t, double> history;
};

extern "C" {

int tc_forecaster_create(double alpha, double gamma, double default_ms, tc_forecaster **out)
try {
    if (!out) return TC_ERR_INVAL;
    *out = nullptr;
    if (!(alpha >= 0.0 && alpha <= 1.0) || !(gamma > 0.0 && gamma <= 1.0) || !(default_ms >= 0.0)) return TC_ERR_INVAL;
    tc_forecaster *f = new (std::nothrow) tc_forecaster;
    if (!f) return TC_ERR_INVAL;
    f->alpha = alpha;
    f->gamma = gamma;
    f->default_ms = default_ms;
    *out = f;
    return TC_OK;
} TC_CATCH_ALL

int tc_forecaster_destroy(tc_forecaster *f)
{
    delete f;
    return TC_OK;
}

int tc_forecaster_observe(tc_forecaster *f, uint32_t fn_type, double elapsed_ms)
try {
    if (!f || !(elapsed_ms >= 0.0)) return TC_ERR_INVAL;
    std::lock_guard<std::mutex> g(f->mu);
    auto it = f->history.find(fn_type);
    if (it == f->history.end()) f->history.emplace(fn_type, elapsed_ms);
    else it->second = f->gamma * elapsed_ms + (1.0 - f->gamma) * it->second;
    return TC_OK;
} TC_CATCH_ALL

double tc_forecaster_estimate(const tc_forecaster *f, uint32_t fn_type, int has_user, double t_user_ms)
{
    if (!f) return std::nan("");
    std::lock_guard<std::mutex> g(f->mu);
    auto it = f->history.find(fn_type);
    if (it == f->history.end()) return has_user ? t_user_ms : f->default_ms;
    if (!has_user) return it->second;
    return f->alpha * t_user_ms + (1.0 - f->alpha) * it->second;
}

}  // extern "C"
