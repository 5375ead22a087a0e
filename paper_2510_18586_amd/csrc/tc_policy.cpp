// Host-side scheduling arithmetic that consumes the copy path's measurements: the linear
// transfer-cost model (paper Eq. 2), the ShouldOffload gate (Alg. 1), the upload budget (Eq. 3)
// and the gradual reservation (Eq. 4).  No GPU work here; tc_calibrate lives in the engine.
#include <cmath>

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

extern "C" {

int tc_cost_fit(const uint32_t *n_blocks, const double *offload_ms, const double *upload_ms, uint32_t m,
                tc_cost_model *out)
{
    if (!n_blocks || !offload_ms || !upload_ms || !out || m < 2) return TC_ERR_INVAL;
    tc_cost_model r;
    if (!fit_line(n_blocks, offload_ms, m, &r.off_a_ms, &r.off_b_ms_per_block)) return TC_ERR_INVAL;
    if (!fit_line(n_blocks, upload_ms, m, &r.up_a_ms, &r.up_b_ms_per_block)) return TC_ERR_INVAL;
    *out = r;
    return TC_OK;
}

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
{
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
}

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

}  // extern "C"
