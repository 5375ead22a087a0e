"""Oracle for the scheduling arithmetic next to the copy path.  TEST INFRASTRUCTURE ONLY.

Plain Python written from the paper's statements, in the paper's notation:

* transfer cost (Sec. 4.2, Eq. 2): T_transfer = T_offload(N_blocks) + T_upload(N_blocks), each term
  linear in N_blocks with constants calibrated from per-block measurements on the target platform;
* ShouldOffload (Sec. 4.2, Alg. 1): the scheduling window is the predicted stall minus the transfer time
  and a window that is not positive rejects; the window times the observed decode throughput is a
  token capacity; the first request in queue order whose incremental KV demand fits the freed blocks
  and whose total work fits that capacity decides;
* upload budget (Sec. 4.3, Eq. 3) and gradual reservation (Sec. 4.3, Eq. 4);
* the hard rejections that come before any scoring (Sec. 4.2): not enough CPU capacity, a stall
  shorter than the transfer, no waiting request that fits, GPU memory pressure under a threshold;
* one scheduling step of predictive upload (Sec. 4.3): candidates ranked by P_upload = I + U, the
  step's budget from Eq. 3, each candidate's reservation from Eq. 4 in rank order.

Readings where the paper is silent: the linear terms are fitted by ordinary least squares; a waiting
request is the pair (kv_blocks, work_tokens); in Eq. 4 B_remain is what is left of this step's budget
after higher-ranked candidates, B_deficit the candidate's blocks still missing.  The hard rejections
are tested in the order the paper lists them and the first that applies is the reason; pressure is
used / total blocks and "below" is strict.  I and U are inputs (the paper gives no formula for U);
equal P_upload: the more urgent candidate first, then the one named first.
"""
import math


def fit_linear(n_blocks, t_ms):
    """Least-squares (a, b) of t = a + b * N."""
    m = len(n_blocks)
    if m < 2 or len(t_ms) != m:
        raise ValueError("need at least two points")
    mean_n = math.fsum(n_blocks) / m
    mean_t = math.fsum(t_ms) / m
    sxx = math.fsum((n - mean_n) ** 2 for n in n_blocks)
    if sxx == 0:
        raise ValueError("all sizes are equal")
    sxy = math.fsum((n - mean_n) * (t - mean_t) for n, t in zip(n_blocks, t_ms))
    b = sxy / sxx
    return mean_t - b * mean_n, b


def estimate_transfer_ms(model, n_blocks):
    """Eq. 2.  model = (a_off, b_off, a_up, b_up) in ms and ms per block."""
    a_off, b_off, a_up, b_up = model
    t_offload = a_off + b_off * n_blocks
    t_upload = a_up + b_up * n_blocks
    return t_offload + t_upload


def should_offload(model, req_blocks, t_fc_ms, v_throughput_tokens_per_ms, waiting):
    """The gate of Sec. 4.2, from its three paragraphs (transfer overhead, scheduling window, waiting-request
    fit).  waiting = [(kv_blocks, work_tokens), ...] in queue order.
    Returns (decision, index of the chosen waiting request or -1)."""
    # scheduling window: what is left of the predicted stall once the round trip is paid for
    window_ms = t_fc_ms - estimate_transfer_ms(model, req_blocks)
    if not window_ms > 0:
        return False, -1
    # the window as decode work, at the throughput the system has been observed to reach
    tokens_that_fit = window_ms * v_throughput_tokens_per_ms
    eligible = [k for k, (kv_blocks, work_tokens) in enumerate(waiting)
                if kv_blocks <= req_blocks and work_tokens <= tokens_that_fit]
    if not eligible:
        return False, -1
    return True, eligible[0]                 # first_fit: the first eligible request in queue order


def upload_budget(b_gpu_free, d_critical, b_shared_free):
    """Eq. 3."""
    return max(0, b_gpu_free - max(0, d_critical - b_shared_free))


def gradual_reserve(b_remain, b_deficit, b_upload):
    """Eq. 4."""
    return min(b_remain, -(-b_deficit // 2), b_upload)


PASS, CPU_FULL, STALL_SHORT, NO_FIT, LOW_PRESSURE = 0, 1, 2, 3, 4


def offload_gate(model, req_blocks, cpu_free_blocks, gpu_used_blocks, gpu_total_blocks, pressure_threshold,
                 t_fc_ms, v_throughput_tokens_per_ms, waiting):
    """The four hard rejections of Sec. 4.2.  Returns (reason, index of the waiting request that fits or -1);
    reason PASS means the offload may go on to be scored / issued."""
    if cpu_free_blocks < req_blocks:
        return CPU_FULL, -1
    if t_fc_ms <= estimate_transfer_ms(model, req_blocks):
        return STALL_SHORT, -1
    ok, k = should_offload(model, req_blocks, t_fc_ms, v_throughput_tokens_per_ms, waiting)
    if not ok:
        return NO_FIT, -1
    if gpu_used_blocks / gpu_total_blocks < pressure_threshold:
        return LOW_PRESSURE, -1
    return PASS, k


def upload_plan(candidates, b_gpu_free, d_critical, b_shared_free):
    """One scheduling step of predictive upload.  candidates = [(importance, urgency, deficit), ...].
    Returns (order, reserve): candidate indices by falling P_upload = I + U, and the blocks to reserve
    for each candidate this step (indexed like `candidates`)."""
    b_upload = upload_budget(b_gpu_free, d_critical, b_shared_free)
    order = sorted(range(len(candidates)),
                   key=lambda i: (-(candidates[i][0] + candidates[i][1]), -candidates[i][1], i))
    reserve = [0] * len(candidates)
    b_remain = b_upload
    for i in order:
        reserve[i] = gradual_reserve(b_remain, candidates[i][2], b_upload)
        b_remain -= reserve[i]
    return order, reserve
