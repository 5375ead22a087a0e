"""Oracle for the scheduling arithmetic next to the copy path.  TEST INFRASTRUCTURE ONLY.

Plain Python written from the paper's statements, in the paper's notation:

* transfer cost (Sec. 4.2, Eq. 2): T_transfer = T_offload(N_blocks) + T_upload(N_blocks), each term
  linear in N_blocks with constants calibrated from per-block measurements on the target platform;
* ShouldOffload (Sec. 4.2, Alg. 1): reject when T_fc <= T_transfer; otherwise T_window = T_fc -
  T_transfer, N_capacity = T_window * v_throughput, and the first request in queue order whose
  incremental KV demand fits the freed blocks and whose work fits N_capacity decides;
* upload budget (Sec. 4.3, Eq. 3) and gradual reservation (Sec. 4.3, Eq. 4).

Readings where the paper is silent: the linear terms are fitted by ordinary least squares; a waiting
request is the pair (kv_blocks, work_tokens); in Eq. 4 B_remain is what is left of this step's budget
after higher-ranked candidates, B_deficit the candidate's blocks still missing.
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
    """Alg. 1.  waiting = [(kv_blocks, work_tokens), ...] in queue order.
    Returns (decision, index of the chosen waiting request or -1)."""
    t_transfer = estimate_transfer_ms(model, req_blocks)
    if t_fc_ms <= t_transfer:
        return False, -1                      # stall too short
    t_window = t_fc_ms - t_transfer
    n_capacity = t_window * v_throughput_tokens_per_ms
    for k, (kv_blocks, work_tokens) in enumerate(waiting):   # first fit, queue order
        if kv_blocks <= req_blocks and work_tokens <= n_capacity:
            return True, k
    return False, -1


def upload_budget(b_gpu_free, d_critical, b_shared_free):
    """Eq. 3."""
    return max(0, b_gpu_free - max(0, d_critical - b_shared_free))


def gradual_reserve(b_remain, b_deficit, b_upload):
    """Eq. 4."""
    return min(b_remain, -(-b_deficit // 2), b_upload)
