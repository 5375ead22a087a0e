"""Seeded synthetic inputs for the KV offload / upload path.

This module serves both the CPU oracle and the HIP library with the *same* inputs
and contains no part of the method: it only describes pool shapes, draws values and
block ids, and scripts sequences of calls against whatever backend it is given.
All randomness comes from ``numpy.random.Generator(PCG64(seed))`` (host side) or a
seeded ``torch.Generator`` (device-side fills of pools too large to draw on the host).

The pools stand in for the serving runs the paper measures on (Sec. 7.1, ShareGPT and
AgentCode driven traffic on Qwen2.5 models): the path moves opaque bytes, so only the
shapes matter.  Shapes follow Sec. 7.6 (16-token blocks, bf16, 64..320 blocks per
request) scaled to the five benchmark configurations.
"""
from dataclasses import dataclass, replace

import numpy as np

BASE_SEED = 251018586


def seed_for(config_index, salt=0):
    return BASE_SEED + int(config_index) + 1000003 * int(salt)


def rng_for(config_index, salt=0):
    return np.random.Generator(np.random.PCG64(seed_for(config_index, salt)))


@dataclass(frozen=True)
class PoolShape:
    name: str
    num_layers: int
    kv_heads: int
    head_dim: int
    block_size: int          # tokens per block
    elem_bytes: int          # 2 = bf16, 1 = fp8
    num_blocks: int          # NB
    scales_per_block: int = 0  # 0, 1 or 2*num_layers fp32 words per block
    dist: str = "normal"     # value distribution of the fill

    @property
    def planes(self):
        return 2 * self.num_layers

    @property
    def page_bytes(self):
        return self.block_size * self.kv_heads * self.head_dim * self.elem_bytes

    @property
    def pool_bytes(self):
        return self.planes * self.num_blocks * self.page_bytes

    def with_blocks(self, nb):
        return replace(self, num_blocks=int(nb))


# The five benchmark configurations (index = position in the list).
CONFIGS = [
    PoolShape("tiny", 2, 4, 64, 16, 2, 256, 0, "uniform"),
    PoolShape("llama3-8b", 32, 8, 128, 16, 2, 16384, 0, "normal"),
    PoolShape("llama3-8b-64agents", 32, 8, 128, 16, 2, 16384, 0, "normal"),
    PoolShape("qwen-32b-trace", 64, 8, 128, 16, 2, 16384, 0, "normal"),
    PoolShape("70b-fp8", 80, 8, 128, 32, 1, 32768, 160, "fp8"),
]
# The shape the paper's own measurement uses (Sec. 7.6: Qwen2.5-14B, 3 MiB per block).
PAPER_14B = PoolShape("qwen2.5-14b", 48, 8, 128, 16, 2, 16384, 0, "normal")


# --------------------------------------------------------------------------- values
def _f32_to_bf16_bits(x):
    """Round-to-nearest-even float32 -> bfloat16 bit patterns (uint16)."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    rounded = u + (np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1)))
    return (rounded >> np.uint32(16)).astype(np.uint16)


def make_pool_host(shape, rng):
    """Pool bytes on the host (small pools only): uint8 array of shape.pool_bytes."""
    n_elem = shape.pool_bytes // shape.elem_bytes
    if shape.dist == "uniform":
        vals = rng.uniform(-1.0, 1.0, size=n_elem).astype(np.float32)
    elif shape.dist in ("normal", "fp8"):
        vals = rng.standard_normal(size=n_elem, dtype=np.float32)
    else:
        raise ValueError(shape.dist)
    if shape.elem_bytes == 2:
        return _f32_to_bf16_bits(vals).view(np.uint8).copy()
    if shape.elem_bytes == 1:
        import torch
        # OCP e4m3 ("fn") bytes, one scale per page: amax / 448
        t = torch.from_numpy(vals).view(shape.planes * shape.num_blocks, -1)
        amax = t.abs().amax(dim=1, keepdim=True).clamp_min(1e-12)
        q = (t * (448.0 / amax)).to(torch.float8_e4m3fn)
        return q.view(torch.uint8).numpy().reshape(-1).copy()
    raise ValueError(shape.elem_bytes)


def make_scales_host(shape, rng):
    """Scale words [S][NB] as raw uint32 bit patterns of positive fp32 values."""
    if not shape.scales_per_block:
        return None
    s = rng.uniform(1e-3, 4.0, size=shape.scales_per_block * shape.num_blocks).astype(np.float32)
    return s.view(np.uint32).copy()


def make_pool_device(shape, seed, device="cuda:0"):
    """Fill a full-size pool on the device with a seeded torch generator; returns uint8 tensor."""
    import torch
    g = torch.Generator(device=device)
    g.manual_seed(int(seed))
    pool = torch.empty(shape.pool_bytes, dtype=torch.uint8, device=device)
    plane_elems = shape.num_blocks * shape.page_bytes // shape.elem_bytes
    view = pool.view(shape.planes, shape.num_blocks * shape.page_bytes)
    for p in range(shape.planes):
        if shape.elem_bytes == 2:
            dst = view[p].view(torch.bfloat16)
            if shape.dist == "uniform":
                dst.uniform_(-1.0, 1.0, generator=g)
            else:
                dst.normal_(0.0, 1.0, generator=g)
        else:
            x = torch.empty(plane_elems, dtype=torch.bfloat16, device=device).normal_(0.0, 1.0, generator=g)
            x = x.view(shape.num_blocks, -1).float()
            amax = x.abs().amax(dim=1, keepdim=True).clamp_min(1e-12)
            view[p].copy_((x * (448.0 / amax)).to(torch.float8_e4m3fn).view(torch.uint8).reshape(-1))
            del x
    return pool


def make_scales_device(shape, seed, device="cuda:0"):
    import torch
    if not shape.scales_per_block:
        return None
    g = torch.Generator(device=device)
    g.manual_seed(int(seed) + 77)
    s = torch.empty(shape.scales_per_block * shape.num_blocks, dtype=torch.float32, device=device)
    s.uniform_(1e-3, 4.0, generator=g)
    return s


# --------------------------------------------------------------------------- ids
def pick_ids(rng, num_blocks, n, exclude=()):
    """n distinct block ids, uniformly at random, none from `exclude`; int32."""
    perm = rng.permutation(num_blocks)
    if len(exclude):
        mask = np.ones(num_blocks, dtype=bool)
        mask[np.asarray(exclude, dtype=np.int64)] = False
        perm = perm[mask[perm]]
    if n > perm.size:
        raise ValueError("not enough blocks")
    return perm[:n].astype(np.int32)


def lognormal_contexts(rng, n_agents, median=2048, sigma=0.8, cap=16384, floor=1):
    """Context lengths in tokens: lognormal(median, sigma), capped."""
    x = rng.lognormal(mean=np.log(median), sigma=sigma, size=n_agents)
    return np.clip(np.rint(x), floor, cap).astype(np.int64)


def uniform_contexts(rng, n_agents, lo=1024, hi=32768):
    return rng.integers(lo, hi + 1, size=n_agents).astype(np.int64)


def blocks_of(tokens, block_size):
    return -(-np.asarray(tokens, dtype=np.int64) // block_size)


# --------------------------------------------------------------------------- scripted call sequences
def fragment_pool(backend, rng, n_ops=50000, median_blocks=128, sigma=0.8, need_free=0):
    """Fragments a block pool with a seeded stream of alloc / free calls.

    `backend` offers alloc(n) -> list of ids or None, free(ids) and n_free().  Each op: with
    probability 1/2 (or when nothing is live) allocate k ~ lognormal(median_blocks, sigma) blocks
    if they fit, otherwise release one live allocation chosen uniformly.  Afterwards live
    allocations are released in seeded random order until at least `need_free` blocks are free.
    Returns the list of (op, size) performed, so two backends can be compared.
    """
    live, log = [], []
    for _ in range(n_ops):
        want_alloc = rng.random() < 0.5 or not live
        k = int(np.clip(np.rint(rng.lognormal(np.log(median_blocks), sigma)), 1, None))
        victim = int(rng.integers(len(live))) if live else 0
        if want_alloc and k <= backend.n_free():
            ids = backend.alloc(k)
            if ids is None:
                raise RuntimeError("alloc failed although the blocks were free")
            live.append(list(ids))
            log.append(("a", k))
        elif live:
            backend.free(live.pop(victim))
            log.append(("f", victim))
    order = rng.permutation(len(live)) if live else []
    for i in order:
        if backend.n_free() >= need_free:
            break
        backend.free(live[int(i)])
        live[int(i)] = None
        log.append(("r", int(i)))
    return log


def dag_trace(rng, n_agents=200, depth=6, mean_call_s=2.0, predicted_s=2.0, lead_s=0.2,
              median_tokens=2048, sigma=0.8, cap_tokens=16384, block_size=16):
    """A seeded trace of agents in a random DAG, each making one function call.

    Nodes are spread over `depth` levels (at least one per level, the rest uniformly); every node
    below level 0 gets 1-3 parents drawn from the level above and starts when all of them have
    finished.  An agent computes for c1 seconds, calls a tool for d ~ Exp(mean_call_s) seconds and
    computes c2 seconds more.  The predictor is the constant `predicted_s`, so the upload is due
    `lead_s` before the predicted finish, or at the real finish when the tool returns earlier.

    Returns (agents, events): agents[i] = dict(blocks, level, parents, ...), events = list of
    (time, order, kind, agent) sorted by virtual time; kind in start / call_start / upload_due /
    call_finish / finish.  Virtual time orders the calls; nothing sleeps.
    """
    levels = np.concatenate([np.arange(depth), rng.integers(0, depth, size=n_agents - depth)])
    levels.sort()
    by_level = [np.flatnonzero(levels == l) for l in range(depth)]
    tokens = lognormal_contexts(rng, n_agents, median_tokens, sigma, cap_tokens)
    agents, finish = [], np.zeros(n_agents)
    events = []
    order = {"finish": 0, "call_finish": 1, "start": 2, "call_start": 3, "upload_due": 4}
    for i in range(n_agents):
        l = int(levels[i])
        parents = []
        if l > 0:
            k = int(rng.integers(1, 4))
            parents = sorted(int(x) for x in rng.choice(by_level[l - 1], size=min(k, len(by_level[l - 1])), replace=False))
        c1, c2 = float(rng.uniform(0.05, 0.5)), float(rng.uniform(0.05, 0.3))
        d = float(rng.exponential(mean_call_s))
        t_start = max([finish[p] for p in parents], default=0.0)
        t_call = t_start + c1
        t_ret = t_call + d
        t_up = min(t_call + max(0.0, predicted_s - lead_s), t_ret)
        finish[i] = t_ret + c2
        agents.append(dict(blocks=int(blocks_of(tokens[i], block_size)), tokens=int(tokens[i]), level=l,
                           parents=parents, call_s=d, early=bool(d < predicted_s - lead_s)))
        for t, kind in ((t_start, "start"), (t_call, "call_start"), (t_up, "upload_due"),
                        (t_ret, "call_finish"), (finish[i], "finish")):
            events.append((float(t), order[kind], kind, i))
    events.sort(key=lambda e: (e[0], e[1], e[3]))
    return agents, events
