"""The same question for the oracle's Python parts (bookkeeping model, scheduling arithmetic,
lifecycle, forecast): a planted mistake in a copy of the source must make at least one pin fail.
CPU only; the copies are exec'd into throw-away modules and swapped into the pin modules' namespaces."""
import inspect
import os
import struct
import types

import pytest

import oracle
import test_oracle_block_pool as pins_pool
import test_oracle_lifecycle as pins_life
import test_oracle_policy as pins_policy
import test_oracle_residency as pins_res
import test_oracle_transfer_plan as pins_plan

ODIR = os.path.dirname(oracle.__file__)

CASES = {
    # (source file, pin module, names to swap in the pin module): {description: (old, new)}
    ("policy.py", pins_policy, ("policy",)): {
        "a stall equal to the transfer time is accepted": ("if not window_ms > 0:", "if not window_ms >= 0:"),
        "last fit instead of first fit": ("return True, eligible[0]", "return True, eligible[-1]"),
        "a request needing exactly the freed blocks does not fit": ("if kv_blocks <= req_blocks and", "if kv_blocks < req_blocks and"),
        "capacity divides by the throughput": ("tokens_that_fit = window_ms * v_throughput_tokens_per_ms", "tokens_that_fit = window_ms / v_throughput_tokens_per_ms"),
        "the window forgets the transfer time": ("window_ms = t_fc_ms - estimate_transfer_ms(model, req_blocks)", "window_ms = t_fc_ms"),
        "work is compared with the window in ms": ("and work_tokens <= tokens_that_fit]", "and work_tokens <= window_ms]"),
        "transfer cost drops the upload": ("return t_offload + t_upload", "return t_offload"),
        "budget lets the inner term go negative": ("return max(0, b_gpu_free - max(0, d_critical - b_shared_free))",
                                                   "return max(0, b_gpu_free - (d_critical - b_shared_free))"),
        "half of the deficit rounds down": ("-(-b_deficit // 2)", "b_deficit // 2"),
        "the fit's slope is inverted": ("b = sxy / sxx", "b = sxx / sxy"),
        "the gate forgets the CPU capacity": ("    if cpu_free_blocks < req_blocks:\n        return CPU_FULL, -1\n", ""),
        "the gate reports the pressure before the fit": ("    ok, k = should_offload(model, req_blocks, t_fc_ms, v_throughput_tokens_per_ms, waiting)\n    if not ok:\n        return NO_FIT, -1\n    if gpu_used_blocks / gpu_total_blocks < pressure_threshold:\n        return LOW_PRESSURE, -1\n",
                                                         "    if gpu_used_blocks / gpu_total_blocks < pressure_threshold:\n        return LOW_PRESSURE, -1\n    ok, k = should_offload(model, req_blocks, t_fc_ms, v_throughput_tokens_per_ms, waiting)\n    if not ok:\n        return NO_FIT, -1\n"),
        "pressure at the threshold is rejected": ("if gpu_used_blocks / gpu_total_blocks < pressure_threshold:", "if gpu_used_blocks / gpu_total_blocks <= pressure_threshold:"),
        "a short stall is reported as no fit": ("    if t_fc_ms <= estimate_transfer_ms(model, req_blocks):\n        return STALL_SHORT, -1\n", ""),
        "uploads ranked by importance alone": ("key=lambda i: (-(candidates[i][0] + candidates[i][1]), -candidates[i][1], i))", "key=lambda i: (-candidates[i][0], -candidates[i][1], i))"),
        "lowest priority uploads first": ("key=lambda i: (-(candidates[i][0] + candidates[i][1]), -candidates[i][1], i))", "key=lambda i: ((candidates[i][0] + candidates[i][1]), -candidates[i][1], i))"),
        "ties go to the less urgent": ("key=lambda i: (-(candidates[i][0] + candidates[i][1]), -candidates[i][1], i))", "key=lambda i: (-(candidates[i][0] + candidates[i][1]), candidates[i][1], i))"),
        "every candidate sees the whole budget": ("        b_remain -= reserve[i]\n", ""),
        "the plan ignores the critical demand": ("    b_upload = upload_budget(b_gpu_free, d_critical, b_shared_free)\n    order", "    b_upload = b_gpu_free\n    order"),
    },
    ("lifecycle.py", pins_life, ("L",)): {
        "uploaded + call_finish waits instead of resuming": ("return (RUNNING, False, False), RESUME          # already back", "return (UPLOADED, True, False), WAIT  #"),
        "offloaded + call_finish does nothing": ("return (OFFLOADED, True, False), UPLOAD_NOW     # returned early", "return (OFFLOADED, True, False), NONE  #"),
        "a finish during the offload is forgotten": ("return (PENDING_OFFLOAD, True, True), WAIT", "return (PENDING_OFFLOAD, False, True), WAIT"),
        "an agent resumes while its upload is in flight": ("return (PENDING_UPLOAD, True, in_flight), WAIT", "return (RUNNING, False, False), RESUME"),
        "the moving average uses alpha": ("self.gamma * elapsed_ms + (1 - self.gamma) * self.history[fn_type]",
                                          "self.alpha * elapsed_ms + (1 - self.alpha) * self.history[fn_type]"),
        "Eq. 1 with the weights swapped": ("return self.alpha * t_user_ms + (1 - self.alpha) * h", "return (1 - self.alpha) * t_user_ms + self.alpha * h"),
        "history wins over the user's estimate entirely": ("return self.alpha * t_user_ms + (1 - self.alpha) * h", "return h"),
        "the first observation is averaged with the default": ("            self.history[fn_type] = elapsed_ms\n",
                                                               "            self.history[fn_type] = self.gamma * elapsed_ms + (1 - self.gamma) * self.default_ms\n"),
    },
    ("block_pool.py", pins_pool, ("OracleBlockPool", "OracleHostArena", "OracleError")): {
        "a released block skips pending-free": ("                if self.inflight[b] > 0:\n                    self.pending[b] = True\n                else:\n                    self.free_stack.append(b)",
                                                "                self.free_stack.append(b)"),
        "the free list is a queue": ("out = [self.free_stack.pop() for _ in range(n)]", "out = [self.free_stack.pop(0) for _ in range(n)]"),
        "retiring forgets the pending-free blocks": ("            if self.inflight[b] == 0 and self.pending[b]:\n                self.pending[b] = False\n                self.free_stack.append(b)",
                                                     "            if self.inflight[b] == 0 and self.pending[b]:\n                self.pending[b] = False"),
        "a short pool hands out what it has": ("        if n > len(self.free_stack):\n            raise OracleError(\"NOMEM\")", "        n = min(n, len(self.free_stack))"),
        "one finished read frees a block two copies read": ("if self.inflight[b] == 0 and self.pending[b]:", "if self.pending[b]:"),
        "shared blocks may move": ("            if self.refcount[b] > 1:\n                raise OracleError(\"SHARED\"", "            if self.refcount[b] > 99:\n                raise OracleError(\"SHARED\""),
        "the arena takes the last run that fits": ("for k, (start, length) in enumerate(self.free_runs):", "for k, (start, length) in reversed(list(enumerate(self.free_runs))):"),
        "released runs are not merged": ("if merged and merged[-1][0] + merged[-1][1] == s:", "if False:"),
        "alloc_prefer claims a pending-free block": ("if 0 <= b < self.NB and b in self.free_stack:", "if 0 <= b < self.NB and self.refcount[b] == 0:"),
        "alloc_prefer fills the gaps before it claims": ("        for i, b in enumerate(preferred):\n            if 0 <= b < self.NB and b in self.free_stack:",
                                                         "        for i, b in reversed(list(enumerate(preferred))):\n            if 0 <= b < self.NB and b in self.free_stack:"),
        "alloc_prefer hands out what it has": ("        if len(preferred) > len(self.free_stack):\n            raise OracleError(\"NOMEM\")", "        preferred = preferred[:len(self.free_stack)]"),
        "a busy arena buffer is recycled at once": ("        if self.inflight.get(start, 0) > 0:\n            self.pending.add(start)\n        else:\n            self._release(start)",
                                                    "        self._release(start)"),
    },
    ("residency.py", pins_res, ("R",)): {
        "FNV-1 instead of FNV-1a": ("        h ^= byte\n        h = (h * FNV_PRIME) & _M64", "        h = (h * FNV_PRIME) & _M64\n        h ^= byte"),
        "the 32-bit FNV prime": ("FNV_PRIME = 0x100000001B3", "FNV_PRIME = 0x01000193"),
        "keys do not chain": ('h = fnv1a64(struct.pack("<Q", h) + struct.pack(', 'h = fnv1a64(struct.pack("<Q", parent) + struct.pack('),
        "a partial block gets a key": ("for i in range(len(tokens) // block_size):", "for i in range(-(-len(tokens) // block_size)):"),
        "tokens hashed big-endian": ('struct.pack(f"<{block_size}i"', 'struct.pack(f">{block_size}i"'),
        "lookup skips a miss instead of stopping": ("            if e is None:\n                break", "            if e is None:\n                continue"),
        "every record at the base address": ("self.entries[k] = [CPU, host_base + j * record_bytes, int(gpu_blocks[j])]", "self.entries[k] = [CPU, host_base, int(gpu_blocks[j])]"),
        "an upload keeps the old GPU block": ("            self.entries[k][2] = int(b)\n", ""),
        "an H2D entry can be uploaded again": ("if k not in self.entries or self.entries[k][0] != CPU:\n                raise OracleError(\"INVAL\", f\"key {k:#x} is not CPU-resident\")",
                                               "if k not in self.entries:\n                raise OracleError(\"INVAL\", f\"key {k:#x} is not CPU-resident\")"),
        "a finished upload stays in the index": ("        for k in keys:\n            del self.entries[k]\n\n    def remove", "\n    def remove"),
        "eviction under a running upload": ("if k not in self.entries or self.entries[k][0] != CPU:\n                raise OracleError(\"INVAL\", f\"key {k:#x} is not an idle",
                                             "if k not in self.entries:\n                raise OracleError(\"INVAL\", f\"key {k:#x} is not an idle"),
        "a key entered twice replaces the first": ("            if k in self.entries:\n                raise OracleError(\"DUP\", f\"key {k:#x} is already CPU-resident\")", "            pass"),
        "pending counts CPU-resident entries": ("[ABSENT])[0] == H2D)", "[ABSENT])[0] != ABSENT)"),
    },
    ("transfer_plan.py", pins_plan, ("T",)): {
        "a request may wrap around the end of the ring": ("        if tail + n > self.cap:\n            skipped = self.cap - tail\n            start = 0\n", ""),
        "the skipped tail is not counted": ("if self.used() + skipped + n > self.cap:", "if self.used() + n > self.cap:"),
        "an empty ring goes on where it stopped": ("        if not self.live:\n            return 0\n        start, n, _ = self.live[-1]", "        if not self.live:\n            return 3\n        start, n, _ = self.live[-1]"),
        "the ring releases the newest span": ("        return self.live.pop(0)\n\n    def cancel_newest", "        return self.live.pop()\n\n    def cancel_newest"),
        "uploads cut the list like offloads": ("return sizes[::-1] if upload else sizes", "return sizes"),
        "a chunk may exceed its slot": ("take = min(int(slot_blocks), left)", "take = min(int(slot_blocks) + 1, left)"),
        "pieces are placed by their list position": ("out.append((k, a - first, a - c0, b - a))", "out.append((k, a - first, a, b - a))"),
        "pieces start at the buffer's head": ("out.append((k, a - first, a - c0, b - a))", "out.append((k, 0, a - c0, b - a))"),
        "a tail may straddle two buffers": ("if first >= s_first and c0 + nblk <= s_first + s_n:", "if first >= s_first and first < s_first + s_n:"),
        "the tail is the head of the chunk": ("first = c0 + nblk - m", "first = c0"),
        "the first toucher counts": ("                if x in op[index]:\n                    last = op", "                if x in op[index] and last is None:\n                    last = op"),
        "same-stream transfers are waited for too": ("if last is not None and last[1] != stream:", "if last is not None:"),
        "host buffers carry no hazard": ("for what, index in ((block_ids, 2), (arena_starts, 3)):", "for what, index in ((block_ids, 2),):"),
        "a large offload goes direct": ("return DIRECT if (upload_in_flight or total_bytes < auto_direct_bytes) else STAGED", "return DIRECT if (upload_in_flight or total_bytes >= auto_direct_bytes) else STAGED"),
        "duplex is ignored": ("return DIRECT if (upload_in_flight or total_bytes < auto_direct_bytes) else STAGED", "return DIRECT if total_bytes < auto_direct_bytes else STAGED"),
        "uploads are staged unless forced": ("return STAGED if mode == PATH_STAGED else DIRECT", "return DIRECT if mode == PATH_DIRECT else STAGED"),
        "a single chunk gets a tail": ("return auto_div if (n_chunks > 1 and not overlapped) else 0", "return auto_div if not overlapped else 0"),
        "overlapped transfers get a tail too": ("return auto_div if (n_chunks > 1 and not overlapped) else 0", "return auto_div if n_chunks > 1 else 0"),
        "a single chunk hops between streams": ("return option == 1 and n_chunks > 1", "return option == 1"),
        "overlap without being asked for": ("return option == 1 and n_chunks > 1", "return n_chunks > 1"),
        "a transfer in line keeps its head": ("    return plan_chunks(total, slot_blocks, upload, 0), False", "    return sizes, False"),
        "short lists get a head too": ("if head > 0 and left > 2 * head:", "if head > 0 and left > head:"),
        "a head may be longer than a slot": ("head = min(int(head_blocks), int(slot_blocks))", "head = int(head_blocks)"),
        "the head is not taken off the list": ("        sizes.append(head)\n        left -= head\n", "        sizes.append(head)\n"),
        "a failed transfer gives its span back": ("        op.update(ticket=self.next_ticket, failed=failed)\n", "        op.update(ticket=self.next_ticket, failed=failed)\n        if failed:\n            self.ring.cancel_newest()\n"),
    },
}

ALL = [(key, name) for key, d in CASES.items() for name in d]


def _load(fname, old, new):
    text = open(os.path.join(ODIR, fname)).read()
    assert text.count(old) == 1, f"expected exactly one occurrence of the line to break in {fname}"
    mod = types.ModuleType("oracle_mutant_" + fname[:-3])
    mod.__package__ = "oracle"          # the sources import their siblings relatively
    exec(compile(text.replace(old, new), fname + " (mutant)", "exec"), mod.__dict__)
    return mod


def _failing(pin_module):
    failed = []
    for name, fn in inspect.getmembers(pin_module, inspect.isfunction):
        if name.startswith("test_") and not inspect.signature(fn).parameters:
            try:
                fn()
            except (AssertionError, KeyError, IndexError, ValueError, ZeroDivisionError, TypeError, struct.error, pytest.fail.Exception) as e:
                failed.append(name)
            except Exception as e:      # noqa: BLE001  the models' own error types
                if type(e).__name__ in ("OracleError", "Invalid"):
                    failed.append(name)
                else:
                    raise
    return failed


@pytest.mark.parametrize("key,name", ALL, ids=[n for _, n in ALL])
def test_planted_mistake_is_caught(key, name):
    fname, pin_module, swap = key
    old, new = CASES[key][name]
    mutant = _load(fname, old, new)
    saved = {s: getattr(pin_module, s) for s in swap}
    try:
        for s in swap:
            setattr(pin_module, s, mutant if s in ("policy", "L", "R", "T") else getattr(mutant, s))
        failed = _failing(pin_module)
    finally:
        for s, v in saved.items():
            setattr(pin_module, s, v)
    assert failed, f"no pin noticed: {name}"


def test_unmodified_sources_pass():
    for (fname, pin_module, swap) in CASES:
        assert _failing(pin_module) == []
