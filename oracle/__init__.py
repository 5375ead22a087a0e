"""CPU oracle for paged-KV offload / upload.  TEST INFRASTRUCTURE ONLY.

Only the test-suite, the smoke check and the benchmark's CPU-baseline leg may import
this package; the product library never does, and this package imports nothing of
the product.  The data movement is defined in plain C (``tc_oracle.c``, built with
gcc into ``liboracle.so`` next to it); the block bookkeeping model is plain Python
(``block_pool.py``).

Arrays are numpy, host memory only:
  pool    uint8, P*NB*pb bytes, plane-major ``[P][NB][pb]`` with P = 2*L
  scales  uint32, ``[S][NB]`` (S in {0, 1, P}), or None
  host    uint8, n*rec bytes, block-major records
  ids     int32
"""
import ctypes
import os
import subprocess

import numpy as np

from .block_pool import OracleBlockPool, OracleHostArena, OracleError  # noqa: F401

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "tc_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")


def compile_c(src, out):
    """gcc, plain C11, no GPU toolchain involved."""
    subprocess.run(["gcc", "-std=c11", "-O2", "-Wall", "-Wextra", "-Werror", "-fPIC", "-shared", src, "-o", out],
                   check=True)
    return out


def build(force=False):
    """Compile tc_oracle.c into liboracle.so next to it."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        compile_c(_SRC, _LIB)
    return _LIB


def _ptr(a, dtype, min_items, name):
    if a is None:
        return None
    if not isinstance(a, np.ndarray) or a.dtype != dtype or not a.flags["C_CONTIGUOUS"]:
        raise TypeError(f"{name}: need a C-contiguous numpy array of {np.dtype(dtype).name}")
    if a.size < min_items:
        raise ValueError(f"{name}: {a.size} items, need at least {min_items}")
    return a.ctypes.data


class OracleLibrary:
    """The C oracle behind one shared object (the tests also load deliberately broken copies of it
    to show that the pins notice)."""
    OracleError = OracleError

    def __init__(self, path):
        lib = ctypes.CDLL(path)
        u8p, u32p, i32p = ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p
        u32, u64 = ctypes.c_uint32, ctypes.c_uint64
        lib.tco_record_bytes.restype = u64
        lib.tco_record_bytes.argtypes = [u32, u64, u32]
        lib.tco_page_bytes.restype = u64
        lib.tco_page_bytes.argtypes = [u32, u32, u32, u32]
        lib.tco_blocks_for_tokens.restype = u64
        lib.tco_blocks_for_tokens.argtypes = [u64, u32]
        lib.tco_offload.restype = ctypes.c_int
        lib.tco_offload.argtypes = [u8p, u32p, u32, u64, u64, u32, i32p, u64, u8p]
        lib.tco_upload.restype = ctypes.c_int
        lib.tco_upload.argtypes = [u8p, u32, u64, u64, u32, i32p, u64, u8p, u32p, i32p]
        lib.tco_read_token.restype = ctypes.c_int
        lib.tco_read_token.argtypes = [u8p, u32, u64, u64, u32, i32p, u64, u32, u32, u8p]
        self._lib = lib

    def record_bytes(self, L, pb, S=0):
        return int(self._lib.tco_record_bytes(L, pb, S))

    def page_bytes(self, block_size, kv_heads, head_dim, elem_bytes):
        return int(self._lib.tco_page_bytes(block_size, kv_heads, head_dim, elem_bytes))

    def blocks_for_tokens(self, tokens, block_size):
        return int(self._lib.tco_blocks_for_tokens(tokens, block_size))

    def offload(self, pool, scales, L, NB, pb, S, ids, host):
        """host[j] <- the record of block ids[j]; see tc_oracle.c for the layout."""
        n = int(ids.size)
        rc = self._lib.tco_offload(
            _ptr(pool, np.uint8, 2 * L * NB * pb, "pool"),
            _ptr(scales, np.uint32, S * NB, "scales") if S else None,
            L, NB, pb, S,
            _ptr(ids, np.int32, n, "ids"), n,
            _ptr(host, np.uint8, n * self.record_bytes(L, pb, S), "host"),
        )
        if rc:
            raise OracleError(f"tco_offload failed: {rc}")

    def upload(self, host, L, NB, pb, S, new_ids, pool, scales, table_row=None):
        """Inverse copy into blocks new_ids, then table_row[i] = new_ids[i]."""
        n = int(new_ids.size)
        rc = self._lib.tco_upload(
            _ptr(host, np.uint8, n * self.record_bytes(L, pb, S), "host"),
            L, NB, pb, S,
            _ptr(new_ids, np.int32, n, "new_ids"), n,
            _ptr(pool, np.uint8, 2 * L * NB * pb, "pool"),
            _ptr(scales, np.uint32, S * NB, "scales") if S else None,
            _ptr(table_row, np.int32, n, "table_row"),
        )
        if rc:
            raise OracleError(f"tco_upload failed: {rc}")

    def read_token(self, pool, L, NB, pb, block_size, table, t, layer, kv):
        """Bytes of logical token t in plane (layer, kv), addressed through `table`."""
        out = np.empty(pb // block_size, dtype=np.uint8)
        rc = self._lib.tco_read_token(
            _ptr(pool, np.uint8, 2 * L * NB * pb, "pool"), L, NB, pb, block_size,
            _ptr(table, np.int32, t // block_size + 1, "table"), t, layer, kv, out.ctypes.data,
        )
        if rc:
            raise OracleError(f"tco_read_token failed: {rc}")
        return out


_default = None


def _lib():
    global _default
    if _default is None:
        _default = OracleLibrary(build())
    return _default


def record_bytes(L, pb, S=0):
    return _lib().record_bytes(L, pb, S)


def page_bytes(block_size, kv_heads, head_dim, elem_bytes):
    return _lib().page_bytes(block_size, kv_heads, head_dim, elem_bytes)


def blocks_for_tokens(tokens, block_size):
    return _lib().blocks_for_tokens(tokens, block_size)


def offload(pool, scales, L, NB, pb, S, ids, host):
    return _lib().offload(pool, scales, L, NB, pb, S, ids, host)


def upload(host, L, NB, pb, S, new_ids, pool, scales, table_row=None):
    return _lib().upload(host, L, NB, pb, S, new_ids, pool, scales, table_row)


def read_token(pool, L, NB, pb, block_size, table, t, layer, kv):
    return _lib().read_token(pool, L, NB, pb, block_size, table, t, layer, kv)
