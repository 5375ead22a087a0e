"""Residency map and CPU prefix-cache index: oracle model.  TEST INFRASTRUCTURE ONLY (see oracle/__init__.py).

Paper Sec. 6.3 ("CPU Migration Infrastructure"): the block pool owns the mapping between GPU
blocks, CPU blocks and block hashes.  An offload links the GPU block to its CPU block, marks the
KV cache CPU-resident and enters the block's hash in a CPU prefix-cache index; a later lookup that
hits there saves the recomputation but leaves an H2D transfer entry that has to complete before
the request runs; the upload puts the GPU mapping back.

The paper names no hash function and no index structure.  Readings taken here:
  * hashes are opaque 64-bit keys to the index;
  * a lookup is a *prefix* lookup: entry i can hit only if entries 0..i-1 hit (a block's key covers
    everything before it), so the answer is the longest leading run of keys that are present;
  * one key names one CPU record: entering a key twice is an error;
  * an entry is CPU-resident from the offload until an upload is begun, then an H2D entry until that
    upload is finished, then gone (the mapping is the GPU's again and the CPU block is unlinked);
  * the convenience hash is a parent-chained FNV-1a (64 bit) over whole blocks of token ids:
    h_i = FNV1a(le64(h_{i-1}) || le32(tokens of block i)), h_{-1} = the caller's parent key; a
    trailing partial block has no key.
"""
import struct

from .block_pool import OracleError

ABSENT, CPU, H2D = 0, 1, 2

FNV_BASIS = 0xCBF29CE484222325
FNV_PRIME = 0x100000001B3
_M64 = (1 << 64) - 1


def fnv1a64(data, basis=FNV_BASIS):
    """FNV-1a, 64 bit: for every byte, xor it in, then multiply by the prime (mod 2^64)."""
    h = basis & _M64
    for byte in bytes(data):
        h ^= byte
        h = (h * FNV_PRIME) & _M64
    return h


def chain_hashes(tokens, block_size, parent=0):
    """One key per *whole* block of token ids, each key covering all tokens up to its block's end."""
    out = []
    h = parent & _M64
    for i in range(len(tokens) // block_size):
        blk = tokens[i * block_size:(i + 1) * block_size]
        h = fnv1a64(struct.pack("<Q", h) + struct.pack(f"<{block_size}i", *[int(t) for t in blk]))
        out.append(h)
    return out


class OracleResidencyIndex:
    def __init__(self):
        self.entries = {}     # key -> [state, cpu_record_address, gpu_block]

    def size(self):
        return len(self.entries)

    @staticmethod
    def _distinct(keys):
        if len(set(keys)) != len(keys):
            raise OracleError("DUP")

    def insert(self, keys, gpu_blocks, host_base, record_bytes):
        """Offload of blocks gpu_blocks[j] into the records host_base + j*record_bytes."""
        keys = [int(k) for k in keys]
        if len(keys) != len(gpu_blocks):
            raise OracleError("INVAL")
        self._distinct(keys)
        for k in keys:
            if k in self.entries:
                raise OracleError("DUP", f"key {k:#x} is already CPU-resident")
        for j, k in enumerate(keys):
            self.entries[k] = [CPU, host_base + j * record_bytes, int(gpu_blocks[j])]

    def lookup(self, keys):
        """[(key, state, cpu_record, gpu_block)] for the longest leading run of keys present."""
        hits = []
        for k in keys:
            e = self.entries.get(int(k))
            if e is None:
                break
            hits.append((int(k), e[0], e[1], e[2]))
        return hits

    def begin_upload(self, keys, new_gpu_blocks):
        """CPU-resident -> H2D entry, to land in new_gpu_blocks."""
        keys = [int(k) for k in keys]
        if len(keys) != len(new_gpu_blocks):
            raise OracleError("INVAL")
        self._distinct(keys)
        for k in keys:
            if k not in self.entries or self.entries[k][0] != CPU:
                raise OracleError("INVAL", f"key {k:#x} is not CPU-resident")
        for k, b in zip(keys, new_gpu_blocks):
            self.entries[k][0] = H2D
            self.entries[k][2] = int(b)

    def finish_upload(self, keys):
        """The H2D transfer has completed: the GPU mapping is restored, the CPU block unlinked."""
        keys = [int(k) for k in keys]
        self._distinct(keys)
        for k in keys:
            if k not in self.entries or self.entries[k][0] != H2D:
                raise OracleError("INVAL", f"key {k:#x} has no upload in flight")
        for k in keys:
            del self.entries[k]

    def remove(self, keys):
        """Eviction of CPU-resident records (never of one an upload is reading)."""
        keys = [int(k) for k in keys]
        self._distinct(keys)
        for k in keys:
            if k not in self.entries or self.entries[k][0] != CPU:
                raise OracleError("INVAL", f"key {k:#x} is not an idle CPU-resident entry")
        for k in keys:
            del self.entries[k]

    def pending(self, keys):
        """How many of the keys still wait for their H2D transfer (the request may run at 0)."""
        return sum(1 for k in keys if self.entries.get(int(k), [ABSENT])[0] == H2D)
