"""The measurement helpers of the library are kernels too: the contiguous copies must be exact and
must reject what their kernels cannot take."""
import numpy as np
import pytest
import torch

import paper_2510_18586_amd as K
from harness import DEV

pytestmark = pytest.mark.gpu


def _src(nbytes, seed):
    g = torch.Generator(device=DEV)
    g.manual_seed(seed)
    return torch.randint(0, 256, (nbytes,), dtype=torch.uint8, device=DEV, generator=g)


@pytest.mark.parametrize("nbytes", [16, 4096 - 16, 32768, 32768 * 5 + 48, 64 << 20])
def test_copy_contiguous_is_exact_including_a_ragged_tail(nbytes):
    guard = 4096
    a = _src(nbytes, 1)
    b = torch.full((guard + nbytes + guard,), 0xEE, dtype=torch.uint8, device=DEV)
    stream = torch.cuda.Stream()
    stream.wait_stream(torch.cuda.current_stream())      # a and b were filled on torch's current stream
    K.check(K.tc_copy_contiguous(b[guard:], a, nbytes, stream))
    stream.synchronize()
    assert torch.equal(b[guard:guard + nbytes], a)
    assert bool((b[:guard] == 0xEE).all()) and bool((b[guard + nbytes:] == 0xEE).all())


@pytest.mark.parametrize("direct_loads", [0, 1])
@pytest.mark.parametrize("nbytes", [16384, 16384 * 7, 48 << 20])
def test_copy_via_lds_is_exact(direct_loads, nbytes):
    guard = 4096
    a = _src(nbytes, 2 + direct_loads)
    b = torch.full((guard + nbytes + guard,), 0xEE, dtype=torch.uint8, device=DEV)
    stream = torch.cuda.Stream()
    stream.wait_stream(torch.cuda.current_stream())
    K.check(K.tc_copy_via_lds(b[guard:], a, nbytes, direct_loads, stream))
    stream.synchronize()
    assert torch.equal(b[guard:guard + nbytes], a)
    assert bool((b[:guard] == 0xEE).all()) and bool((b[guard + nbytes:] == 0xEE).all())


def test_helpers_reject_sizes_and_alignments_their_kernels_cannot_take():
    a = torch.zeros(1 << 16, dtype=torch.uint8, device=DEV)
    b = torch.zeros(1 << 16, dtype=torch.uint8, device=DEV)
    assert K.tc_copy_contiguous(b, a, 24) == K.TC_ERR_INVAL                 # not a multiple of 16
    assert K.tc_copy_contiguous(b[8:], a, 32) == K.TC_ERR_INVAL             # misaligned
    assert K.tc_copy_contiguous(None, a, 32) == K.TC_ERR_INVAL
    assert K.tc_copy_contiguous(b, a, 0) == K.TC_OK
    assert K.tc_copy_via_lds(b, a, 16384 + 16, 0) == K.TC_ERR_INVAL         # whole tiles only
    assert K.tc_copy_via_lds(b[16:], a[8:], 16384, 1) == K.TC_ERR_INVAL
    assert K.tc_copy_via_lds(b, a, 0, 1) == K.TC_OK
    torch.cuda.synchronize()


def test_hbm_stream_computes_the_triad():
    n = (1 << 20) + 4 * 37
    g = torch.Generator(device=DEV)
    g.manual_seed(9)
    b = torch.randn(n, device=DEV, generator=g)
    c = torch.randn(n, device=DEV, generator=g)
    a = torch.zeros(n, device=DEV)
    stream = torch.cuda.Stream()
    stream.wait_stream(torch.cuda.current_stream())
    K.check(K.tc_hbm_stream(a, b, c, n, 0.5, 2, stream))
    stream.synchronize()
    # a = b + 0.5 * c in fp32: multiplying by 0.5 is exact, so fused or not the result is the rounded sum
    assert torch.equal(a, b + 0.5 * c)
    assert K.tc_hbm_stream(a, b, c, n + 1, 0.5, 1, stream) == K.TC_ERR_INVAL
