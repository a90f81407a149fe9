"""GPU: the allocation-free entry point gives the message of atomo_encode_entrywise, bit for bit, on two calls
in a row (the second on a smaller input, so what the first left in the shared scratch array must not matter)."""
import ctypes as C

import numpy as np
import pytest
import torch

from paper_1806_04090_amd import binding, inputs
from gpu_common import ctx, dev

pytestmark = pytest.mark.gpu


def both(g, s, seed, stream_id, capacity):
    d = dev(g)
    p_a = torch.zeros(g.size, device="cuda")
    p_b = torch.full((g.size,), -1.0, device="cuda")
    ref = binding.alloc_entrywise_message(g.size, capacity, "cuda")
    binding.atomo_encode_entrywise(ctx(), d, s, seed, stream_id, msg=ref, p_out=p_a)
    got = binding.alloc_entrywise_message(g.size, capacity, "cuda")
    got.idx.fill_(-1)
    got.val.fill_(float("nan"))
    got.count.fill_(-7)
    binding.atomo_encode_entrywise_noalloc(ctx(), d, s, seed, stream_id, got, p_out=p_b)
    torch.cuda.synchronize()
    a, b = ref.to_host(), got.to_host()
    assert a["count"] == b["count"] and a["count"] > 0
    assert np.array_equal(a["idx"], b["idx"])
    assert np.array_equal(a["val"], b["val"])
    assert np.array_equal(p_a.cpu().numpy(), p_b.cpu().numpy())
    return a["count"]


def test_two_calls_in_a_row_match_the_allocating_entry_point():
    big = inputs.flat_heavy_tail(seed=3, n=1_000_003)
    small = inputs.flat_heavy_tail(seed=4, n=70_001, heavy_fraction=0.01)
    k1 = both(big, 10_000.0, 11, 5, binding.default_capacity(10_000.0, big.size))
    k2 = both(small, 300.0, 12, 6, binding.default_capacity(300.0, small.size))
    assert k1 > k2
    assert ctx().status()[0] == 0


def test_rejects_inputs_beyond_the_fixed_scratch_and_bad_arguments():
    L = binding.lib()
    n = (1 << 24) + 1
    msg = binding.alloc_entrywise_message(16, 16, "cuda")
    cm = msg.c_struct()
    cm.n = n                                                    # rejected before anything is read or enqueued
    g = torch.zeros(16, device="cuda")
    assert L.atomo_encode_entrywise_noalloc(ctx()._h, g.data_ptr(), 1.0, 0, 0, C.byref(cm), None, None) == binding.ATOMO_ETOOLARGE
    assert b"scratch" in L.atomo_strerror(binding.ATOMO_ETOOLARGE)
    cm.n = 16
    assert L.atomo_encode_entrywise_noalloc(ctx()._h, None, 1.0, 0, 0, C.byref(cm), None, None) == binding.ATOMO_EINVAL
    assert L.atomo_encode_entrywise_noalloc(ctx()._h, g.data_ptr(), 0.0, 0, 0, C.byref(cm), None, None) == binding.ATOMO_EINVAL
    assert L.atomo_encode_entrywise_noalloc(None, g.data_ptr(), 1.0, 0, 0, C.byref(cm), None, None) == binding.ATOMO_EINVAL


def test_the_largest_supported_length():
    n = 1 << 24
    g = torch.empty(n, device="cuda").normal_(0.0, 1e-3)
    s = n / 100
    ref = binding.alloc_entrywise_message(n, binding.default_capacity(s, n), "cuda")
    got = binding.alloc_entrywise_message(n, binding.default_capacity(s, n), "cuda")
    binding.atomo_encode_entrywise(ctx(), g, s, 1, 2, msg=ref)
    binding.atomo_encode_entrywise_noalloc(ctx(), g, s, 1, 2, got)
    torch.cuda.synchronize()
    a, b = ref.to_host(), got.to_host()
    assert a["count"] == b["count"] and np.array_equal(a["idx"], b["idx"]) and np.array_equal(a["val"], b["val"])
    assert ctx().status()[0] == 0
