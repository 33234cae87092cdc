"""jq_evict_static -- the fused eviction for callers that cannot allocate (its scratch memory is a fixed device array
inside the library) -- against jq_evict on the same inputs, through the C ABI: two calls in a row, the second on a
smaller problem, so that what the first call left in the shared array must not matter."""
import numpy as np
import pytest

import paper_2509_10798_amd as jq
from parity import to_dev_bf16
from workloads import make_workload

pytestmark = pytest.mark.gpu


def run_both(torch, w):
    Q, K, V = w.assemble()
    Qd, Kd, Vd = to_dev_bf16(Q), to_dev_bf16(K), to_dev_bf16(V)
    sh = jq.Shape(n_layers=w.n_layers, seq_lens=w.seq_lens, n_q=w.n_q, h_q=w.h_q, h_kv=w.h_kv, pool_k=w.pool_k,
                  budgets=w.budgets)
    assert jq.workspace_bytes(sh) <= jq.STATIC_WS_BYTES
    ref = jq.evict(sh, Qd, Kd, Vd)
    Ko = torch.full_like(ref[0], 1.5); Vo = torch.full_like(ref[1], 1.5)
    idx = torch.full_like(ref[2], -7); pooled = torch.full_like(ref[3], -1.0)
    before = torch.cuda.memory_allocated()
    jq.evict_static(sh, Qd, Kd, Vd, Ko, Vo, idx, pooled)
    assert torch.cuda.memory_allocated() == before          # nothing came from torch's allocator either
    torch.cuda.synchronize()
    assert torch.equal(idx, ref[2]) and torch.equal(pooled, ref[3])
    assert torch.equal(Ko.view(torch.int16), ref[0].view(torch.int16))
    assert torch.equal(Vo.view(torch.int16), ref[1].view(torch.int16))


def test_static_scratch_eviction_equals_jq_evict_twice_in_a_row():
    import torch
    assert torch.cuda.is_available(), "this test needs the GPU"
    print("static scratch: 2 layers x (5000, 1300) tokens", flush=True)
    run_both(torch, make_workload(1, seq_lens=[5000, 1300], budget=[600, 100], n_layers=2))
    print("static scratch: 1 layer x 700 tokens", flush=True)
    run_both(torch, make_workload(1, seq_lens=[700], budget=[64], n_layers=1))   # smaller: stale scratch contents all around


def test_static_scratch_rejects_problems_beyond_its_size():
    import ctypes
    sh = jq.Shape(n_layers=4, seq_lens=[131072], n_q=32, h_q=32, h_kv=8, budgets=[2048])
    assert jq.workspace_bytes(sh) > jq.STATIC_WS_BYTES
    cs = sh.c_struct()
    big = 1 << 40
    rc = jq.lib().jq_evict_static(ctypes.byref(cs), big, big + (1 << 34), big + (2 << 34), big + (3 << 34), big + (4 << 34),
                                  None, None, None)
    assert rc == -5
