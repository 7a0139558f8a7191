"""The entry point for callers that cannot allocate (hcl_reduce_scatter_sim_static):
its partial sums live in the library's fixed scratch array.  Its result must be
the bits hcl_reduce_scatter_sim produces with a caller-supplied workspace (and
the oracle's), on two calls in a row that share the array, the second smaller."""
import numpy as np
import pytest
import torch

import workloads as wl
from gpu_util import CODE, assert_same_bits, device_inputs, fresh
from oracle import ring_oracle as orc
from paper_2601_22585_amd import hcl

pytestmark = pytest.mark.gpu


def _both(seed, W, n, dtype, dist, chunk_bytes, ring=None):
    cpu, dev = device_inputs(seed, W, W * n, dtype, dist)
    need = hcl.workspace_bytes(hcl.KIND_REDUCE_SCATTER, W, n, CODE[dtype], chunk_bytes)
    assert 0 < need <= hcl.static_scratch_bytes()
    ws = torch.empty(need, dtype=torch.uint8, device="cuda")
    a = fresh(W, n, dtype, fill=0)
    b = fresh(W, n, dtype, fill=0)
    la = hcl.reduce_scatter_sim(dev, a, chunk_bytes=chunk_bytes, ring=ring, workspace=ws)
    lb = hcl.reduce_scatter_sim_static(dev, b, chunk_bytes=chunk_bytes, ring=ring)
    torch.cuda.synchronize()
    assert la == lb == W - 1
    want = orc.reduce_scatter([wl.to_wire(t) for t in cpu], CODE[dtype], ring=ring,
                              chunk_elems=chunk_bytes // wl.ESIZE[dtype])
    for r in range(W):
        assert np.array_equal(wl.to_wire(a[r]), wl.to_wire(b[r])), (W, n, dtype, r)
        assert_same_bits(b[r], want[r], dtype, f"static scratch W={W} n={n} {dtype} rank {r}")
        assert_same_bits(dev[r], wl.to_wire(cpu[r]), dtype, f"send[{r}] must stay untouched")


def test_static_scratch_reduce_scatter_two_calls_in_a_row():
    # the first call fills nearly all of the array, the second reuses its head with other data
    _both(900, 8, 2_000_003, "bf16", ("normal", 0.0, 1e-3), 64 * 1024)
    _both(901, 5, 70_001, "fp32", ("uniform", -1.0, 1.0), 0, ring=[3, 0, 4, 1, 2])
    _both(902, 16, 9, "fp16", ("normal", 0.0, 1.0), 0)


def test_static_scratch_limit_and_forms_that_need_no_scratch():
    W, dtype = 4, "int32"
    limit = hcl.static_scratch_bytes()
    n_max = (limit // W - 4096) // 4                   # largest block whose W slots (block + 4 KiB each) fit
    assert hcl.workspace_bytes(hcl.KIND_REDUCE_SCATTER, W, n_max, CODE[dtype]) == limit
    cpu, dev = device_inputs(903, W, W * (n_max + 64), dtype, ("randint", -1000, 1000))
    out = fresh(W, n_max + 64, dtype, fill=0)
    # exactly at the limit: runs, and equals the plain integer sum
    hcl.reduce_scatter_sim_static([t[:W * n_max] for t in dev], [t[:n_max] for t in out])
    torch.cuda.synchronize()
    for r in range(W):
        tot = sum(t[r * n_max:(r + 1) * n_max].to(torch.int64) for t in dev).to(torch.int32)
        assert torch.equal(out[r][:n_max], tot)
        assert bool((out[r][n_max:] == 0).all())
    # one 256-byte granule beyond: refused, nothing launched
    with pytest.raises(hcl.HclError) as e:
        hcl.reduce_scatter_sim_static(dev, out)
    assert e.value.status == "HCL_ERR_WORKSPACE"
    # the FUSED schedule and the in-place form keep no partial sums outside the buffers: any size goes
    hcl.reduce_scatter_sim_static(dev, out, sched="fused")
    n = n_max + 64
    inpl = [dev[r][r * n:(r + 1) * n] for r in range(W)]
    want = [sum(t[r * n:(r + 1) * n].to(torch.int64) for t in dev).to(torch.int32) for r in range(W)]
    hcl.reduce_scatter_sim_static(dev, inpl)
    torch.cuda.synchronize()
    for r in range(W):
        assert torch.equal(out[r], want[r])
        assert torch.equal(inpl[r], want[r])
