"""gsr_spmm_noalloc, the entry point for callers that cannot allocate: same results as gsr_spmm, bit for bit,
on two calls in a row that share the library's fixed scratch array, the second on a smaller input."""
import numpy as np
import pytest
import torch

import paper_2603_27156_amd as gsr
from paper_2603_27156_amd import synth

pytestmark = pytest.mark.gpu


def _graph(n, seed):
    w = synth.scaled(synth.workload(2), n)
    rng = np.random.Generator(np.random.PCG64(seed))
    rp, ci = synth.circuit_dag(w, rng)
    return gsr.gsr_graph_create(rp, ci)


def test_spmm_noalloc_matches_spmm_on_two_calls_in_a_row():
    dev = torch.device("cuda:0")
    # rows above 6 stored entries are split, so both the counters and the first-pass sums of the scratch are used
    gsr.gsr_set_option("hub_threshold", 6)
    gsr.gsr_set_option("hub_chunk", 4)
    try:
        big, small, too_big = _graph(9001, 3), _graph(3001, 4), _graph(20011, 3)
    finally:
        gsr.gsr_set_option("hub_threshold", 0)
        gsr.gsr_set_option("hub_chunk", 0)
    assert gsr.gsr_graph_info(big)["n_hub_rows"] > 100 and gsr.gsr_graph_info(small)["n_hub_rows"] > 10
    rng = np.random.default_rng(5)
    for g, n in ((big, 9001), (small, 3001)):          # the second call: smaller input, stale scratch contents
        for width in (64, 32):
            x = torch.from_numpy(rng.standard_normal((n, width)).astype(np.float32)).to(dev)
            for transpose in (False, True):
                want = gsr.gsr_spmm(g, x, transpose=transpose)
                got = torch.full_like(want, float("nan"))
                # allocations made through torch's allocator since the process started (frees by the garbage collector,
                # which other tests' tensors may meet here, do not count)
                before = torch.cuda.memory_stats().get("allocation.all.allocated", 0)
                gsr.gsr_spmm_noalloc(g, x, got, transpose=transpose)
                assert torch.cuda.memory_stats().get("allocation.all.allocated", 0) == before
                torch.cuda.synchronize()
                assert torch.equal(got, want), (n, width, transpose)
    # a width without a tiled path takes the row-per-wave kernel, which needs no scratch at all
    x = torch.from_numpy(rng.standard_normal((3001, 24)).astype(np.float32)).to(dev)
    got = torch.empty_like(x)
    gsr.gsr_spmm_noalloc(small, x, got)
    assert torch.equal(got, gsr.gsr_spmm(small, x))
    # more first-pass chunks than the fixed array holds: refused with a message, nothing launched
    x = torch.zeros((20011, 64), dtype=torch.float32, device=dev)
    with pytest.raises(gsr.GsrError) as e:
        gsr.gsr_spmm_noalloc(too_big, x, torch.empty_like(x))
    assert e.value.status == gsr.GSR_ERR_UNSUPPORTED and "16384" in str(e.value)
