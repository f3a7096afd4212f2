"""The library's calls only launch kernels on the caller's stream (no allocation, no
synchronisation, no memset), so they can be recorded into a HIP graph.  Each replay is
checked against the eager result, with eager work and synchronisations between replays."""
import numpy as np
import pytest
import torch

from paper_2601_15473_amd import workloads as W
from paper_2601_15473_amd.device import DeviceLayer

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def sk():
    from paper_2601_15473_amd import libsk
    yield libsk
    libsk.sk_set_plan(0)


CASES = [
    W.scaled(W.BERT_BASE_FFN_UP, tokens=1000),      # fused forward, split + expand input gradient
    W.scaled(W.BERT_LARGE_FFN_UP, tokens=600),      # two GEMMs per call
    W.scaled(W.BY_NAME["grid8192_l1_k16"], tokens=300),   # split first contractions, sum-to-bf16 kernel
]


@pytest.mark.parametrize("w", CASES, ids=lambda w: f"{w.name}_T{w.tokens}")
def test_calls_replay_from_a_graph(sk, w):
    sk.sk_set_plan(0)
    t = W.generate(w)
    eager = DeviceLayer(t, sk)
    eager.run_all()
    ref = {n: getattr(eager, n).clone() for n in ("y", "dX", "dU", "db")}

    dev = DeviceLayer(t, sk, poison=False)
    stream = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(stream):
        # one eager pass on the capture stream first (nothing in the library is lazily set up,
        # but the first launch of a kernel loads its code object)
        for st in (dev.fwd(stream), dev.bwd_input(stream), dev.bwd_weight(stream)):
            sk.check(st)
    torch.cuda.synchronize()
    with torch.cuda.graph(graph, stream=stream):
        cap = torch.cuda.current_stream()
        for st in (dev.fwd(cap), dev.bwd_input(cap), dev.bwd_weight(cap)):
            sk.check(st)
    for rep in range(3):
        for n in ("y", "dX", "dU", "db"):
            getattr(dev, n).fill_(float("nan"))     # eager work between the replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for n in ("y", "dX", "dU", "db"):
            got, want = getattr(dev, n), ref[n]
            assert torch.equal(got.view(torch.int16 if got.dtype == torch.bfloat16 else torch.int32),
                               want.view(torch.int16 if want.dtype == torch.bfloat16 else torch.int32)), (rep, n)


STEP_CASES = [
    W.scaled(W.BERT_BASE_FFN_UP, tokens=1000),      # backward pass with shared launches, sums carried by the expansion
    W.scaled(W.BERT_LARGE_FFN_UP, tokens=5000),     # two dual launches + the split sum
    W.scaled(W.BERT_BASE_PROJ[0], tokens=700),      # one-pass backward (32-token tiles) + the sum of the tiles' slabs
    W.scaled(W.BERT_BASE_PROJ[0], tokens=9000),     # ... with 64-token tiles
]


@pytest.mark.parametrize("w", STEP_CASES, ids=lambda w: f"{w.name}_T{w.tokens}")
def test_timed_step_replays_from_a_graph(sk, w):
    """The benchmark's step (sk_linear_fwd + sk_linear_bwd) recorded once and replayed."""
    sk.sk_set_plan(0)
    t = W.generate(w)
    eager = DeviceLayer(t, sk)
    sk.check(eager.fwd())
    sk.check(eager.bwd())
    torch.cuda.synchronize()
    ref = {n: getattr(eager, n).clone() for n in ("y", "dX", "dU", "db")}

    dev = DeviceLayer(t, sk, poison=False)
    stream = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(stream):
        for st in (dev.fwd(stream), dev.bwd(stream)):
            sk.check(st)
    torch.cuda.synchronize()
    with torch.cuda.graph(graph, stream=stream):
        cap = torch.cuda.current_stream()
        for st in (dev.fwd(cap), dev.bwd(cap)):
            sk.check(st)
    for rep in range(3):
        for n in ("y", "dX", "dU", "db"):
            getattr(dev, n).fill_(float("nan"))     # eager work between the replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for n in ("y", "dX", "dU", "db"):
            got, want = getattr(dev, n), ref[n]
            assert torch.equal(got.view(torch.int16 if got.dtype == torch.bfloat16 else torch.int32),
                               want.view(torch.int16 if want.dtype == torch.bfloat16 else torch.int32)), (rep, n)
