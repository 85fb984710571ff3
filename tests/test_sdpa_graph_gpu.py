"""The entry points allocate nothing, synchronise nothing and set no memory: a caller can record them
into a HIP graph.  Forward, split-KV forward (+ merge) and backward are captured once with
caller-owned outputs and workspaces and replayed several times with eager launches and
synchronisations in between; every replay must reproduce the eager result bit for bit (all
reductions run in a fixed order), also after the inputs were overwritten in place.
"""
import sys

import pytest
import torch

from paper_2603_01960_amd import binding
from paper_2603_01960_amd.workloads import make_qkv

pytestmark = pytest.mark.gpu


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


@pytest.fixture(scope="module", autouse=True)
def _device():
    assert torch.cuda.is_available(), "these tests need the MI355X"
    binding.load_library()
    yield
    torch.cuda.synchronize()


def _refill(tensors, seed):
    """New seeded values written into the SAME device buffers (what a graph replays on)."""
    g = torch.Generator(device="cpu").manual_seed(seed)
    for t in tensors:
        t.copy_(torch.randn(*t.shape, dtype=torch.float32, generator=g).to(t.dtype))


def _capture(run):
    """Warm up eagerly on a side stream (first calls set kernel attributes), then record `run`."""
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        for _ in range(2):
            run()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        run()
    return graph


@pytest.mark.parametrize("causal", [False, True])
def test_forward_replays_bit_exactly(causal):
    say(f"[case] graph forward causal={causal}")
    q, k, v = (t.cuda() for t in make_qkv(2, 3, 333, 128, "bf16", seed=21))
    o = torch.empty_like(q)
    lse = torch.empty(2, 3, 333, dtype=torch.float32, device="cuda")
    run = lambda: binding.sdpa(q, k, v, causal=causal, out=o, lse_out=lse, return_lse=True)
    graph = _capture(run)
    for rep in range(4):
        _refill((q, k, v), 100 + rep)
        o_ref, lse_ref = binding.sdpa(q, k, v, causal=causal, return_lse=True)      # eager, own outputs
        torch.cuda.synchronize()
        o.fill_(float("nan")); lse.fill_(float("nan"))
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(o, o_ref), f"replay {rep}: O differs from the eager launch"
        assert torch.equal(lse, lse_ref), f"replay {rep}: LSE differs from the eager launch"


def test_split_kv_forward_and_merge_replay_bit_exactly():
    say("[case] graph split-KV forward + merge")
    B, H, Sq, Skv, D, splits = 1, 4, 1, 4096, 128, 8
    q = make_qkv(B, H, Sq, D, "f16", seed=31)[0].cuda()
    _, k, v = (t.cuda() for t in make_qkv(B, H, Skv, D, "f16", seed=32))
    o = torch.empty_like(q)
    ws = torch.empty(binding.kv_workspace_bytes(B, H, Sq, D, splits), dtype=torch.uint8, device="cuda")
    run = lambda: binding.sdpa_kv(q, k, v, splits=splits, out=o, workspace=ws)
    graph = _capture(run)
    for rep in range(4):
        _refill((q, k, v), 200 + rep)
        o_ref = binding.sdpa_kv(q, k, v, splits=splits)
        torch.cuda.synchronize()
        o.fill_(float("nan")); ws.fill_(0xFF)       # stale partial states must not leak into a replay
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(o, o_ref), f"replay {rep}: O differs from the eager launch"


def test_backward_replays_bit_exactly():
    say("[case] graph backward")
    B, H, S, D = 1, 2, 300, 64
    q, k, v = (t.cuda() for t in make_qkv(B, H, S, D, "bf16", seed=41))
    dout = torch.empty_like(q)
    o = torch.empty_like(q)
    lse = torch.empty(B, H, S, dtype=torch.float32, device="cuda")
    grads = tuple(torch.empty_like(q) for _ in range(3))
    ws = torch.empty(binding.bwd_workspace_bytes(B, H, S), dtype=torch.uint8, device="cuda")

    def run():      # forward and backward in one graph, as a training step would record them
        binding.sdpa(q, k, v, causal=True, out=o, lse_out=lse, return_lse=True)
        binding.sdpa_backward(q, k, v, o, dout, lse, causal=True, workspace=ws, grads=grads)

    _refill((dout,), 40)
    graph = _capture(run)
    for rep in range(4):
        _refill((q, k, v, dout), 300 + rep)
        o_ref, lse_ref = binding.sdpa(q, k, v, causal=True, return_lse=True)
        ref = binding.sdpa_backward(q, k, v, o_ref, dout, lse_ref, causal=True)
        torch.cuda.synchronize()
        for g in grads:
            g.fill_(float("nan"))
        ws.fill_(0xFF)
        graph.replay()
        torch.cuda.synchronize()
        for name, got, want in zip(("dq", "dk", "dv"), grads, ref):
            assert torch.equal(got, want), f"replay {rep}: {name} differs from the eager launch"


def test_host_threads_on_their_own_streams_do_not_disturb_each_other():
    """The library keeps no state besides its kernel table (set up under std::call_once): four host
    threads launch different problems on their own streams at the same time, each repeatedly, and every
    result must equal the one computed alone."""
    import threading

    say("[case] four host threads, four streams")
    problems = []
    for i, (S, D, dtype, causal) in enumerate([(700, 128, "bf16", False), (333, 64, "f16", True),
                                               (1024, 96, "bf16", True), (150, 160, "f16", False)]):
        q, k, v = (t.cuda() for t in make_qkv(2, 4, S, D, dtype, seed=500 + i))
        ref = binding.sdpa(q, k, v, causal=causal, return_lse=True)
        problems.append((q, k, v, causal, ref))
    torch.cuda.synchronize()
    failures = []

    def work(idx):
        q, k, v, causal, (o_ref, lse_ref) = problems[idx]
        stream = torch.cuda.Stream()
        try:
            with torch.cuda.stream(stream):
                for rep in range(20):
                    o, lse = binding.sdpa(q, k, v, causal=causal, return_lse=True)
                    stream.synchronize()
                    if not (torch.equal(o, o_ref) and torch.equal(lse, lse_ref)):
                        failures.append((idx, rep))
        except Exception as e:          # surfaced below: an exception in a thread would otherwise be lost
            failures.append((idx, repr(e)))

    threads = [threading.Thread(target=work, args=(i,)) for i in range(4)]
    for t in threads:
        t.start()
    for t in threads:
        t.join(timeout=100)
    assert not any(t.is_alive() for t in threads), "a worker did not finish"
    assert not failures, failures
