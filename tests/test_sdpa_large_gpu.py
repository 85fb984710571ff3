"""Sizes at the limits the entry points accept (through the C-ABI, against the float64 CPU oracle).

* tensors of more than 2^31 elements (more than 4 GiB each): every head offset, output index and
  statistics index beyond 32 bits; heads on both sides of the 2^31-element boundary are checked;
* the longest key sequence one head may have (its K and V just below the 2^30-byte range a buffer
  descriptor of the kernel covers), as a decoding step with and without splitting the key range.

The inputs are seeded normal tensors drawn on the device (the host generator would take minutes at
these sizes); the slices the oracle checks are copied back.
"""
import sys

import numpy as np
import pytest
import torch

from oracle import sdpa_oracle as orc
from paper_2603_01960_amd import binding

pytestmark = pytest.mark.gpu

TOL = {"f16": 2e-3, "bf16": 1.6e-2}
LSE_TOL = 1e-4


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


@pytest.fixture(scope="module", autouse=True)
def _device():
    assert torch.cuda.is_available(), "these tests need the MI355X"
    binding.load_library()
    yield
    torch.cuda.synchronize()
    torch.cuda.empty_cache()


def device_normal(shape, dtype, seed):
    g = torch.Generator(device="cuda").manual_seed(seed)
    return torch.randn(*shape, dtype=dtype, device="cuda", generator=g)


def f64(t):
    return t.float().cpu().numpy()


def test_tensors_beyond_2_to_31_elements_forward_and_backward():
    B, H, S, D, dtype = 1, 1100, 16384, 128, torch.bfloat16
    assert B * H * S * D > 2 ** 31
    say(f"[case] large tensors B={B} H={H} S={S} D={D} bf16: {B * H * S * D * 2 / 2 ** 30:.2f} GiB per tensor")
    q, k, v, do = (device_normal((B, H, S, D), dtype, 900 + i) for i in range(4))
    o, lse = binding.sdpa(q, k, v, causal=True, return_lse=True)
    dq, dk, dv = binding.sdpa_backward(q, k, v, o, do, lse, causal=True)
    torch.cuda.synchronize()
    rows = [0, 1, 127, 128, 4095, 8192, 16000, S - 1]
    boundary = 2 ** 31 // (S * D)                       # first head that starts at element 2^31
    for h in (0, boundary - 1, boundary, H - 1):
        say(f"        head {h}")
        sl = lambda t: f64(t[:, h:h + 1])
        ref_o, ref_lse = orc.sdpa(sl(q), sl(k), sl(v), rows=rows, return_lse=True, causal=True)
        err = float(np.abs(o[:, h:h + 1][:, :, rows].double().cpu().numpy() - ref_o).max())
        lerr = float(np.abs(lse[:, h:h + 1][:, :, rows].double().cpu().numpy() - ref_lse).max())
        say(f"        forward max|dO|={err:.3e} max|dLSE|={lerr:.3e}")
        assert err <= TOL["bf16"] and lerr <= LSE_TOL * max(1.0, float(np.abs(ref_lse).max()) / 16)
        ref = orc.sdpa_bwd(sl(q), sl(k), sl(v), sl(do), causal=True, qrows=rows, krows=rows, scale=None)
        for name, g, r in zip(("dq", "dk", "dv"), (dq, dk, dv), ref):
            got = g[:, h:h + 1][:, :, rows].double().cpu().numpy()
            assert np.isfinite(got).all()
            e = float(np.abs(got - r).max())
            bound = TOL["bf16"] * max(1.0, float(np.abs(r).max()))
            say(f"        {name}: max|err|={e:.3e} bound={bound:.3e}")
            assert e <= bound, f"head {h}: {name} error {e} > {bound}"
    # untouched neighbours: the output of one head does not depend on any other head
    assert torch.isfinite(o[:, ::97].float()).all()


@pytest.mark.parametrize("D", [64, 128])
def test_longest_key_sequence_of_one_head_as_a_decoding_step(D):
    skv_max = (1 << 30) // (2 * D) - 1025               # (Skv + 1024) * D * 2 < 2^30
    B, H, Sq, dtype = 1, 2, 1, torch.float16
    say(f"[case] longest cache D={D}: Skv={skv_max} ({skv_max * D * 2 / 2 ** 20:.0f} MiB of K per head)")
    st = binding.tiled_sdpa_fwd_kv(None, None, None, None, None, B, H, Sq, skv_max + 1, D, float("nan"),
                                   binding.F16, None)
    assert st == 2, "one row more must be refused as a bad shape"
    q = device_normal((B, H, Sq, D), dtype, 910)
    k = device_normal((B, H, skv_max, D), dtype, 911)
    v = device_normal((B, H, skv_max, D), dtype, 912)
    refs = None
    for splits in (0, 1, 128):
        o, lse = binding.sdpa_kv(q, k, v, splits=splits, return_lse=True)
        torch.cuda.synchronize()
        if refs is None:
            refs = orc.sdpa(f64(q), f64(k), f64(v), return_lse=True)
        err = float(np.abs(o.double().cpu().numpy() - refs[0]).max())
        lerr = float(np.abs(lse.double().cpu().numpy() - refs[1]).max())
        say(f"        splits={splits}: max|dO|={err:.3e} max|dLSE|={lerr:.3e}")
        assert err <= TOL["f16"] and lerr <= LSE_TOL * max(1.0, float(np.abs(refs[1]).max()) / 16)
