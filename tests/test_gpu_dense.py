"""GPU parity for the dense steps: GCN update (paper Section 3.5, Listing 1) and the GRU / LSTM step
(Section 3.3: three and four gates), each against the fp64 CPU reference."""
import numpy as np
import pytest

import oracle
from helpers import RTOL_BF16, RTOL_FP32, assert_close
from paper_2501_15348_amd import synth

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ctx():
    from paper_2501_15348_amd import reinc

    c = reinc.Context(64, 1, (16, 16), "gru", 16, "sum", True, arena_bytes=1 << 20)
    yield c
    c.close()


def _dev(a, dtype=None):
    import torch

    t = torch.from_numpy(np.ascontiguousarray(a)).cuda()
    return t if dtype is None else t.to(dtype)


@pytest.mark.parametrize("n,k,m,relu,scale,bias", [
    (1000, 16, 16, True, False, True),
    (5003, 64, 64, True, True, True),
    (4099, 128, 128, True, True, False),
    (3001, 256, 128, True, False, True),
    (777, 64, 192, False, False, True),
    (513, 100, 72, False, True, True),   # widths that are no multiple of the tile
    (129, 256, 512, True, False, True),
    (31, 8, 40, False, False, False),
    (2077, 512, 128, False, True, False),   # deep product: two passes over the halves of K
    (2077, 512, 128, True, False, True),    # the same depth with bias and ReLU: single pass
    (1500, 384, 256, False, False, False),
])
def test_gcn_transform(ctx, n, k, m, relu, scale, bias):
    rng = np.random.default_rng(n + k + m)
    a = rng.standard_normal((n, k)).astype(np.float32)
    w = (rng.standard_normal((k, m)) / np.sqrt(k)).astype(np.float32)
    b = rng.standard_normal(m).astype(np.float32) if bias else None
    rs = rng.uniform(0.1, 1.0, n).astype(np.float32) if scale else None
    ref = oracle.dense_layer(a.astype(np.float64) * (rs[:, None] if scale else 1.0), w, b, relu)
    out = ctx.gcn_transform(_dev(a), _dev(w), _dev(b) if bias else None, _dev(rs) if scale else None, relu=relu)
    assert_close(out.cpu().numpy(), ref, RTOL_FP32, f"gcn_transform {n}x{k}x{m}")


def test_gcn_transform_identity_weight(ctx):
    import torch

    a = np.random.default_rng(0).standard_normal((300, 64)).astype(np.float32)
    out = ctx.gcn_transform(_dev(a), torch.eye(64, device="cuda"), None, None, relu=True)
    assert np.array_equal(out.cpu().numpy(), np.maximum(a, 0))


def test_gcn_transform_bf16_input(ctx):
    import torch

    rng = np.random.default_rng(5)
    a = synth.round_to_bf16(rng.standard_normal((2049, 256)).astype(np.float32))
    w = (rng.standard_normal((256, 256)) / 16).astype(np.float32)
    ref = oracle.dense_layer(a, w, None, True)
    out = ctx.gcn_transform(_dev(a, torch.bfloat16), _dev(w), None, None, relu=True)
    assert_close(out.cpu().numpy(), ref, RTOL_BF16, "bf16 input")


@pytest.mark.parametrize("kind,n,d,h,zero_state", [
    ("gru", 1000, 16, 16, False),
    ("gru", 4099, 64, 64, False),
    ("gru", 4099, 64, 64, True),
    ("gru", 1027, 128, 128, False),
    ("lstm", 2051, 128, 128, False),
    ("lstm", 2051, 128, 128, True),
    ("lstm", 333, 24, 40, False),
    ("gru", 65, 100, 48, False),
])
def test_rnn_step(ctx, kind, n, d, h, zero_state):
    import torch

    rng = np.random.default_rng(n + d + h)
    kg = 3 if kind == "gru" else 4
    x = rng.standard_normal((n, d)).astype(np.float32)
    hp = np.zeros((n, h), np.float32) if zero_state else rng.standard_normal((n, h)).astype(np.float32)
    cp = np.zeros((n, h), np.float32) if zero_state else rng.standard_normal((n, h)).astype(np.float32)
    wi = (rng.standard_normal((d, kg * h)) / np.sqrt(d)).astype(np.float32)
    wh = (rng.standard_normal((h, kg * h)) / np.sqrt(h)).astype(np.float32)
    bi = rng.standard_normal(kg * h).astype(np.float32) * 0.3
    bh = rng.standard_normal(kg * h).astype(np.float32) * 0.3
    saved = torch.empty((n, 4 * h), device="cuda")
    h_out, c_out = ctx.rnn_step(kind, _dev(x), None if zero_state else _dev(hp), None if zero_state or kind == "gru" else _dev(cp),
                                _dev(wi), _dev(wh), _dev(bi), _dev(bh), saved)
    f = lambda a: a.astype(np.float64)
    if kind == "gru":
        ref_h, gates = oracle.gru_cell(f(x), f(hp), f(wi), f(wh), f(bi), f(bh))
    else:
        ref_h, ref_c, gates = oracle.lstm_cell(f(x), f(hp), f(cp), f(wi), f(wh), f(bi), f(bh))
        assert_close(c_out.cpu().numpy(), ref_c, RTOL_FP32, "c")
    assert_close(h_out.cpu().numpy(), ref_h, RTOL_FP32, "h")
    assert_close(saved.cpu().numpy(), np.concatenate(gates, axis=1), RTOL_FP32, "saved gates")


def test_zero_weights_closed_form(ctx):
    import torch

    n, d, h = 200, 16, 32
    x = torch.randn(n, d, device="cuda")
    hp = torch.randn(n, h, device="cuda")
    cp = torch.randn(n, h, device="cuda")
    z = lambda *s: torch.zeros(*s, device="cuda")
    out, _ = ctx.rnn_step("gru", x, hp, None, z(d, 3 * h), z(h, 3 * h), z(3 * h), z(3 * h))
    assert torch.allclose(out, 0.5 * hp, atol=1e-7)
    out, c = ctx.rnn_step("lstm", x, hp, cp, z(d, 4 * h), z(h, 4 * h), z(4 * h), z(4 * h))
    assert torch.allclose(c, 0.5 * cp, atol=1e-7) and torch.allclose(out, 0.5 * torch.tanh(0.5 * cp), atol=1e-6)


def test_fp32_instruction_path_in_a_child_process():
    """REINC_DENSE=fp32 keeps the dense kernels on the fp32 matrix instructions; the switch is read once per process,
    so the cases above are run again in one child process with it set."""
    import os
    import subprocess
    import sys

    if os.environ.get("REINC_DENSE") == "fp32":
        pytest.skip("this is the child")
    env = dict(os.environ, REINC_DENSE="fp32")
    here = os.path.abspath(__file__)
    out = subprocess.run([sys.executable, "-m", "pytest", here, "-q", "-x", "-m", "gpu", "-p", "no:cacheprovider"], env=env,
                         cwd=os.path.dirname(os.path.dirname(here)), capture_output=True, text=True, timeout=600)
    assert out.returncode == 0, out.stdout[-3000:] + out.stderr[-2000:]
