"""Pins of the QKNorm-before-attention oracle (the paper's QKNorm benchmark: layer normalisation of
the query and key vectors before attention), CPU only.  None of them re-types the oracle's formula:
a closed form, invariances, degenerate cases with a known answer, and a library evaluation."""
import numpy as np
import pytest

import oracle
import workloads


def _w(a):
    return np.asarray(a, dtype=np.float32)


ONE2, ZERO2 = _w([1, 1]), _w([0, 0])


def test_closed_form_d2():
    """D = 2, eps = 0, unit gain, no bias: a normalised vector is (+1, -1) or (-1, +1), so a score is
    +-2 / sqrt(2) = +-sqrt(2) and two opposite keys get the weights 1 / (1 + exp(-+2 sqrt 2))."""
    q = _w([[[3.0, 1.0]]])                        # normalises to (+1, -1)
    k = _w([[[[2.0, 0.0], [0.0, 5.0]]]])          # (+1, -1) and (-1, +1)
    v = _w([[[[1.0, 0.0], [0.0, 1.0]]]])
    o = oracle.qknorm_attention(q, k, v, ONE2, ZERO2, ONE2, ZERO2, "f32", 0.0)
    p1 = 1.0 / (1.0 + np.exp(-2.0 * np.sqrt(2.0)))
    np.testing.assert_allclose(o, [[[p1, 1.0 - p1]]], rtol=1e-14)
    # the gain of the keys scales the score: gain 3 on both components -> scores +-3 sqrt 2
    o3 = oracle.qknorm_attention(q, k, v, ONE2, ZERO2, 3 * ONE2, ZERO2, "f32", 0.0)
    p3 = 1.0 / (1.0 + np.exp(-6.0 * np.sqrt(2.0)))
    np.testing.assert_allclose(o3, [[[p3, 1.0 / (1.0 + np.exp(6.0 * np.sqrt(2.0)))]]], rtol=1e-13)
    # a bias on the keys adds qn . bk / sqrt(2) to every score alike: nothing changes
    ob = oracle.qknorm_attention(q, k, v, ONE2, ZERO2, ONE2, _w([0.25, -0.5]), "f32", 0.0)
    np.testing.assert_allclose(ob, o, rtol=1e-14)
    # a bias on the query changes qn to (1.5, -1): scores (1.5 + 1) / sqrt 2 and -(2.5) / sqrt 2
    oq = oracle.qknorm_attention(q, k, v, ONE2, _w([0.5, 0.0]), ONE2, ZERO2, "f32", 0.0)
    pq = 1.0 / (1.0 + np.exp(-2.0 * 2.5 / np.sqrt(2.0)))
    np.testing.assert_allclose(oq, [[[pq, 1.0 - pq]]], rtol=1e-14)


def test_hand_case_q1(golden_hand_cases):
    """Golden case Q1 (closed form, 40-digit decimals): a query bias makes qn = (3/2, -1)."""
    q = _w([[[3.0, 1.0]]])
    k = _w([[[[2.0, 0.0], [0.0, 5.0]]]])
    v = _w([[[[1.0, 0.0], [0.0, 1.0]]]])
    for dtype in ("f32", "f16", "bf16"):                 # every value is exact in all three types
        args = [workloads.to_storage(a, dtype) for a in (q, k, v, ONE2, _w([0.5, 0.0]), ONE2, ZERO2)]
        o = oracle.qknorm_attention(*args, dtype, 0.0)
        want = [golden_hand_cases["Q1"][(0, j)] for j in range(2)]
        np.testing.assert_allclose(o[0, 0], want, rtol=1e-14)


def _case(dtype="bf16", B=2, H=3, S=37, D=16, seed=5):
    return workloads.make_attention(B, H, S, D, dtype, seed)


def _run(c, dtype, eps, **over):
    a = dict(c, **over)
    return oracle.qknorm_attention(a["Q"], a["K"], a["V"], a["gq"], a["bq"], a["gk"], a["bk"], dtype, eps)


def test_shift_and_scale_invariance():
    """Layer normalisation removes a vector's offset and (eps = 0) its scale: keys and queries
    moved by a constant along D, or multiplied by a positive power of two, give the same output."""
    c = _case("f32")
    base = _run(c, "f32", 0.0)
    K2 = (c["K"] * np.float32(4.0)).astype(np.float32)
    np.testing.assert_allclose(_run(c, "f32", 0.0, K=K2), base, rtol=1e-9)
    Q2 = (c["Q"] * np.float32(0.5)).astype(np.float32)
    np.testing.assert_allclose(_run(c, "f32", 0.0, Q=Q2), base, rtol=1e-9)
    # offsets are exact in float32 only for small integers: use integer-valued inputs
    rng = np.random.default_rng(3)
    Ki = rng.integers(-8, 9, c["K"].shape).astype(np.float32)
    Qi = rng.integers(-8, 9, c["Q"].shape).astype(np.float32)
    a = _run(c, "f32", 1e-5, K=Ki, Q=Qi)
    b = _run(c, "f32", 1e-5, K=Ki + np.float32(5.0), Q=Qi - np.float32(3.0))
    np.testing.assert_allclose(b, a, rtol=1e-10)


def test_uniform_attention_cases():
    """Equal keys, or a zero key gain, make every score equal: the output is the mean of V."""
    c = _case("f32")
    meanV = c["V"].astype(np.float64).mean(axis=2)
    Ksame = np.broadcast_to(c["K"][:, :, :1, :], c["K"].shape).copy()
    np.testing.assert_allclose(_run(c, "f32", 1e-5, K=Ksame), meanV, rtol=1e-12, atol=1e-15)
    np.testing.assert_allclose(_run(c, "f32", 1e-5, gk=np.zeros_like(c["gk"])), meanV, rtol=1e-12, atol=1e-15)
    # one position: the output is that value row, whatever the rest
    c1 = _case("f32", S=1)
    np.testing.assert_allclose(_run(c1, "f32", 1e-5), c1["V"].astype(np.float64)[:, :, 0, :], rtol=1e-15)


@pytest.mark.parametrize("dtype", ["f32", "f16", "bf16"])
def test_against_library_float64(dtype):
    """torch's layer_norm and scaled_dot_product_attention in float64 on the widened inputs."""
    import torch
    import torch.nn.functional as F
    c = _case(dtype, B=2, H=2, S=50, D=32, seed=9)
    eps = 1e-5
    wide = {k: torch.from_numpy(workloads.to_f32(v, dtype).astype(np.float64)) for k, v in c.items()}
    D = wide["Q"].shape[-1]
    qn = F.layer_norm(wide["Q"], (D,), wide["gq"], wide["bq"], eps)
    kn = F.layer_norm(wide["K"], (D,), wide["gk"], wide["bk"], eps)
    want = F.scaled_dot_product_attention(qn.unsqueeze(2), kn, wide["V"]).squeeze(2).numpy()
    np.testing.assert_allclose(_run(c, dtype, eps), want, rtol=1e-10, atol=1e-13)


MISTAKES = {
    "sample variance": lambda v, g, b, eps: (v - v.mean(-1, keepdims=True)) / np.sqrt(v.var(-1, ddof=1, keepdims=True) + eps) * g + b,
    "eps outside the root": lambda v, g, b, eps: (v - v.mean(-1, keepdims=True)) / (np.sqrt(v.var(-1, keepdims=True)) + eps) * g + b,
    "mean not removed": lambda v, g, b, eps: v / np.sqrt(v.var(-1, keepdims=True) + eps) * g + b,
    "bias dropped": lambda v, g, b, eps: (v - v.mean(-1, keepdims=True)) / np.sqrt(v.var(-1, keepdims=True) + eps) * g,
}


def _numpy_version(c, dtype, eps, norm, scale=None):
    w = {k: workloads.to_f32(v, dtype).astype(np.float64) for k, v in c.items()}
    D = w["Q"].shape[-1]
    qn = norm(w["Q"], w["gq"], w["bq"], eps)
    kn = norm(w["K"], w["gk"], w["bk"], eps)
    s = np.einsum("bhd,bhsd->bhs", qn, kn) * (D ** -0.5 if scale is None else scale)
    p = np.exp(s - s.max(-1, keepdims=True))
    p /= p.sum(-1, keepdims=True)
    return np.einsum("bhs,bhsd->bhd", p, w["V"])


@pytest.mark.parametrize("mistake", list(MISTAKES) + ["scores not scaled"])
def test_pins_catch_planted_mistakes(mistake):
    """Each plausible mistake, planted in a numpy stand-in, moves the result away from the library
    evaluation by far more than the pin's tolerance (so the pin would catch it in the oracle)."""
    import torch
    import torch.nn.functional as F
    c = _case("f32", B=1, H=2, S=40, D=8, seed=21)
    eps = 1e-2
    wide = {k: torch.from_numpy(v.astype(np.float64)) for k, v in c.items()}
    qn = F.layer_norm(wide["Q"], (8,), wide["gq"], wide["bq"], eps)
    kn = F.layer_norm(wide["K"], (8,), wide["gk"], wide["bk"], eps)
    want = F.scaled_dot_product_attention(qn.unsqueeze(2), kn, wide["V"]).squeeze(2).numpy()
    good = lambda v, g, b, e: (v - v.mean(-1, keepdims=True)) / np.sqrt(v.var(-1, keepdims=True) + e) * g + b
    np.testing.assert_allclose(_numpy_version(c, "f32", eps, good), want, rtol=1e-10)
    if mistake == "scores not scaled":
        bad = _numpy_version(c, "f32", eps, good, scale=1.0)
    else:
        bad = _numpy_version(c, "f32", eps, MISTAKES[mistake])
    assert np.abs(bad - want).max() > 1e-4 * np.abs(want).max()
    np.testing.assert_allclose(_run(c, "f32", eps), want, rtol=1e-10)
