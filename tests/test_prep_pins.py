"""Pins of the weight-preparation oracle (oracle/prep_oracle.py) against what the paper's
appendix "GPTAlpha-2 Attention weight preparation" and plain mathematics fix: closed forms,
library routines for the special cases that have one, and invariants of the rotation.  Each
is chosen so that a plausible slip (a sign, a swapped operand, an off-by-one token, the wrong
channel pairing) breaks it."""
import numpy as np
import torch

from oracle import prep_oracle as po

rng = np.random.default_rng(0x9877)


def rand(*shape):
    return rng.standard_normal(shape)


def test_token_shift_closed_forms():
    a = rand(7, 3, 8)
    # alpha = 0: identity; alpha = 1: the previous token's row; first token unshifted
    np.testing.assert_array_equal(po.token_shift(a, np.zeros((3, 8)), None), a)
    s1 = po.token_shift(a, np.ones((3, 8)), None)
    np.testing.assert_allclose(s1[1:], a[:-1], atol=1e-15)
    np.testing.assert_array_equal(s1[0], a[0])
    # per-channel interpolation, written out for one element: a_t + alpha (a_{t-1} - a_t)
    al = rng.uniform(0, 1, (3, 8))
    s = po.token_shift(a, al, None)
    t, h, c = 4, 2, 5
    assert abs(s[t, h, c] - ((1 - al[h, c]) * a[t, h, c] + al[h, c] * a[t - 1, h, c])) < 1e-15
    # a block that continues a sequence equals the tail of the whole sequence
    whole = po.token_shift(a, al, None)
    tail = po.token_shift(a[3:], al, a[2])
    np.testing.assert_allclose(tail, whole[3:], atol=1e-15)


def test_value_residual_closed_forms():
    v, vf = rand(5, 2, 4), rand(5, 2, 4)
    np.testing.assert_array_equal(po.value_residual(v, vf, np.zeros((2, 4))), v)
    np.testing.assert_allclose(po.value_residual(v, vf, np.ones((2, 4))), vf, atol=1e-15)
    lam = rng.uniform(0, 1, (2, 4))
    out = po.value_residual(v, vf, lam)
    assert abs(out[3, 1, 2] - ((1 - lam[1, 2]) * v[3, 1, 2] + lam[1, 2] * vf[3, 1, 2])) < 1e-15
    np.testing.assert_array_equal(po.value_residual(v, None, lam), v)


def test_layer_norm_is_torch_layer_norm_per_head():
    x = rand(6, 3, 16)
    g, b = rng.uniform(0.5, 1.5, (3, 16)), 0.1 * rand(3, 16)
    y = po.layer_norm_heads(x, g, b, 1e-5)
    for h in range(3):
        ref = torch.nn.functional.layer_norm(torch.from_numpy(x[:, h]), (16,), torch.from_numpy(g[h]),
                                             torch.from_numpy(b[h]), 1e-5).numpy()
        np.testing.assert_allclose(y[:, h], ref, rtol=1e-12, atol=1e-12)
    # without parameters: zero mean, unit (biased) variance
    y0 = po.layer_norm_heads(x, None, None, 0.0)
    np.testing.assert_allclose(y0.mean(-1), 0, atol=1e-14)
    np.testing.assert_allclose((y0 ** 2).mean(-1), 1, atol=1e-12)


def test_rope_invariants():
    T, H, d, r = 9, 2, 16, 8
    x = rand(T, H, d)
    pos = np.arange(100, 100 + T)
    y = po.rope_r(x, pos, r)
    # channels >= r untouched; position 0 is the identity; norms of rotated pairs kept
    np.testing.assert_array_equal(y[..., r:], x[..., r:])
    np.testing.assert_allclose(po.rope_r(x, np.zeros(T, dtype=np.int64), r), x, atol=1e-15)
    half = r // 2
    np.testing.assert_allclose(y[..., :half] ** 2 + y[..., half:r] ** 2,
                               x[..., :half] ** 2 + x[..., half:r] ** 2, rtol=1e-12)
    # relative-position property: <R(p1) q, R(p2) k> depends on p1 - p2 only
    q, k = rand(1, 1, d), rand(1, 1, d)
    def dot(p1, p2):
        return float((po.rope_r(q, np.array([p1]), r) * po.rope_r(k, np.array([p2]), r)).sum())
    assert abs(dot(17, 5) - dot(1012, 1000)) < 1e-9
    assert abs(dot(17, 5) - dot(18, 5)) > 1e-6
    # the first pair rotates by exactly `pos` radians (base^0 = 1), counter-clockwise
    e = np.zeros((1, 1, d)); e[0, 0, 0] = 1.0
    out = po.rope_r(e, np.array([1]), r)
    np.testing.assert_allclose([out[0, 0, 0], out[0, 0, half]], [np.cos(1.0), np.sin(1.0)], atol=1e-15)
    # the last pair rotates by pos * base^(-(r-2)/r)
    e = np.zeros((1, 1, d)); e[0, 0, half - 1] = 1.0
    out = po.rope_r(e, np.array([3]), r, base=10000.0)
    ang = 3.0 * 10000.0 ** (-(r - 2) / r)
    np.testing.assert_allclose([out[0, 0, half - 1], out[0, 0, r - 1]], [np.cos(ang), np.sin(ang)], atol=1e-15)
    # composition: rotating by p1 then by p2 (on the already rotated vector) = rotating by p1 + p2
    np.testing.assert_allclose(po.rope_r(po.rope_r(x, pos, r), pos * 2, r), po.rope_r(x, pos * 3, r), atol=1e-12)


def test_merge_gate_closed_forms():
    x = rand(5, 12)
    w = rand(12, 3)
    g = po.merge_gate(x, w)
    z = x @ w
    assert np.all(g > 0)
    np.testing.assert_allclose(g[z > 0], 1 + z[z > 0], rtol=1e-14)
    np.testing.assert_allclose(g[z <= 0], np.exp(z[z <= 0]), rtol=1e-14)
    np.testing.assert_allclose(po.merge_gate(x, np.zeros((12, 3))), 1.0)
    ref = 1 + torch.nn.functional.elu(torch.from_numpy(z)).numpy()
    np.testing.assert_allclose(g, ref, rtol=1e-12)


def test_prepare_order_and_rounding():
    T, Hq, Hk, d, r = 6, 4, 2, 16, 8
    q, k, v, vf = rand(T, Hq, d), rand(T, Hk, d), rand(T, Hk, d), rand(T, Hk, d)
    pos = np.arange(T)
    al = rng.uniform(0, 1, (Hk, d))
    lam = rng.uniform(0, 1, (Hk, d))
    qo, ko_, vo, g = po.prepare(q, k, v, pos, r, "f32", v_first=vf, lam=lam, alpha_v=al)
    # v: residual first, then shift (the shift sees the residual-mixed previous token)
    mixed = (1 - lam) * v + lam * vf
    want = mixed.copy()
    want[1:] = mixed[1:] + al * (mixed[:-1] - mixed[1:])
    np.testing.assert_allclose(vo, want.astype(np.float32), rtol=1e-7)
    # q, k without shift: rotation of the normalised rows; outputs carry the I/O dtype's values
    np.testing.assert_allclose(qo, po.rope_r(po.layer_norm_heads(q, None, None, 1e-5), pos, r).astype(np.float32),
                               rtol=1e-7)
    assert g is None
    qb = po.prepare(q, k, v, pos, r, "bf16")[0]
    as_f32 = qb.astype(np.float32).view(np.uint32)
    assert np.all(as_f32 & 0xFFFF == 0)       # bf16 values: low 16 bits of the fp32 pattern are zero
    # a continued block equals the tail of the whole run
    full = po.prepare(q, k, v, pos, r, "f32", v_first=vf, lam=lam, alpha_q=rng.uniform(0, 1, (Hq, d)) * 0 + 0.3,
                      alpha_k=al, alpha_v=al)
    mixed_prev = mixed[2]
    part = po.prepare(q[3:], k[3:], v[3:], pos[3:], r, "f32", v_first=vf[3:], lam=lam,
                      alpha_q=np.full((Hq, d), 0.3), alpha_k=al, alpha_v=al, prev_q=q[2], prev_k=k[2],
                      prev_v=mixed_prev)
    for a, b in zip(full[:3], part[:3]):
        np.testing.assert_array_equal(a[3:], b)
