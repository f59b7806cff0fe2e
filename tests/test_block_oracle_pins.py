"""Pins of the mini-Transformer block oracle (oracle/block.py) against textbook forms and
library routines; CPU only."""
import numpy as np
import pytest
import torch

from oracle import block as ob

RNG = np.random.default_rng(20251102)


def test_rmsnorm_matches_library_and_definition():
    x = RNG.standard_normal((7, 96)) * 3.0
    ref = torch.nn.functional.rms_norm(torch.from_numpy(x), (96,), eps=1e-6).numpy()
    assert np.allclose(ob.rmsnorm(x), ref, rtol=1e-13, atol=1e-13)
    # unit gain: the mean square of a normalised row is 1 (up to eps)
    assert np.allclose(np.mean(ob.rmsnorm(x) ** 2, axis=-1), 1.0, atol=1e-6)
    # a constant row c maps to sign(c) (eps negligible)
    assert np.allclose(ob.rmsnorm(np.full((1, 8), -5.0)), -1.0, atol=1e-7)


def test_rope_is_a_rotation_by_position_times_frequency():
    T, H, D = 9, 3, 16
    x = RNG.standard_normal((T, H, D))
    pos = np.array([0, 1, 2, 5, 17, 100, 1000, 40000, 65535])
    y = ob.rope(x, pos)
    # complex form: (x_i + j x_{i+D/2}) * exp(j pos theta^(-2i/D))
    z = x[..., :D // 2] + 1j * x[..., D // 2:]
    w = np.exp(1j * pos[:, None, None] * 10000.0 ** (-2.0 * np.arange(D // 2) / D)[None, None, :])
    zr = z * w
    assert np.allclose(y[..., :D // 2], zr.real, atol=1e-9) and np.allclose(y[..., D // 2:], zr.imag, atol=1e-9)
    assert np.allclose(y[0], x[0])                                        # position 0: identity
    assert np.allclose(np.linalg.norm(y, axis=-1), np.linalg.norm(x, axis=-1))   # norms preserved
    # the first pair turns by exactly pos radians (frequency 1)
    assert np.allclose(ob.rope(np.eye(1, D)[None], [np.pi / 2])[0, 0, D // 2], 1.0)


def test_rope_scores_depend_on_relative_position_only():
    D = 32
    q, k = RNG.standard_normal((1, 1, D)), RNG.standard_normal((1, 1, D))
    s0 = float(np.sum(ob.rope(q, [7]) * ob.rope(k, [3])))
    for shift in (1, 100, 4096, 60000):
        s = float(np.sum(ob.rope(q, [7 + shift]) * ob.rope(k, [3 + shift])))
        assert abs(s - s0) < 1e-8
    assert abs(float(np.sum(ob.rope(q, [8]) * ob.rope(k, [3]))) - s0) > 1e-3   # and do depend on it


def test_swiglu_matches_library():
    g, u = RNG.standard_normal((5, 11)) * 4, RNG.standard_normal((5, 11))
    ref = (torch.nn.functional.silu(torch.from_numpy(g)) * torch.from_numpy(u)).numpy()
    assert np.allclose(ob.swiglu(g, u), ref, rtol=1e-13, atol=1e-13)
    assert np.allclose(ob.swiglu(np.zeros(3), np.ones(3)), 0.0)
    assert np.allclose(ob.swiglu(np.full(3, 50.0), np.full(3, 2.0)), 100.0)    # silu(z) -> z for large z


def _weights(d_model, Hq, Hkv, D, F, scale=0.2):
    mk = lambda *s: RNG.standard_normal(s) * scale
    return {"qkv": mk(d_model, (Hq + 2 * Hkv) * D), "o": mk(Hq * D, d_model), "gate_up": mk(d_model, 2 * F), "down": mk(F, d_model)}


def _torch_block(x, w, Hq, Hkv, D, mask):
    """The same block assembled from library routines (fp64), attention with an explicit mask."""
    t = lambda a: torch.from_numpy(np.asarray(a, dtype=np.float64))
    x = t(x)
    T, d_model = x.shape
    h = torch.nn.functional.rms_norm(x, (d_model,), eps=1e-6)
    qkv = h @ t(w["qkv"])
    q, k, v = qkv[:, :Hq * D].view(T, Hq, D), qkv[:, Hq * D:(Hq + Hkv) * D].view(T, Hkv, D), qkv[:, (Hq + Hkv) * D:].view(T, Hkv, D)
    pos = torch.arange(T, dtype=torch.float64)
    inv = 10000.0 ** (-2.0 * torch.arange(D // 2, dtype=torch.float64) / D)
    ang = pos[:, None] * inv[None, :]
    cos, sin = torch.cos(ang)[:, None, :], torch.sin(ang)[:, None, :]
    rot = lambda a: torch.cat([a[..., :D // 2] * cos - a[..., D // 2:] * sin, a[..., D // 2:] * cos + a[..., :D // 2] * sin], dim=-1)
    q, k = rot(q), rot(k)
    q, k, v = q.float().double(), k.float().double(), v.float().double()   # stored at float32 at most
    G = Hq // Hkv
    kk, vv = k.repeat_interleave(G, dim=1), v.repeat_interleave(G, dim=1)
    o = torch.nn.functional.scaled_dot_product_attention(q.transpose(0, 1), kk.transpose(0, 1), vv.transpose(0, 1),
                                                         attn_mask=torch.from_numpy(mask))
    x1 = x + o.transpose(0, 1).reshape(T, Hq * D) @ t(w["o"])
    h2 = torch.nn.functional.rms_norm(x1, (d_model,), eps=1e-6)
    gu = h2 @ t(w["gate_up"])
    F = w["down"].shape[0]
    return (x1 + (torch.nn.functional.silu(gu[:, :F]) * gu[:, F:]) @ t(w["down"])).numpy()


@pytest.mark.parametrize("is_sync", [False, True])
def test_block_matches_the_same_block_built_from_library_routines(is_sync):
    d_model, Hq, Hkv, D, F = 48, 4, 2, 16, 40
    seg = np.array([0, 9, 9, 20, 31])
    T = 31
    x = RNG.standard_normal((T, d_model))
    w = _weights(d_model, Hq, Hkv, D, F)
    got = ob.block_forward(x, w, seg, n_q_heads=Hq, n_kv_heads=Hkv, head_dim=D, is_sync=is_sync)["out"]
    i, j = np.arange(T)[:, None], np.arange(T)[None, :]
    mask = j <= i
    if not is_sync:
        owner = np.searchsorted(seg, np.arange(T), side="right")
        mask = mask & (owner[:, None] == owner[None, :])
    assert np.allclose(got, _torch_block(x, w, Hq, Hkv, D, mask), rtol=1e-10, atol=1e-10)


def test_sync_block_does_not_depend_on_the_segmentation():
    # H = 1 is centralized inference (Remark after Corollary 1): a sync block over N participants
    # equals the block on the undivided sequence
    d_model, Hq, Hkv, D, F = 32, 2, 1, 16, 24
    x = RNG.standard_normal((26, d_model))
    w = _weights(d_model, Hq, Hkv, D, F)
    kw = dict(n_q_heads=Hq, n_kv_heads=Hkv, head_dim=D, is_sync=True)
    a = ob.block_forward(x, w, [0, 5, 13, 26], **kw)["out"]
    b = ob.block_forward(x, w, [0, 26], **kw)["out"]
    assert np.allclose(a, b, rtol=1e-12, atol=1e-12)


def test_local_block_equals_each_participant_alone_with_local_positions():
    # Phase I: a participant needs nothing from the others; and because rotary scores depend on
    # relative positions only, its own position count gives the same result as the global index
    d_model, Hq, Hkv, D, F = 32, 2, 2, 16, 24
    seg = [0, 7, 19, 30]
    x = RNG.standard_normal((30, d_model))
    w = _weights(d_model, Hq, Hkv, D, F)
    kw = dict(n_q_heads=Hq, n_kv_heads=Hkv, head_dim=D, is_sync=False)
    joint = ob.block_forward(x, w, seg, **kw)["out"]
    for n in range(3):
        s, e = seg[n], seg[n + 1]
        alone = ob.block_forward(x[s:e], w, [0, e - s], pos=np.arange(e - s), **kw)["out"]
        assert np.allclose(joint[s:e], alone, rtol=1e-5, atol=1e-5)   # q, k are stored as float32 after the rotation


def test_rounding_hook_touches_interfaces_only():
    d_model, Hq, Hkv, D, F = 32, 2, 1, 16, 24
    x = RNG.standard_normal((12, d_model))
    w = _weights(d_model, Hq, Hkv, D, F)
    kw = dict(n_q_heads=Hq, n_kv_heads=Hkv, head_dim=D, is_sync=True)
    exact = ob.block_forward(x, w, [0, 12], **kw)
    calls = []
    ident = ob.block_forward(x, w, [0, 12], round_fn=lambda a: (calls.append(a.shape), a)[1], **kw)
    assert len(calls) == 10         # h, qkv, q, k, attn, o-proj, h2, gate_up, act, down
    assert np.allclose(ident["out"], exact["out"], atol=1e-5)      # float32 pass-through of the hook only


@pytest.mark.parametrize("is_sync", [False, True])
def test_row_sampled_block_matches_the_library_block_on_those_rows(is_sync):
    """block_forward_rows (keys and values for every token, everything else for the requested rows
    only) against the block assembled from library routines, and against block_forward, with a
    keep-list and with the rounding hook."""
    d_model, Hq, Hkv, D, F = 48, 4, 2, 16, 40
    seg = np.array([0, 9, 9, 20, 31])
    T = 31
    x = RNG.standard_normal((T, d_model))
    w = _weights(d_model, Hq, Hkv, D, F)
    rows = np.array([0, 8, 9, 19, 20, 30, 14])
    kw = dict(n_q_heads=Hq, n_kv_heads=Hkv, head_dim=D, is_sync=is_sync)
    got = ob.block_forward_rows(x, w, seg, rows, **kw)
    i, j = np.arange(T)[:, None], np.arange(T)[None, :]
    mask = j <= i
    owner = np.searchsorted(seg, np.arange(T), side="right")
    if not is_sync:
        mask = mask & (owner[:, None] == owner[None, :])
    assert np.allclose(got["out"], _torch_block(x, w, Hq, Hkv, D, mask)[rows], rtol=1e-10, atol=1e-10)
    # sparse exchange and the rounding hook: the same numbers as the full block on those rows
    keep = (RNG.random(T) < 0.5).astype(np.uint8)
    rnd = lambda a: np.round(a * 64.0) / 64.0
    full = ob.block_forward(x, w, seg, keep_tok=keep, round_fn=rnd, **kw)
    part = ob.block_forward_rows(x, w, seg, rows, keep_tok=keep, round_fn=rnd, **kw)
    assert np.allclose(part["out"], full["out"][rows], rtol=1e-12, atol=1e-12)
    assert np.allclose(part["attn"], full["attn"][rows], rtol=1e-12, atol=1e-12)
