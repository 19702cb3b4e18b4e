"""Pins for the fp64 oracle: brute force, library special cases, closed forms and invariants.

Every test here checks oracle/gta_oracle.py against something other than itself, chosen so that
a dropped term, a wrong sign or index, or a transposed operand fails at least one of them.
"""
import numpy as np
import pytest
import torch

from oracle import gta_oracle as orc
from oracle.gta_loops import brute_force_sequence


def _weights(rng, cfg, with_wo=False, std=0.3):
    H, dh, dl = cfg.d_model, cfg.head_dim, cfg.latent_dim
    w = orc.OracleWeights(
        wq=rng.standard_normal((H, cfg.n_qgroups * dh)) * std,
        wk=rng.standard_normal((H, cfg.n_kgroups * dh)) * std,
        wc=rng.standard_normal((H, cfg.n_cgroups * dl)) * std,
        wg=rng.standard_normal((H, cfg.n_heads * dh)) * std,
        wp=rng.standard_normal((cfg.n_heads, dl, dh)) * std,
        wo=rng.standard_normal((cfg.n_heads * dh, H)) * std if with_wo else None)
    return w


# ------------------------------------------------------------------ brute force on tiny inputs
@pytest.mark.parametrize("n_h,n_q,n_k,n_c,dh,dl,rope,wo", [
    (4, 2, 2, 1, 4, 6, False, False),
    (4, 2, 1, 2, 4, 6, True, False),
    (6, 3, 1, 1, 2, 5, True, True),
    (4, 4, 2, 4, 4, 4, False, True),
    (2, 1, 1, 1, 6, 8, True, False),
])
def test_oracle_equals_unreformulated_per_head_loops(n_h, n_q, n_k, n_c, dh, dl, rope, wo):
    rng = np.random.default_rng(n_h * 100 + dl)
    cfg = orc.OracleConfig(d_model=5, n_heads=n_h, n_qgroups=n_q, n_kgroups=n_k, n_cgroups=n_c,
                           head_dim=dh, latent_dim=dl, rope=rope, rope_base=50.0)
    w = _weights(rng, cfg, with_wo=wo)
    T = 7
    x = rng.standard_normal((T, cfg.d_model))
    got, _, _ = orc.prefill_sequence(cfg, w, x)
    ref = brute_force_sequence(
        x.tolist(), w.wq.tolist(), w.wk.tolist(), w.wc.tolist(), w.wg.tolist(), w.wp.tolist(),
        n_heads=n_h, n_qgroups=n_q, n_kgroups=n_k, n_cgroups=n_c, head_dim=dh, latent_dim=dl,
        rope=rope, rope_base=50.0, wo=None if w.wo is None else w.wo.tolist())
    np.testing.assert_allclose(got, np.array(ref), rtol=0, atol=1e-12)


# ------------------------------------------------------------------ library special cases
def _sdpa(q, k, v):
    """torch CPU fp64 causal attention; q,k,v: [heads, T, d]."""
    out = torch.nn.functional.scaled_dot_product_attention(
        torch.from_numpy(q)[None], torch.from_numpy(k)[None], torch.from_numpy(v)[None], is_causal=True)
    return out[0].numpy()


def test_degenerate_setting_is_multi_head_attention():
    """One head per group, d_l = d_h, identity decoder, gate off => plain causal MHA (Sec. 3.1)."""
    rng = np.random.default_rng(1)
    n_h, dh, H, T = 3, 8, 16, 33
    cfg = orc.OracleConfig(H, n_h, n_h, n_h, n_h, dh, dh, gate=False)
    w = _weights(rng, cfg)
    w.wp = np.stack([np.eye(dh)] * n_h)
    x = rng.standard_normal((T, H))
    got, K, C = orc.prefill_sequence(cfg, w, x)
    q = (x @ w.wq).reshape(T, n_h, dh).transpose(1, 0, 2).copy()
    k = (x @ w.wk).reshape(T, n_h, dh).transpose(1, 0, 2).copy()
    v = (x @ w.wc).reshape(T, n_h, dh).transpose(1, 0, 2).copy()
    ref = _sdpa(q, k, v).transpose(1, 0, 2).reshape(T, n_h * dh)
    np.testing.assert_allclose(got, ref, rtol=0, atol=1e-12)
    np.testing.assert_allclose(K, x @ w.wk, atol=1e-13)
    np.testing.assert_allclose(C, x @ w.wc, atol=1e-13)


def test_degenerate_setting_is_grouped_query_attention():
    """n_q = n_h maps, n_k = n_c = n_kv < n_h, identity decoder, gate off => GQA (App. B.3), with
    contiguous blocks of heads sharing a KV head (a relabelling of the appendix's i mod n_k)."""
    rng = np.random.default_rng(2)
    n_h, n_kv, dh, H, T = 6, 2, 4, 12, 21
    cfg = orc.OracleConfig(H, n_h, n_h, n_kv, n_kv, dh, dh, gate=False)
    w = _weights(rng, cfg)
    w.wp = np.stack([np.eye(dh)] * n_h)
    x = rng.standard_normal((T, H))
    got, _, _ = orc.prefill_sequence(cfg, w, x)
    rep = n_h // n_kv
    q = (x @ w.wq).reshape(T, n_h, dh).transpose(1, 0, 2).copy()
    k = np.repeat((x @ w.wk).reshape(T, n_kv, dh).transpose(1, 0, 2), rep, axis=0).copy()
    v = np.repeat((x @ w.wc).reshape(T, n_kv, dh).transpose(1, 0, 2), rep, axis=0).copy()
    ref = _sdpa(q, k, v).transpose(1, 0, 2).reshape(T, n_h * dh)
    np.testing.assert_allclose(got, ref, rtol=0, atol=1e-12)


def test_gva_setting_shares_one_map_among_heads_with_their_own_values():
    """Sec. 3.1, "Grouping Values to Share Attention Matrix": one attention map per group of heads,
    every head its own value projection.  As a GTA setting: n_q = n_k = n_c = groups, the group's
    latent holds its heads' values side by side (d_l = heads-per-group * d_h), W_{P,i} selects head
    i's slice, gate off.  Checked against torch's attention with the group's q, k repeated per head."""
    rng = np.random.default_rng(3)
    n_h, G, dh, H, T = 6, 2, 4, 10, 19
    hpq = n_h // G
    cfg = orc.OracleConfig(H, n_h, G, G, G, dh, hpq * dh, gate=False)
    w = _weights(rng, cfg)
    w.wp = np.zeros((n_h, hpq * dh, dh))
    for i in range(n_h):
        w.wp[i, (i % hpq) * dh:(i % hpq + 1) * dh, :] = np.eye(dh)
    x = rng.standard_normal((T, H))
    got, _, C = orc.prefill_sequence(cfg, w, x)
    q = np.repeat((x @ w.wq).reshape(T, G, dh).transpose(1, 0, 2), hpq, axis=0).copy()
    k = np.repeat((x @ w.wk).reshape(T, G, dh).transpose(1, 0, 2), hpq, axis=0).copy()
    v = (x @ w.wc).reshape(T, n_h, dh).transpose(1, 0, 2).copy()     # head i's own values: columns i*dh.. of X W_C
    ref = _sdpa(q, k, v).transpose(1, 0, 2).reshape(T, n_h * dh)
    np.testing.assert_allclose(got, ref, rtol=0, atol=1e-12)
    assert C.shape == (T, n_h * dh)      # the cache holds a full set of values: what GVA does not save


def test_gha_setting_shares_query_key_and_a_value_source_within_a_group():
    """Sec. 3.1, "Grouping Heads to Compress Attention": the heads of a group share query and key and
    derive their values from one shared source.  As a GTA setting: n_q = n_k = n_c = groups, the
    latent is the shared source (d_l = d_h here), W_{P,i} a dense per-head map, gate off: GTA without
    its nonlinearity.  Checked against torch's attention on V_i = C_g W_{P,i} built per head."""
    rng = np.random.default_rng(4)
    n_h, G, dh, H, T = 6, 3, 4, 10, 17
    hpq = n_h // G
    cfg = orc.OracleConfig(H, n_h, G, G, G, dh, dh, gate=False)
    w = _weights(rng, cfg)
    x = rng.standard_normal((T, H))
    got, _, C = orc.prefill_sequence(cfg, w, x)
    q = np.repeat((x @ w.wq).reshape(T, G, dh).transpose(1, 0, 2), hpq, axis=0).copy()
    k = np.repeat((x @ w.wk).reshape(T, G, dh).transpose(1, 0, 2), hpq, axis=0).copy()
    src = (x @ w.wc).reshape(T, G, dh)
    v = np.stack([src[:, i // hpq, :] @ w.wp[i] for i in range(n_h)]).copy()
    ref = _sdpa(q, k, v).transpose(1, 0, 2).reshape(T, n_h * dh)
    np.testing.assert_allclose(got, ref, rtol=0, atol=1e-12)
    assert C.shape == (T, G * dh)        # one shared source per group is all that is cached


def test_rope_matches_complex_rotation_and_properties():
    rng = np.random.default_rng(3)
    T, n, d, base = 9, 2, 8, 10000.0
    v = rng.standard_normal((T, n, d))
    pos = np.array([0, 1, 2, 5, 17, 100, 1000, 4095, 32768])
    out = orc.rope_rotate(v, pos, base)
    z = v[..., : d // 2] + 1j * v[..., d // 2:]
    theta = base ** (-2.0 * np.arange(d // 2) / d)
    zr = z * np.exp(1j * pos[:, None, None] * theta[None, None, :])
    np.testing.assert_allclose(out[..., : d // 2], zr.real, atol=1e-11)
    np.testing.assert_allclose(out[..., d // 2:], zr.imag, atol=1e-11)
    np.testing.assert_array_equal(out[0], v[0])                       # position 0 is the identity
    np.testing.assert_allclose(np.linalg.norm(out, axis=-1), np.linalg.norm(v, axis=-1), rtol=1e-13)
    # theta_0 = 1 (pair 0 turns by exactly p radians), theta_{d/2-1} = base^(-(d-2)/d)
    e = np.zeros((1, 1, d)); e[0, 0, 0] = 1.0
    r = orc.rope_rotate(e, np.array([1]), base)[0, 0]
    assert abs(r[0] - np.cos(1.0)) < 1e-15 and abs(r[d // 2] - np.sin(1.0)) < 1e-15


def test_rope_scores_depend_on_relative_position_only():
    rng = np.random.default_rng(4)
    cfg = orc.OracleConfig(6, 4, 2, 1, 1, 4, 6, rope=True, rope_base=100.0)
    w = _weights(rng, cfg)
    x = rng.standard_normal((10, 6))
    out0, _, _ = orc.prefill_sequence(cfg, w, x)
    # shift all positions by 37: emulate by projecting with shifted positions
    Q, K, C, G = orc.project_tokens(cfg, w.f64(), x, np.arange(10) + 37)
    L = np.empty((10, 2, 6))
    for g in range(2):
        A = orc.attention_map_rows(cfg, Q[:, g], np.arange(10), K[:, 0])
        L[:, g] = A @ C[:, 0]
    out1 = orc.decode_heads(cfg, w.f64(), L, G)
    np.testing.assert_allclose(out0, out1, atol=1e-12)


# ------------------------------------------------------------------ closed forms
def _cfg(**kw):
    base = dict(d_model=10, n_heads=4, n_qgroups=2, n_kgroups=2, n_cgroups=1, head_dim=4, latent_dim=6)
    base.update(kw)
    return orc.OracleConfig(**base)


def test_zero_keys_give_running_mean_of_latents():
    rng = np.random.default_rng(5)
    cfg = _cfg()
    w = _weights(rng, cfg)
    w.wk[:] = 0.0
    T = 12
    x = rng.standard_normal((T, cfg.d_model))
    got, _, C = orc.prefill_sequence(cfg, w, x)
    run_mean = np.cumsum(C, axis=0) / np.arange(1, T + 1)[:, None]          # [T, d_l]
    gate = 1.0 / (1.0 + np.exp(-(x @ w.wg)))
    ref = np.concatenate([run_mean @ w.wp[i] for i in range(cfg.n_heads)], axis=1) * gate
    np.testing.assert_allclose(got, ref, atol=1e-13)


def test_zero_gate_weights_give_one_half():
    rng = np.random.default_rng(6)
    cfg = _cfg()
    w = _weights(rng, cfg)
    x = rng.standard_normal((9, cfg.d_model))
    on, _, _ = orc.prefill_sequence(cfg, w, x)
    w0 = orc.OracleWeights(w.wq, w.wk, w.wc, np.zeros_like(w.wg), w.wp)
    half, _, _ = orc.prefill_sequence(cfg, w0, x)
    off, _, _ = orc.prefill_sequence(_cfg(gate=False), w, x)
    np.testing.assert_allclose(half, 0.5 * off, atol=1e-14)
    assert np.abs(on - off).max() > 1e-3                                     # the gate does act


@pytest.mark.parametrize("kind", ["silu", "relu2"])
def test_other_gate_nonlinearities(kind):
    """The ablation's Silu and ReLU^2 gates: against the brute-force per-head loops, against torch's own
    functions on the gate pre-activations (the gated output is the ungated one times the factor, row by
    row), and the closed forms silu(0) = relu(0)^2 = 0 for zero gate weights."""
    rng = np.random.default_rng(16)
    cfg = orc.OracleConfig(d_model=5, n_heads=4, n_qgroups=2, n_kgroups=1, n_cgroups=2, head_dim=4, latent_dim=6,
                           rope=True, rope_base=50.0, gate=kind)
    w = _weights(rng, cfg)
    x = rng.standard_normal((7, cfg.d_model))
    got, _, _ = orc.prefill_sequence(cfg, w, x)
    ref = brute_force_sequence(
        x.tolist(), w.wq.tolist(), w.wk.tolist(), w.wc.tolist(), w.wg.tolist(), w.wp.tolist(),
        n_heads=4, n_qgroups=2, n_kgroups=1, n_cgroups=2, head_dim=4, latent_dim=6, rope=True, rope_base=50.0, gate=kind)
    np.testing.assert_allclose(got, np.array(ref), rtol=0, atol=1e-12)
    off, _, _ = orc.prefill_sequence(orc.OracleConfig(**{**cfg.__dict__, "gate": False}), w, x)
    z = torch.from_numpy(x @ w.wg)
    fac = torch.nn.functional.silu(z) if kind == "silu" else torch.relu(z) ** 2
    np.testing.assert_allclose(got, off * fac.numpy(), rtol=0, atol=1e-13)
    w0 = orc.OracleWeights(w.wq, w.wk, w.wc, np.zeros_like(w.wg), w.wp)
    zero, _, _ = orc.prefill_sequence(cfg, w0, x)
    assert np.all(zero == 0.0)
    dec = orc.OracleConfig(**{**cfg.__dict__, "gate": "sigmoid"})
    sig, _, _ = orc.prefill_sequence(dec, w, x)
    on, _, _ = orc.prefill_sequence(orc.OracleConfig(**{**cfg.__dict__, "gate": True}), w, x)
    assert np.array_equal(sig, on) and np.abs(got - sig).max() > 1e-3


def test_single_token():
    rng = np.random.default_rng(7)
    cfg = _cfg(rope=True)
    w = _weights(rng, cfg, with_wo=True)
    x = rng.standard_normal((1, cfg.d_model))
    got, _, _ = orc.prefill_sequence(cfg, w, x)
    c0 = x @ w.wc
    heads = np.concatenate([c0 @ w.wp[i] for i in range(cfg.n_heads)], axis=1)
    ref = (heads / (1.0 + np.exp(-(x @ w.wg)))) @ w.wo
    np.testing.assert_allclose(got, ref, atol=1e-13)


def test_softmax_shift_invariance_constant_key_offset():
    """Adding one constant vector to every key adds a per-row constant to the scores."""
    rng = np.random.default_rng(8)
    cfg = _cfg()
    w = _weights(rng, cfg).f64()
    x = rng.standard_normal((8, cfg.d_model))
    Q, K, C, G = orc.project_tokens(cfg, w, x, np.arange(8))
    off = rng.standard_normal(cfg.head_dim)
    for g in range(cfg.n_qgroups):
        a0 = orc.attention_map_rows(cfg, Q[:, g], np.arange(8), K[:, g])
        a1 = orc.attention_map_rows(cfg, Q[:, g], np.arange(8), K[:, g] + off)
        np.testing.assert_allclose(a0, a1, atol=1e-13)


# ------------------------------------------------------------------ invariants
def test_map_rows_sum_to_one_are_causal_and_shared_within_group():
    rng = np.random.default_rng(9)
    cfg = _cfg(n_heads=6, n_qgroups=2, n_kgroups=1, rope=True)
    w = _weights(rng, cfg)
    T = 15
    x = rng.standard_normal((T, cfg.d_model))
    out, _, _, maps = orc.prefill_sequence(cfg, w, x, return_maps=True)
    assert len(maps) == cfg.n_qgroups                  # one map per group, not per head
    for A in maps:
        np.testing.assert_allclose(A.sum(axis=1), 1.0, atol=1e-14)
        assert np.all(np.triu(A, 1) == 0.0) and np.all(A[np.tril_indices(T)] > 0.0)
    # heads of one group with equal decoder weights give identical output blocks
    w.wp[1] = w.wp[0]; w.wg[:, 4:8] = w.wg[:, 0:4]
    out, _, _ = orc.prefill_sequence(cfg, w, x)
    np.testing.assert_array_equal(out[:, 0:4], out[:, 4:8])
    # softmax scale is 1/sqrt(d_h)
    Q, K, _, _ = orc.project_tokens(cfg, w.f64(), x, np.arange(T))
    s = Q[5, 1] @ K[:6, 0].T / np.sqrt(cfg.head_dim)
    e = np.exp(s - s.max())
    np.testing.assert_allclose(maps[1][5, :6], e / e.sum(), atol=1e-14)


def test_future_tokens_do_not_change_earlier_rows():
    rng = np.random.default_rng(10)
    cfg = _cfg(rope=True)
    w = _weights(rng, cfg)
    x = rng.standard_normal((14, cfg.d_model))
    a, _, _ = orc.prefill_sequence(cfg, w, x)
    x2 = x.copy(); x2[9:] = rng.standard_normal((5, cfg.d_model))
    b, _, _ = orc.prefill_sequence(cfg, w, x2)
    np.testing.assert_allclose(a[:9], b[:9], rtol=0, atol=1e-14)
    assert np.abs(a[9:] - b[9:]).max() > 1e-3


def test_head_permutation_within_group_permutes_output_blocks():
    rng = np.random.default_rng(11)
    cfg = _cfg()
    w = _weights(rng, cfg)
    x = rng.standard_normal((6, cfg.d_model))
    a, _, _ = orc.prefill_sequence(cfg, w, x)
    dh = cfg.head_dim
    w2 = orc.OracleWeights(w.wq, w.wk, w.wc, w.wg.copy(), w.wp.copy())
    w2.wp[[0, 1]] = w.wp[[1, 0]]
    w2.wg[:, 0:dh], w2.wg[:, dh:2 * dh] = w.wg[:, dh:2 * dh], w.wg[:, 0:dh]
    b, _, _ = orc.prefill_sequence(cfg, w2, x)
    np.testing.assert_allclose(b[:, 0:dh], a[:, dh:2 * dh], atol=1e-14)
    np.testing.assert_allclose(b[:, dh:2 * dh], a[:, 0:dh], atol=1e-14)
    np.testing.assert_allclose(b[:, 2 * dh:], a[:, 2 * dh:], atol=1e-14)


def test_rows_subset_and_packed_batch_equal_separate_sequences():
    rng = np.random.default_rng(12)
    cfg = _cfg(rope=True)
    w = _weights(rng, cfg)
    lens = [5, 1, 9]
    cu = np.concatenate([[0], np.cumsum(lens)])
    x = rng.standard_normal((cu[-1], cfg.d_model))
    out, K, C = orc.prefill(cfg, w, x, cu)
    for b in range(3):
        o, k, c = orc.prefill_sequence(cfg, w, x[cu[b]:cu[b + 1]])
        np.testing.assert_array_equal(out[cu[b]:cu[b + 1]], o)
        np.testing.assert_array_equal(K[cu[b]:cu[b + 1]], k)
    full, _, _ = orc.prefill_sequence(cfg, w, x[cu[2]:cu[3]])
    sub, _, _ = orc.prefill_sequence(cfg, w, x[cu[2]:cu[3]], rows=[0, 4, 8])
    np.testing.assert_allclose(sub, full[[0, 4, 8]], atol=1e-14)


@pytest.mark.parametrize("with_wo", [False, True])
def test_decode_over_cache_equals_last_row_of_prefill(with_wo):
    rng = np.random.default_rng(13)
    cfg = _cfg(n_heads=4, n_qgroups=2, n_kgroups=1, n_cgroups=2, rope=True)
    w = _weights(rng, cfg, with_wo=with_wo)
    T = 11
    x = rng.standard_normal((T, cfg.d_model))
    full, K, C = orc.prefill_sequence(cfg, w, x)
    kw, cw = K.shape[1], C.shape[1]
    kc = rng.standard_normal((3, 16, kw)); cc = rng.standard_normal((3, 16, cw))   # noise beyond valid rows
    kc0, cc0 = kc.copy(), cc.copy()
    seq = np.zeros(3, dtype=np.int32); status = np.zeros(3, dtype=np.int32)
    slot = 2
    orc.cache_append(kc, cc, seq, status, [slot], K[:T - 1], C[:T - 1], [0, T - 1])
    assert seq[slot] == T - 1
    got = orc.decode(cfg, w, x[T - 1:T], kc, cc, seq, status, [slot])
    np.testing.assert_allclose(got[0], full[T - 1], atol=1e-12)
    assert seq.tolist() == [0, 0, T] and status.tolist() == [0, 0, 0]
    np.testing.assert_allclose(kc[slot, :T], K, atol=1e-13)
    np.testing.assert_allclose(cc[slot, :T], C, atol=1e-13)
    # untouched rows and slots stay bit-identical
    np.testing.assert_array_equal(kc[slot, T:], kc0[slot, T:])
    np.testing.assert_array_equal(kc[:2], kc0[:2])
    np.testing.assert_array_equal(cc[:2], cc0[:2])


def test_decode_on_empty_cache_and_on_full_cache():
    rng = np.random.default_rng(14)
    cfg = _cfg(rope=True)
    w = _weights(rng, cfg)
    x = rng.standard_normal((2, cfg.d_model))
    kc = np.zeros((2, 3, 8)); cc = np.zeros((2, 3, 6))
    seq = np.array([0, 3], dtype=np.int32); status = np.zeros(2, dtype=np.int32)
    out = orc.decode(cfg, w, x, kc, cc, seq, status, [0, 1])
    c0 = x[0:1] @ w.wc
    ref = np.concatenate([c0 @ w.wp[i] for i in range(4)], axis=1) / (1.0 + np.exp(-(x[0:1] @ w.wg)))
    np.testing.assert_allclose(out[0], ref[0], atol=1e-13)
    assert status.tolist() == [0, orc.CACHE_FULL] and seq.tolist() == [1, 3]
    assert np.all(out[1] == 0.0) and np.all(kc[1] == 0.0)


def test_cache_append_is_an_integer_indexed_row_copy():
    rng = np.random.default_rng(15)
    kc = rng.standard_normal((4, 8, 6)); cc = rng.standard_normal((4, 8, 10))
    kc0, cc0 = kc.copy(), cc.copy()
    seq = np.array([2, 0, 7, 5], dtype=np.int32); status = np.zeros(4, dtype=np.int32)
    k_new = rng.standard_normal((6, 6)); c_new = rng.standard_normal((6, 10))
    # sequences: slot 3 gets 3 rows, slot 2 gets 2 rows (overflow: 7+2 > 8), slot 1 gets 1 row
    orc.cache_append(kc, cc, seq, status, [3, 2, 1], k_new, c_new, [0, 3, 5, 6])
    assert seq.tolist() == [2, 1, 7, 8]
    assert status.tolist() == [0, 0, orc.CACHE_FULL, 0]
    np.testing.assert_array_equal(kc[3, 5:8], k_new[0:3])
    np.testing.assert_array_equal(cc[3, 5:8], c_new[0:3])
    np.testing.assert_array_equal(kc[1, 0], k_new[5])
    np.testing.assert_array_equal(kc[2], kc0[2])
    np.testing.assert_array_equal(kc[0], kc0[0])
    np.testing.assert_array_equal(kc[3, :5], kc0[3, :5])
    np.testing.assert_array_equal(cc[1, 1:], cc0[1, 1:])
