"""Pins for the oracle's forward with out-of-span caching (Section 3.3): the
special cases that must reduce to the full forward, and the stale-feature
semantics written out independently from the oracle's separately pinned ops."""
import numpy as np
import pytest

import oracle
from paper_2506_10848_amd import synth
from util import weights_bits


def small_model(n_layers=2):
    cfg = dict(synth.CONFIGS["tiny"], vocab=96, mask_id=95, prompt=5, gen=11, d_model=64, n_heads=2, head_dim=32,
               d_ffn=80, n_layers=n_layers)
    w = synth.make_weights(cfg, std=0.3)
    return cfg, synth.model_config(cfg), weights_bits(w)


def state(cfg, B, seed=0):
    rng = np.random.default_rng(seed)
    L = cfg["prompt"] + cfg["gen"]
    tok = rng.integers(0, cfg["mask_id"], (B, L)).astype(np.int32)
    tok[:, cfg["prompt"]:] = cfg["mask_id"]
    return tok


def test_refresh_equals_the_full_forward():
    cfg, mc, wb = small_model()
    tok = state(cfg, 2)
    B, L = tok.shape
    cache = oracle.KVCache(mc, B, L)
    got = oracle.forward_cached(mc, wb, tok, cache, np.arange(B * L))
    assert np.array_equal(got, oracle.forward(mc, wb, tok))
    assert np.abs(cache.k).max() > 0 and np.abs(cache.v).max() > 0


def test_fresh_cache_changes_nothing():
    # features cached from the same tokens are what a recomputation would give
    cfg, mc, wb = small_model()
    tok = state(cfg, 2)
    B, L = tok.shape
    full = oracle.forward(mc, wb, tok)
    cache = oracle.KVCache(mc, B, L)
    oracle.forward_cached(mc, wb, tok, cache, np.arange(B * L))
    skip = np.zeros((B, L), np.uint8); skip[0, 9:] = 1; skip[1, 12:15] = 1
    rows = np.flatnonzero(skip.reshape(-1) == 0)
    k0 = cache.k.copy()
    got = oracle.forward_cached(mc, wb, tok, cache, rows, skip)
    np.testing.assert_allclose(got, full[rows], rtol=0, atol=1e-11 * np.abs(full).max())
    np.testing.assert_allclose(cache.k, k0, rtol=0, atol=1e-11 * np.abs(k0).max())
    with pytest.raises(ValueError):                      # a skipped row has no logits
        oracle.forward_cached(mc, wb, tok, cache, np.array([9]), skip)


def test_one_layer_features_never_go_stale():
    # first-layer keys/values depend on a position's own token only, and skipped
    # positions are still [MASK]: with one layer the cached forward is exact
    cfg, mc, wb = small_model(n_layers=1)
    tok = state(cfg, 1)
    B, L = tok.shape
    cache = oracle.KVCache(mc, B, L)
    oracle.forward_cached(mc, wb, tok, cache, np.arange(L))
    tok2 = tok.copy(); tok2[0, 5:8] = [3, 17, 40]        # committed since
    skip = np.zeros((1, L), np.uint8); skip[0, 10:] = 1
    rows = np.arange(10)
    got = oracle.forward_cached(mc, wb, tok2, cache, rows, skip)
    full = oracle.forward(mc, wb, tok2)
    np.testing.assert_allclose(got, full[rows], rtol=0, atol=1e-11 * np.abs(full).max())


def layer_by_layer(mc, wb, tok, stale=None, skip=None):
    """The transformer written out with the oracle's ops for one sequence; if `stale`
    (per-layer (K, V) of an earlier pass) is given, the rows in `skip` present those
    keys/values to everyone instead of their own.  Returns final hidden states and the
    per-layer (K, V) actually used."""
    L = tok.shape[0]
    d, H, dh, f = mc["d_model"], mc["n_heads"], mc["head_dim"], mc["d_ffn"]
    x = oracle.bf16_to_f64(wb["embed"])[tok]
    pos = np.arange(L)
    used = []
    for l in range(mc["n_layers"]):
        h = oracle.rmsnorm(x, wb["attn_norm"][l], mc["rms_eps"])
        qkv = oracle.linear(h, wb["wqkv"][l])
        q = oracle.rope(qkv[:, :d].reshape(L, H, dh), pos, mc["rope_theta"])
        k = oracle.rope(qkv[:, d:2 * d].reshape(L, H, dh), pos, mc["rope_theta"])
        v = qkv[:, 2 * d:].reshape(L, H, dh).copy()
        if stale is not None:
            k[skip], v[skip] = stale[l][0][skip], stale[l][1][skip]
        used.append((k.copy(), v.copy()))
        x = x + oracle.linear(oracle.attention(q, k, v).reshape(L, d), wb["wo"][l])
        h = oracle.rmsnorm(x, wb["ffn_norm"][l], mc["rms_eps"])
        gu = oracle.linear(h, wb["w_gate_up"][l])
        x = x + oracle.linear(oracle.swiglu(gu[:, :f], gu[:, f:]), wb["w_down"][l])
    return oracle.rmsnorm(x, wb["final_norm"], mc["rms_eps"]), used


def test_stale_features_semantics():
    cfg, mc, wb = small_model(n_layers=3)
    tok = state(cfg, 1, seed=4)
    L = tok.shape[1]
    cache = oracle.KVCache(mc, 1, L)
    oracle.forward_cached(mc, wb, tok, cache, np.arange(L))
    _, kv0 = layer_by_layer(mc, wb, tok[0])
    for l in range(3):                                   # the cache holds K after RoPE and V
        np.testing.assert_allclose(cache.k[l].reshape(L, 2, 32), kv0[l][0], atol=1e-10)
        np.testing.assert_allclose(cache.v[l].reshape(L, 2, 32), kv0[l][1], atol=1e-10)
    tok2 = tok.copy(); tok2[0, 5:9] = [3, 17, 40, 7]
    skip = np.zeros(L, bool); skip[11:] = True; skip[9] = True
    rows = np.flatnonzero(~skip)
    got = oracle.forward_cached(mc, wb, tok2, cache, rows, skip.astype(np.uint8)[None])
    hid, kv1 = layer_by_layer(mc, wb, tok2[0], stale=kv0, skip=skip)
    want = oracle.linear(hid[rows], wb["lm_head"])
    np.testing.assert_allclose(got, want, rtol=0, atol=1e-10 * np.abs(want).max())
    fresh = oracle.forward(mc, wb, tok2)[rows]
    assert np.abs(got - fresh).max() > 1e-6 * np.abs(fresh).max()      # and it is an approximation
    # recomputed rows refreshed their cache rows, skipped rows kept theirs
    for l in range(3):
        np.testing.assert_allclose(cache.k[l].reshape(L, 2, 32), kv1[l][0], atol=1e-10)
