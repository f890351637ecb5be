"""Pins for the oracle's forward-pass operators and row phase.

Each check ties the oracle to something other than itself: a closed form, a
hand-computed value, an invariant of the mathematics, or an independent
library routine (numpy / scipy / torch in fp64)."""
import math
import os

import numpy as np
import pytest
import scipy.special
import torch

import oracle
from paper_2506_10848_amd import synth
from util import bits, weights_bits

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")
rng = np.random.default_rng(7)


def bf(x):
    """float array -> bf16 bit patterns through torch (library rounding)."""
    return bits(torch.as_tensor(np.asarray(x), dtype=torch.float32).to(torch.bfloat16))


# ---- bf16 ---------------------------------------------------------------------

def test_bf16_roundtrip_all_patterns():
    allb = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    vals = oracle.bf16_to_f64(allb)
    finite = np.isfinite(vals)
    back = oracle.round_to_bf16(vals[finite])
    assert np.array_equal(back, allb[finite])


def test_bf16_rounding_matches_torch_on_float32_inputs():
    x = np.concatenate([rng.standard_normal(20000) * 10.0 ** rng.integers(-30, 30, 20000),
                        [0.0, -0.0, 1.0, 1.00390625, 1.01171875, 3.3895e38, 1e-40, -1e-45]]).astype(np.float32)
    ours = oracle.round_to_bf16(x.astype(np.float64))
    ref = bf(x)
    assert np.array_equal(ours, ref)


def test_bf16_ties_to_even_and_single_rounding():
    # 1 + 2^-8 is halfway between 1 and 1 + 2^-7: goes to the even one (1.0)
    assert oracle.lib().orc_f64_to_bf16(1.0 + 2.0 ** -8) == 0x3F80
    # 1 + 3*2^-8 is halfway between 1+2^-7 and 1+2^-6: even is 1+2^-6
    assert oracle.lib().orc_f64_to_bf16(1.0 + 3 * 2.0 ** -8) == 0x3F82
    # just above the tie, by less than float32 can see: must round up (a
    # double -> float -> bf16 chain would land on the tie and round down)
    assert oracle.lib().orc_f64_to_bf16(1.0 + 2.0 ** -8 + 2.0 ** -40) == 0x3F81


# ---- RMSNorm ------------------------------------------------------------------

def test_rmsnorm_hand_values_and_invariants():
    g = bf(np.ones(2))
    out = oracle.rmsnorm(np.array([[3.0, 4.0]]), g, 0.0)
    # mean square = 12.5
    assert np.allclose(out, [[3 / math.sqrt(12.5), 4 / math.sqrt(12.5)]], rtol=1e-14)
    # eps enters under the root, added to the mean square
    out = oracle.rmsnorm(np.array([[3.0, 4.0]]), g, 3.5)
    assert np.allclose(out, [[0.75, 1.0]], rtol=1e-14)
    # constant row -> sign * gain
    gg = np.array([0.5, -2.0, 1.0, 4.0])
    out = oracle.rmsnorm(np.full((1, 4), -7.0), bf(gg), 0.0)
    assert np.allclose(out, [-gg], rtol=1e-14)
    # scale invariance and unit mean square
    x = rng.standard_normal((5, 64))
    a = oracle.rmsnorm(x, bf(np.ones(64)), 0.0)
    b = oracle.rmsnorm(x * 37.0, bf(np.ones(64)), 0.0)
    assert np.allclose(a, b, rtol=1e-12)
    assert np.allclose((a * a).mean(axis=1), 1.0, rtol=1e-12)
    # library cross-check
    ref = torch.nn.functional.rms_norm(torch.from_numpy(x), (64,), eps=1e-5).numpy()
    assert np.allclose(oracle.rmsnorm(x, bf(np.ones(64)), 1e-5), ref, rtol=1e-12)


# ---- linear -------------------------------------------------------------------

def test_linear_orientation_and_library():
    # W[n][k]: one-hot rows pick input coordinates -> catches a transposed operand
    W = np.zeros((3, 5)); W[0, 4] = 1; W[1, 0] = 2; W[2, 2] = -1
    x = np.arange(10.0).reshape(2, 5)
    y = oracle.linear(x, bf(W))
    assert np.array_equal(y, [[4, 0, -2], [9, 10, -7]])
    x = rng.standard_normal((7, 33))
    Wb = bf(rng.standard_normal((19, 33)))
    ref = x @ oracle.bf16_to_f64(Wb).T
    assert np.allclose(oracle.linear(x, Wb), ref, rtol=1e-12, atol=1e-12)


# ---- RoPE ---------------------------------------------------------------------

def test_rope_hand_values():
    # dh = 4: pairs (0,2) with frequency 1 and (1,3) with frequency theta^-1/2
    theta = 100.0
    x = np.array([[[1.0, 2.0, 3.0, 4.0]]])
    out = oracle.rope(x, [0], theta)
    assert np.array_equal(out, x)                       # position 0 is the identity
    p = 3
    out = oracle.rope(x, [p], theta)[0, 0]
    a0, a1 = p * 1.0, p * theta ** -0.5
    exp = [1 * math.cos(a0) - 3 * math.sin(a0), 2 * math.cos(a1) - 4 * math.sin(a1),
           1 * math.sin(a0) + 3 * math.cos(a0), 2 * math.sin(a1) + 4 * math.cos(a1)]
    assert np.allclose(out, exp, rtol=1e-13)


def test_rope_is_a_rotation_and_relative():
    H, dh, theta = 2, 16, 10000.0
    q = rng.standard_normal((1, H, dh)); k = rng.standard_normal((1, H, dh))
    def dot(m, n):
        return (oracle.rope(q, [m], theta) * oracle.rope(k, [n], theta)).sum(axis=2)
    assert np.allclose(dot(9, 4), dot(14, 9), rtol=1e-10)       # depends on m - n only
    assert not np.allclose(dot(9, 4), dot(9, 5), rtol=1e-3)
    x = rng.standard_normal((6, H, dh))
    r = oracle.rope(x, np.arange(6), theta)
    assert np.allclose((r ** 2).sum(axis=2), (x ** 2).sum(axis=2), rtol=1e-12)
    # heads are rotated independently with the same angles
    assert np.allclose(oracle.rope(x[:, :1], np.arange(6), theta), r[:, :1])
    # inverse rotation: rotating by -p undoes p (angles are linear in the position)
    back = oracle.rope(r, -np.arange(6), theta)
    assert np.allclose(back, x, rtol=1e-10, atol=1e-12)


# ---- attention ----------------------------------------------------------------

def attention_lib(q, k, v):
    L, H, dh = q.shape
    out = np.empty_like(q)
    for h in range(H):
        p = scipy.special.softmax(q[:, h] @ k[:, h].T / math.sqrt(dh), axis=1)
        out[:, h] = p @ v[:, h]
    return out


def test_attention_against_library_and_sdpa():
    L, H, dh = 11, 3, 8
    q, k, v = (rng.standard_normal((L, H, dh)) for _ in range(3))
    ours = oracle.attention(q, k, v)
    assert np.allclose(ours, attention_lib(q, k, v), rtol=1e-11, atol=1e-13)
    tq, tk, tv = (torch.from_numpy(a).permute(1, 0, 2)[None] for a in (q, k, v))
    ref = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, is_causal=False)[0].permute(1, 0, 2).numpy()
    assert np.allclose(ours, ref, rtol=1e-10, atol=1e-12)


def test_attention_is_bidirectional_and_special_cases():
    L, H, dh = 9, 2, 4
    q, k, v = (rng.standard_normal((L, H, dh)) for _ in range(3))
    base = oracle.attention(q, k, v)
    # permuting the keys/values leaves every output unchanged (no causal mask)
    perm = rng.permutation(L)
    assert np.allclose(oracle.attention(q, k[perm], v[perm]), base, rtol=1e-11)
    # the first query sees the last value
    v2 = v.copy(); v2[-1] += 1.0
    assert np.abs(oracle.attention(q, k, v2)[0] - base[0]).max() > 1e-3
    # equal keys -> plain average of the values
    keq = np.broadcast_to(k[:1], k.shape)
    assert np.allclose(oracle.attention(q, keq, v), np.broadcast_to(v.mean(axis=0), v.shape), rtol=1e-12)
    # one key -> its value
    assert np.allclose(oracle.attention(q[:1], k[:1], v[:1]), v[:1])
    # the 1/sqrt(dh) scale: q.k = dh*ln(3)*... two keys with scores s and 0
    q1 = np.zeros((1, 1, 4)); q1[0, 0, 0] = 2.0
    k2 = np.zeros((2, 1, 4)); k2[0, 0, 0] = math.log(3.0)      # score 2 ln3 / sqrt(4) = ln 3
    v2 = np.zeros((2, 1, 4)); v2[0, 0, 0] = 1.0
    out = oracle.attention(np.repeat(q1, 2, axis=0), k2, v2)
    assert np.allclose(out[0, 0, 0], 0.75, rtol=1e-13)


# ---- SwiGLU -------------------------------------------------------------------

def test_swiglu_values():
    g = np.array([0.0, 1.0, -1.0, 30.0, -30.0])
    u = np.array([5.0, 2.0, 2.0, 1.0, 1.0])
    out = oracle.swiglu(g, u)
    exp = [0.0, 2 * 0.7310585786300049, 2 * -0.2689414213699951, 30.0, -30 * math.exp(-30)]
    assert np.allclose(out, exp, rtol=1e-12, atol=1e-15)
    x = rng.standard_normal(100) * 3
    ref = torch.nn.functional.silu(torch.from_numpy(x)).numpy() * x[::-1]
    assert np.allclose(oracle.swiglu(x, x[::-1].copy()), ref, rtol=1e-12)


# ---- whole forward ------------------------------------------------------------

def torch_forward(cfg, w, tokens):
    """Independent fp64 forward out of torch library routines (F.rms_norm,
    F.scaled_dot_product_attention, F.silu, matmul) plus a complex-number RoPE."""
    F = torch.nn.functional
    d, H, dh, f = cfg["d_model"], cfg["n_heads"], cfg["head_dim"], cfg["d_ffn"]
    W = lambda t: t.to(torch.float64)
    B, L = tokens.shape
    x = W(w["embed"])[tokens.long()]
    pos = torch.arange(L, dtype=torch.float64)
    freqs = cfg["rope_theta"] ** (-torch.arange(0, dh // 2, dtype=torch.float64) * 2 / dh)
    rot = torch.polar(torch.ones(L, dh // 2, dtype=torch.float64), pos[:, None] * freqs[None])

    def rope(t):                                   # t [B, L, H, dh]
        z = torch.complex(t[..., : dh // 2], t[..., dh // 2:]) * rot[None, :, None, :]
        return torch.cat([z.real, z.imag], dim=-1)

    for l in range(cfg["n_layers"]):
        h = F.rms_norm(x, (d,), W(w["attn_norm"][l]), cfg["rms_eps"])
        qkv = h @ W(w["wqkv"][l]).T
        q, k, v = (t.reshape(B, L, H, dh) for t in qkv.split(d, dim=-1))
        q, k = rope(q), rope(k)
        a = F.scaled_dot_product_attention(q.transpose(1, 2), k.transpose(1, 2), v.transpose(1, 2))
        x = x + a.transpose(1, 2).reshape(B, L, d) @ W(w["wo"][l]).T
        h = F.rms_norm(x, (d,), W(w["ffn_norm"][l]), cfg["rms_eps"])
        gu = h @ W(w["w_gate_up"][l]).T
        x = x + (F.silu(gu[..., :f]) * gu[..., f:]) @ W(w["w_down"][l]).T
    return (F.rms_norm(x, (d,), W(w["final_norm"]), cfg["rms_eps"]) @ W(w["lm_head"]).T).reshape(B * L, -1).numpy()


@pytest.mark.parametrize("std,batch", [(0.02, 1), (0.2, 2)])
def test_forward_against_torch_library_ops(std, batch):
    cfg = dict(synth.CONFIGS["tiny"], n_layers=2, vocab=300, mask_id=299, prompt=5, gen=8, d_ffn=80,
               d_model=64, n_heads=2, head_dim=32)
    w = synth.make_weights(cfg, std=std)
    w["attn_norm"][0] = synth.normal_bf16((64,), 1.0, 5, "g")      # non-trivial gains
    w["final_norm"] = synth.normal_bf16((64,), 1.0, 6, "g")
    tokens, _, _ = synth.make_state(cfg, batch=batch)
    ours = oracle.forward(synth.model_config(cfg), weights_bits(w), tokens.numpy())
    ref = torch_forward(cfg, w, tokens)
    assert np.allclose(ours, ref, rtol=1e-9, atol=1e-11)


def test_forward_zero_layers_and_dead_branches():
    cfg = dict(synth.CONFIGS["tiny"], n_layers=0, vocab=50, mask_id=49, prompt=3, gen=4, d_model=16,
               n_heads=2, head_dim=8, d_ffn=24)
    w = synth.make_weights(cfg)
    tokens, _, _ = synth.make_state(cfg)
    E = oracle.bf16_to_f64(bits(w["embed"])); Wv = oracle.bf16_to_f64(bits(w["lm_head"]))
    x = E[tokens.numpy()[0]]
    ref = (x / np.sqrt((x * x).mean(axis=1, keepdims=True) + 1e-5)) @ Wv.T
    ours = oracle.forward(synth.model_config(cfg), weights_bits(w), tokens.numpy())
    assert np.allclose(ours, ref, rtol=1e-12)
    # a layer whose output projections are zero leaves the residual stream alone
    cfg1 = dict(cfg, n_layers=1)
    w1 = synth.make_weights(cfg1)
    w1["wo"][0].zero_(); w1["w_down"][0].zero_()
    ours1 = oracle.forward(synth.model_config(cfg1), weights_bits(w1), tokens.numpy())
    assert np.allclose(ours1, ref, rtol=1e-12)


def test_forward_sequences_in_a_batch_are_independent():
    cfg = dict(synth.CONFIGS["tiny"], vocab=120, mask_id=119, prompt=4, gen=5, d_model=32, n_heads=2,
               head_dim=16, d_ffn=40, n_layers=1)
    w = weights_bits(synth.make_weights(cfg))
    tokens, _, _ = synth.make_state(cfg, batch=3)
    t = tokens.numpy()
    both = oracle.forward(synth.model_config(cfg), w, t).reshape(3, 9, -1)
    for b in range(3):
        alone = oracle.forward(synth.model_config(cfg), w, t[b:b + 1])
        assert np.allclose(both[b], alone, rtol=1e-12)


# ---- row phase ----------------------------------------------------------------

def test_softmax_row_definition():
    V, mid = 37, 36
    row = bf(rng.standard_normal(V) * 3)
    arg, conf, prob = oracle.softmax_row(row, mid)
    x = oracle.bf16_to_f64(row)[:mid]
    ref = scipy.special.softmax(x)
    assert abs(prob.sum() - 1.0) < 1e-12                        # rows sum to 1
    assert prob[mid] == 0.0
    assert np.allclose(prob[:mid], ref, rtol=1e-12)
    assert arg == int(np.argmax(x)) and abs(conf - ref.max()) < 1e-15


def test_closed_form_confidences():
    V, mid = 17, 16                         # 16 legal ids
    for line in open(os.path.join(GOLDEN, "closed_form_conf.txt")):
        if line.startswith("#") or not line.strip():
            continue
        m, expected = (float(t) for t in line.split())
        row = np.zeros(V); row[5] = math.log(m); row[mid] = 50.0   # a huge [MASK] logit must not matter
        rb = bf(row)
        arg, conf, _ = oracle.softmax_row(rb, mid)
        lm = oracle.bf16_to_f64(rb)[5]                            # the bf16-rounded ln m
        assert abs(conf - 1.0 / (1.0 + 15.0 * math.exp(-lm))) < 1e-14
        assert abs(conf - expected) < 5e-3                        # bf16 rounding of ln m only
        assert arg == (5 if m > 1 else 0)                         # uniform row: lowest id


def test_row_phase_ties_mask_and_activity():
    V, mid = 40, 7
    rows = np.zeros((3, V))
    rows[0, [9, 3, 30]] = 2.5                                    # equal maxima -> lowest id
    rows[1, mid] = 9.0; rows[1, 20] = 1.0                       # [MASK] is never predicted
    rows[2, 11] = 4.0
    pred, conf = oracle.row_phase(bf(rows), mid, active=[1, 1, 0])
    assert list(pred) == [3, 20, -1] and conf[2] == 0.0
    assert conf.dtype == np.float32
    assert abs(conf[0] - 1.0 / (3 + 36 * math.exp(-2.5))) < 1e-7
    assert abs(conf[1] - 1.0 / (1 + 38 * math.exp(-1.0))) < 1e-7


def test_forward_row_subset_equals_full():
    cfg = dict(synth.CONFIGS["tiny"], vocab=120, mask_id=119, prompt=4, gen=5, d_model=32, n_heads=2,
               head_dim=16, d_ffn=40, n_layers=1)
    w = weights_bits(synth.make_weights(cfg))
    tokens, _, _ = synth.make_state(cfg, batch=2)
    full = oracle.forward(synth.model_config(cfg), w, tokens.numpy())
    rows = [17, 0, 9]
    assert np.array_equal(oracle.forward(synth.model_config(cfg), w, tokens.numpy(), rows=rows), full[rows])
