"""Pins for the CPU oracle: each piece is checked against something other than itself --
closed forms, invariants, library routines (numpy/scipy/torch fp64), brute force on tiny inputs,
and special cases of the whole layer that reduce to one-line computations."""
import math
import os

import numpy as np
import pytest
import scipy.special
import torch

from oracle import oracle
from paper_2505_22758_amd import synth

RNG = np.random.default_rng(22758)


def bf16_bits(a):
    """numpy float array (bf16-representable after rounding by torch) -> uint16 bit patterns."""
    t = torch.from_numpy(np.asarray(a, dtype=np.float32)).to(torch.bfloat16)
    return t.view(torch.int16).numpy().view(np.uint16).copy()


# ---------------------------------------------------------------- formats
def test_f16_decode_matches_numpy_for_all_patterns():
    L = oracle.lib()
    bits = np.arange(65536, dtype=np.uint16)
    ref = bits.view(np.float16).astype(np.float64)
    got = np.array([L.ffo_f16_to_f64(int(b)) for b in bits])
    fin = np.isfinite(ref)
    assert np.array_equal(got[fin], ref[fin])
    assert np.all(np.isnan(got[np.isnan(ref)]))
    assert np.array_equal(got[np.isinf(ref)], ref[np.isinf(ref)])


def test_bf16_round_ties_to_even_and_matches_torch_on_fp32_inputs():
    assert oracle.bf16_round(1.0) == 0x3F80
    assert oracle.bf16_round(1.0 + 2.0 ** -8) == 0x3F80          # tie -> even mantissa 0
    assert oracle.bf16_round(1.0 + 3 * 2.0 ** -8) == 0x3F82      # tie -> even mantissa 2
    assert oracle.bf16_round(1.0 + 2.0 ** -8 + 2.0 ** -30) == 0x3F81  # just above the tie
    assert oracle.bf16_round(-2.5) == 0xC020
    assert oracle.bf16_round(0.0) == 0
    x = RNG.standard_normal(20000).astype(np.float32) * np.float32(3.0)
    ref = bf16_bits(x)
    got = np.array([oracle.bf16_round(float(v)) for v in x], dtype=np.uint16)
    assert np.array_equal(got, ref)
    # widening is exact
    assert np.array_equal(oracle.bf16_bits_to_f64(ref), torch.from_numpy(x).to(torch.bfloat16).double().numpy())


# ---------------------------------------------------------------- RoPE
def test_rope_closed_forms():
    hd, theta = 64, 10000.0
    q = RNG.standard_normal(hd)
    k = RNG.standard_normal(hd)
    # position 0 is the identity
    assert np.array_equal(oracle.rope(q, 0, theta), q)
    # pair (0, hd/2) has frequency theta^0 = 1: rotated by exactly `pos` radians
    p = 7
    r = oracle.rope(q, p, theta)
    assert r[0] == pytest.approx(q[0] * math.cos(p) - q[hd // 2] * math.sin(p), abs=1e-14)
    assert r[hd // 2] == pytest.approx(q[hd // 2] * math.cos(p) + q[0] * math.sin(p), abs=1e-14)
    # last pair has frequency theta^(-(hd-2)/hd)
    f = theta ** (-(hd - 2) / hd)
    i = hd // 2 - 1
    assert r[i] == pytest.approx(q[i] * math.cos(p * f) - q[i + hd // 2] * math.sin(p * f), abs=1e-14)
    # per-pair norms are preserved
    half = hd // 2
    assert np.allclose(r[:half] ** 2 + r[half:] ** 2, q[:half] ** 2 + q[half:] ** 2, rtol=1e-13)
    # rotations compose additively
    assert np.allclose(oracle.rope(oracle.rope(q, 5, theta), 11, theta), oracle.rope(q, 16, theta), atol=1e-12)
    # the inner product depends only on the position difference
    d0 = oracle.rope(q, 3, theta) @ oracle.rope(k, 1, theta)
    d1 = oracle.rope(q, 1003, theta) @ oracle.rope(k, 1001, theta)
    assert d0 == pytest.approx(d1, abs=1e-9)
    assert abs(d0 - q @ k) > 1e-3     # ...and the rotation is not a no-op


def test_rope_theta_is_used():
    q = RNG.standard_normal(128)
    a = oracle.rope(q, 9, 10000.0)
    b = oracle.rope(q, 9, 500000.0)
    assert a[0] == pytest.approx(b[0], abs=1e-14)     # frequency-1 pair is theta independent
    assert abs(a[5] - b[5]) > 1e-6


# ---------------------------------------------------------------- RMSNorm, SiLU
def test_rmsnorm_closed_forms():
    d, eps = 512, 1e-5
    ones = bf16_bits(np.ones(d))
    x = RNG.standard_normal(d) * 0.37
    y = oracle.rmsnorm(x, ones, eps)
    ms = np.mean(x * x)
    assert np.sqrt(np.mean(y * y)) == pytest.approx(1.0 / math.sqrt(1.0 + eps / ms), rel=1e-13)
    # scale invariance up to eps
    y2 = oracle.rmsnorm(1000.0 * x, ones, 0.0)
    y3 = oracle.rmsnorm(x, ones, 0.0)
    assert np.allclose(y2, y3, rtol=1e-12)
    # gain is applied elementwise, after normalisation
    g = RNG.standard_normal(d).astype(np.float32)
    gb = bf16_bits(g)
    yg = oracle.rmsnorm(x, gb, eps)
    assert np.allclose(yg, y * oracle.bf16_bits_to_f64(gb), rtol=1e-14)
    # constant vector c: every output is c / sqrt(c^2 + eps)
    yc = oracle.rmsnorm(np.full(d, 3.0), ones, 0.25)
    assert np.allclose(yc, 3.0 / math.sqrt(9.25), rtol=1e-15)


def test_silu_identities_and_library():
    assert oracle.silu(0.0) == 0.0
    for z in (0.1, 1.0, 3.7, 12.0):
        assert oracle.silu(z) - oracle.silu(-z) == pytest.approx(z, rel=1e-14)   # z*(sigma(z)+sigma(-z)) = z
        assert oracle.silu(z) + oracle.silu(-z) == pytest.approx(z * math.tanh(z / 2), rel=1e-13)
        assert oracle.silu(z) == pytest.approx(z * scipy.special.expit(z), rel=1e-14)
    assert oracle.silu(50.0) == pytest.approx(50.0, rel=1e-15)
    assert abs(oracle.silu(-50.0)) < 1e-19


# ---------------------------------------------------------------- matvec and dequantisation
def test_matvec_against_numpy_fp64_nonsquare():
    n, k = 37, 256
    w = RNG.standard_normal((n, k)).astype(np.float32)
    wt = torch.from_numpy(w).to(torch.bfloat16)
    x = RNG.standard_normal(k)
    y = oracle.matvec({"w": wt}, x)
    ref = wt.double().numpy() @ x
    assert y.shape == (n,)
    assert np.allclose(y, ref, rtol=1e-12, atol=1e-12)


def test_int8_dequant_exhaustive_and_exact_in_fp32():
    L = oracle.lib()
    scales = np.array([0.02 / 73.6, 3.051e-4, 1.0, 6.1e-5, 2.5e-4 * 1.25], dtype=np.float16)
    for s in scales:
        sb = int(s.view(np.uint16))
        for q in range(-127, 128):
            v = L.ffo_dequant_int8(q, sb)
            assert v == q * float(s)                      # closed form in exact arithmetic
            assert float(np.float32(v)) == v              # representable in fp32 (<= 7+11 bits)


def test_int4_dequant_exhaustive_nibble_order_and_groups():
    L = oracle.lib()
    # nibble order: low nibble = even k
    row = np.array([0x21, 0xF4], dtype=np.uint8)
    one = int(np.float16(1.0).view(np.uint16))
    zero = int(np.float16(0.0).view(np.uint16))
    got = [L.ffo_dequant_int4(row.ctypes.data, k, one, zero) for k in range(4)]
    assert got == [1.0, 2.0, 4.0, 15.0]
    for s in np.array([0.02 / 6.5, 3.8e-3, 1.5], dtype=np.float16):
        for z in range(16):
            zb = int(np.float16(z).view(np.uint16))
            sb = int(s.view(np.uint16))
            for code in range(16):
                b = np.array([code | (code << 4)], dtype=np.uint8)
                v = L.ffo_dequant_int4(b.ctypes.data, 1, sb, zb)
                assert v == (code - z) * float(s)
                assert float(np.float32(v)) == v
    # group indexing along K through the matrix path: scale/zero change every 128 columns
    n, k = 3, 384
    codes = RNG.integers(0, 16, size=(n, k)).astype(np.uint8)
    packed = torch.from_numpy((codes[:, 0::2] | (codes[:, 1::2] << 4)).astype(np.uint8))
    s = torch.tensor(RNG.uniform(0.001, 0.004, size=(n, 3)), dtype=torch.float16)
    z = torch.tensor(RNG.integers(0, 16, size=(n, 3)), dtype=torch.float16)
    deq = oracle.dequant_matrix({"w": packed, "s": s, "z": z})
    ref = (codes.astype(np.float64) - np.repeat(z.double().numpy(), 128, axis=1)) * np.repeat(s.double().numpy(), 128, axis=1)
    assert np.array_equal(deq.astype(np.float64), ref)
    x = RNG.standard_normal(k)
    assert np.allclose(oracle.matvec({"w": packed, "s": s, "z": z}, x), ref @ x, rtol=1e-12)


def test_int8_matrix_path_row_scales():
    n, k = 5, 64
    q = torch.from_numpy(RNG.integers(-127, 128, size=(n, k)).astype(np.int8))
    s = torch.tensor(RNG.uniform(1e-4, 5e-4, size=(n,)), dtype=torch.float16)
    deq = oracle.dequant_matrix({"w": q, "s": s})
    ref = q.double().numpy() * s.double().numpy()[:, None]
    assert np.array_equal(deq.astype(np.float64), ref)


# ---------------------------------------------------------------- core attention
def _rand_kv(n, hd):
    K = bf16_bits(RNG.standard_normal((n, hd)))
    V = bf16_bits(RNG.standard_normal((n, hd)))
    return K, V


def test_attention_against_full_softmax_matrix():
    """Brute force: materialise the whole [heads, keys] score matrix, library softmax, dense P V."""
    hd, n, heads = 64, 57, 5
    K, V = _rand_kv(n, hd)
    Q = RNG.standard_normal((heads, hd))
    alpha = 1.0 / math.sqrt(hd)
    Kf, Vf = oracle.bf16_bits_to_f64(K), oracle.bf16_bits_to_f64(V)
    P = scipy.special.softmax(alpha * (Q @ Kf.T), axis=1)
    O = P @ Vf
    for h in range(heads):
        o, p = oracle.attention_head(Q[h], K, V, alpha, return_probs=True)
        assert np.allclose(o, O[h], rtol=1e-12, atol=1e-13)
        assert np.allclose(p, P[h], rtol=1e-12, atol=1e-15)
        assert abs(p.sum() - 1.0) < 1e-12          # rows of the softmax sum to one


def test_attention_single_key_returns_its_value():
    hd = 64
    K, V = _rand_kv(1, hd)
    o = oracle.attention_head(RNG.standard_normal(hd) * 10, K, V, 0.125)
    assert np.array_equal(o, oracle.bf16_bits_to_f64(V)[0])


def test_attention_is_invariant_to_key_order_and_uses_alpha():
    hd, n = 32, 40
    K, V = _rand_kv(n, hd)
    q = RNG.standard_normal(hd)
    perm = RNG.permutation(n)
    a = oracle.attention_head(q, K, V, 0.2)
    b = oracle.attention_head(q, K[perm].copy(), V[perm].copy(), 0.2)
    assert np.allclose(a, b, rtol=1e-12, atol=1e-14)
    # alpha = 0 gives the plain mean of the values; a large alpha picks the arg-max key
    m = oracle.attention_head(q, K, V, 0.0)
    assert np.allclose(m, oracle.bf16_bits_to_f64(V).mean(axis=0), rtol=1e-12, atol=1e-14)
    s = oracle.bf16_bits_to_f64(K) @ q
    hard = oracle.attention_head(q, K, V, 1e4)
    assert np.allclose(hard, oracle.bf16_bits_to_f64(V)[int(np.argmax(s))], atol=1e-9)


def test_split_kv_merge_identity_holds_for_the_oracle_definition():
    """The kernel's split-KV partial (max, denominator, unnormalised output) merge must equal the
    full softmax for any split; checked here on the definition so the identity itself is pinned."""
    hd, n = 64, 101
    K, V = _rand_kv(n, hd)
    q = RNG.standard_normal(hd)
    alpha = 0.125
    full = oracle.attention_head(q, K, V, alpha)
    s = alpha * (oracle.bf16_bits_to_f64(K) @ q)
    for nsplit in (1, 2, 7, 32):
        bounds = np.linspace(0, n, nsplit + 1).astype(int)
        parts = []
        for a, b in zip(bounds[:-1], bounds[1:]):
            if b == a:
                continue
            o = oracle.attention_head(q, K[a:b].copy(), V[a:b].copy(), alpha)
            m = s[a:b].max()
            l = np.exp(s[a:b] - m).sum()
            parts.append((m, l, o))
        M = max(p[0] for p in parts)
        Lg = sum(p[1] * math.exp(p[0] - M) for p in parts)
        merged = sum(p[2] * (p[1] * math.exp(p[0] - M) / Lg) for p in parts)
        assert np.allclose(merged, full, rtol=1e-12, atol=1e-14)


# ---------------------------------------------------------------- whole layer / model
def _zero_like(m):
    return {"w": torch.zeros_like(m["w"])}


def test_zero_output_projections_leave_residual_unchanged(tiny_model_cpu):
    S, seed, layers, head, _ = tiny_model_cpu
    mod = []
    for lw in layers:
        lw2 = dict(lw)
        lw2["wo"] = _zero_like(lw["wo"])
        lw2["w_down"] = _zero_like(lw["w_down"])
        mod.append(lw2)
    M = oracle.OracleModel(S, mod, head)
    kv = M.new_kv(1, 8)
    tok = 1234
    logits = M.decode_step([tok], [3], kv)[0]
    # one-line computation with library routines: W_lm * RMSNorm(E[tok]) * g_f
    e = head["embed"][tok].double().numpy()
    n = e / np.sqrt(np.mean(e * e) + S.rms_eps) * head["final_norm"].double().numpy()
    ref = head["lm_head"]["w"].double().numpy() @ n
    assert np.allclose(logits, ref, rtol=1e-12, atol=1e-13)


def test_first_token_attends_to_its_own_stored_value_and_gqa_head_mapping(tiny_model_cpu):
    """pos = 0: softmax over one key is 1, so the attention output of q head h is the bf16 value
    just stored for kv head h // G.  With W_o = I (d_model == n_q_heads*head_dim at this shape)
    and W_down = 0 the layer output is x + that vector."""
    S, seed, layers, head, _ = tiny_model_cpu
    assert S.d_model == S.q_dim
    lw = dict(layers[0])
    lw["wo"] = {"w": torch.eye(S.d_model, dtype=torch.bfloat16)}
    lw["w_down"] = _zero_like(lw["w_down"])
    M = oracle.OracleModel(S.replace(n_layers=1), [lw], head)
    x0 = RNG.standard_normal(S.d_model)
    x = x0.copy()
    Kc = np.zeros((4, S.n_kv_heads, S.head_dim), dtype=np.uint16)
    Vc = np.zeros_like(Kc)
    M.layer_step(0, x, Kc, Vc, 0)
    assert not Kc[1:].any() and not Vc[1:].any() and Vc[0].any()
    # stored V is the bf16 rounding of W_v RMSNorm(x0)
    n = oracle.rmsnorm(x0, lw["attn_norm"], S.rms_eps)
    v = lw["wv"]["w"].double().numpy() @ n
    assert np.array_equal(Vc[0].reshape(-1), bf16_bits(v.astype(np.float32)))  # v far from fp32 double-rounding ties
    G = S.n_q_heads // S.n_kv_heads
    vstored = oracle.bf16_bits_to_f64(Vc[0])                   # [Hkv, hd]
    expect = x0 + np.concatenate([vstored[h // G] for h in range(S.n_q_heads)])
    assert np.allclose(x, expect, rtol=0, atol=1e-13)
    # stored K is the bf16 rounding of the rotated key; at pos 0 the rotation is the identity
    k = lw["wk"]["w"].double().numpy() @ n
    assert np.array_equal(Kc[0].reshape(-1), bf16_bits(k.astype(np.float32)))


def test_gqa_equals_mha_with_replicated_kv_heads(tiny_model_cpu):
    S, seed, layers, head, _ = tiny_model_cpu
    G = S.n_q_heads // S.n_kv_heads
    hd = S.head_dim
    lw = layers[1]

    def rep(w):  # [Hkv*hd, d] -> [Hq*hd, d], each kv head copied G times
        return {"w": w["w"].view(S.n_kv_heads, 1, hd, -1).expand(-1, G, -1, -1).reshape(S.n_q_heads * hd, -1).contiguous()}

    lw_mha = dict(lw)
    lw_mha["wk"], lw_mha["wv"] = rep(lw["wk"]), rep(lw["wv"])
    S1 = S.replace(n_layers=1)
    A = oracle.OracleModel(S1, [lw], head)
    Bm = oracle.OracleModel(S1.replace(n_kv_heads=S.n_q_heads), [lw_mha], head)
    T = 9
    Kp, Vp = synth.make_kv_prefill(S, seed, 1, 0, T, "cpu")
    Ka = np.zeros((T + 2, S.n_kv_heads, hd), dtype=np.uint16)
    Va = np.zeros_like(Ka)
    Ka[:T], Va[:T] = oracle._np(Kp), oracle._np(Vp)
    Kb = np.repeat(Ka, G, axis=1).copy()
    Vb = np.repeat(Va, G, axis=1).copy()
    x0 = RNG.standard_normal(S.d_model)
    xa, xb = x0.copy(), x0.copy()
    for pos in (T, T + 1):
        A.layer_step(0, xa, Ka, Va, pos)
        Bm.layer_step(0, xb, Kb, Vb, pos)
        assert np.array_equal(xa, xb)
        assert np.array_equal(np.repeat(Ka, G, axis=1), Kb)


def _torch_reference_step(S, layers, head, tok, pos, Kc, Vc):
    """Independent composition from torch fp64 library routines (rms_norm, matmul, SDPA, silu).
    Kc/Vc: lists per layer of float64 tensors [rows, Hkv, hd] with rows 0..pos-1 valid."""
    F = torch.nn.functional
    d, hd, Hq, Hkv = S.d_model, S.head_dim, S.n_q_heads, S.n_kv_heads
    x = head["embed"][tok].double()
    inv = S.rope_theta ** (-torch.arange(0, hd, 2, dtype=torch.float64) / hd)
    ang = pos * inv
    cos, sin = torch.cos(ang).repeat(2), torch.sin(ang).repeat(2)

    def rot(t):  # [H, hd]
        t1, t2 = t[:, : hd // 2], t[:, hd // 2:]
        return t * cos + torch.cat([-t2, t1], dim=1) * sin

    for l, lw in enumerate(layers):
        n = F.rms_norm(x, (d,), lw["attn_norm"].double(), S.rms_eps)
        q = (lw["wq"]["w"].double() @ n).view(Hq, hd)
        k = (lw["wk"]["w"].double() @ n).view(Hkv, hd)
        v = (lw["wv"]["w"].double() @ n).view(Hkv, hd)
        q, k = rot(q), rot(k)
        Kc[l][pos] = k.float().to(torch.bfloat16).double()
        Vc[l][pos] = v.float().to(torch.bfloat16).double()
        Kall = Kc[l][: pos + 1].permute(1, 0, 2)   # [Hkv, T, hd]
        Vall = Vc[l][: pos + 1].permute(1, 0, 2)
        o = F.scaled_dot_product_attention(q.view(1, Hq, 1, hd), Kall.unsqueeze(0), Vall.unsqueeze(0),
                                           enable_gqa=True)
        x = x + lw["wo"]["w"].double() @ o.reshape(-1)
        m = F.rms_norm(x, (d,), lw["ffn_norm"].double(), S.rms_eps)
        h = F.silu(lw["w_gate"]["w"].double() @ m) * (lw["w_up"]["w"].double() @ m)
        x = x + lw["w_down"]["w"].double() @ h
    n = F.rms_norm(x, (d,), head["final_norm"].double(), S.rms_eps)
    return head["lm_head"]["w"].double() @ n


def test_whole_model_against_torch_fp64_library_composition(tiny_model_cpu):
    S, seed, layers, head, M = tiny_model_cpu
    T0, steps = 20, 3
    kv = M.new_kv(1, T0 + steps)
    Kc, Vc = [], []
    for l in range(S.n_layers):
        k, v = synth.make_kv_prefill(S, seed, l, 0, T0, "cpu")
        kv[l, 0, 0, :T0], kv[l, 0, 1, :T0] = oracle._np(k), oracle._np(v)
        Kc.append(torch.cat([k.double(), torch.zeros(steps, S.n_kv_heads, S.head_dim, dtype=torch.float64)]))
        Vc.append(torch.cat([v.double(), torch.zeros(steps, S.n_kv_heads, S.head_dim, dtype=torch.float64)]))
    toks = synth.make_tokens(S, seed, steps, 1)
    for s in range(steps):
        got = M.decode_step(toks[s].numpy(), [T0 + s], kv)[0]
        ref = _torch_reference_step(S, layers, head, int(toks[s, 0]), T0 + s, Kc, Vc).numpy()
        assert np.allclose(got, ref, rtol=1e-9, atol=1e-10)
        for l in range(S.n_layers):
            assert np.array_equal(oracle.bf16_bits_to_f64(kv[l, 0, 0, T0 + s]), Kc[l][T0 + s].numpy())


def test_batch_rows_are_independent_sequences(tiny_model_cpu):
    S, seed, layers, head, M = tiny_model_cpu
    T0 = 6
    kvb = M.new_kv(2, T0 + 1)
    for l in range(S.n_layers):
        for b in range(2):
            k, v = synth.make_kv_prefill(S, seed, l, b, T0, "cpu")
            kvb[l, b, 0, :T0], kvb[l, b, 1, :T0] = oracle._np(k), oracle._np(v)
    toks = np.array([17, 4000], dtype=np.int32)
    both = M.decode_step(toks, [T0, T0 - 2], kvb.copy())
    for b, pos in ((0, T0), (1, T0 - 2)):
        kv1 = kvb[:, b:b + 1].copy()
        one = M.decode_step(toks[b:b + 1], [pos], kv1)
        assert np.array_equal(one[0], both[b])


def test_quantised_layer_equals_bf16_free_dense_evaluation():
    """int8/int4 models: the step must equal the same step run on explicitly dequantised fp64
    matrices (numpy), i.e. quantisation enters only through w = q*s / (q-z)*s."""
    S = synth.TINY.replace(n_layers=1, d_ffn=1408)   # int4 groups need K % 128 == 0
    for wd in (synth.WDTYPE_INT8, synth.WDTYPE_INT4):
        lw = synth.make_layer(S, 7, 0, wd, "cpu")
        head = synth.make_head(S, 7, wd, "cpu")
        M = oracle.OracleModel(S, [lw], head)
        kv = M.new_kv(1, 4)
        got = M.decode_step([99], [0], kv)[0]
        W = {k: oracle.dequant_matrix(lw[k]).astype(np.float64) for k in synth.LAYER_MATS}
        x = head["embed"][99].double().numpy()
        n = oracle.rmsnorm(x, lw["attn_norm"], S.rms_eps)
        v = W["wv"] @ n                      # pos 0: attention output = stored value
        vs = oracle.bf16_bits_to_f64(bf16_bits(v.astype(np.float32))).reshape(S.n_kv_heads, S.head_dim)
        G = S.n_q_heads // S.n_kv_heads
        o = np.concatenate([vs[h // G] for h in range(S.n_q_heads)])
        x = x + W["wo"] @ o
        m = oracle.rmsnorm(x, lw["ffn_norm"], S.rms_eps)
        g = W["w_gate"] @ m
        h = g * scipy.special.expit(g) * (W["w_up"] @ m)
        x = x + W["w_down"] @ h
        ref = oracle.dequant_matrix(head["lm_head"]).astype(np.float64) @ oracle.rmsnorm(x, head["final_norm"], S.rms_eps)
        assert np.allclose(got, ref, rtol=1e-9, atol=1e-11)
        std = oracle.dequant_matrix(lw["w_up"]).std()
        assert 0.015 < std < 0.03


# ---------------------------------------------------------------- fixtures from the paper's tables
def test_shapes_match_the_papers_configuration_table():
    path = os.path.join(os.path.dirname(__file__), "golden", "llama_shapes.txt")
    rows = [l.split() for l in open(path) if l.strip() and not l.startswith("#")]
    assert len(rows) == 2
    for name, L, d, f, hd, hq, hkv, params in rows:
        S = synth.SHAPES[name]
        assert (S.n_layers, S.d_model, S.d_ffn, S.head_dim, S.n_q_heads, S.n_kv_heads) == tuple(
            int(v) for v in (L, d, f, hd, hq, hkv))
        assert S.params_per_layer() == int(params)
