"""Pins for the CPU oracle: every operator and the whole forward are checked against
something other than the oracle itself -- library routines (torch, numpy, the
transformers Qwen2 implementation run in fp64), closed forms, invariants, and an
independently structured numpy brute force.  No GPU needed."""
import numpy as np
import pytest
import torch

import oracle
import synth
from synth import BF16, F16

OPS = oracle.Ops("f64")
RNG = np.random.default_rng(1234)


def rel_l2(a, b):
    a = np.asarray(a, dtype=np.float64); b = np.asarray(b, dtype=np.float64)
    return float(np.linalg.norm(a - b) / max(np.linalg.norm(b), 1e-300))


# --------------------------------------------------------------------------- storage formats
def test_upcast_matches_library_casts():
    bits = np.arange(0, 65536, 7, dtype=np.uint16)
    f16 = bits.view(np.float16).astype(np.float64)
    bf = torch.from_numpy(bits.view(np.int16).copy()).view(torch.bfloat16).to(torch.float64).numpy()
    for b, x16, xbf in zip(bits, f16, bf):
        a = OPS.upcast(int(b), F16); c = OPS.upcast(int(b), BF16)
        assert (np.isnan(a) and np.isnan(x16)) or a == x16
        assert (np.isnan(c) and np.isnan(xbf)) or c == xbf


def test_round_kv_matches_library_rne():
    xs = np.concatenate([
        RNG.standard_normal(4000).astype(np.float32) * 3,
        RNG.standard_normal(500).astype(np.float32) * 1e-6,   # fp16 subnormal range
        RNG.standard_normal(200).astype(np.float32) * 1e5,    # fp16 overflow
        # exact ties in both formats
        np.array([1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8, 1.0 + 2.0 ** -11, 1.0 + 3 * 2.0 ** -11,
                  -(2.0 + 2.0 ** -7), 65520.0, 65519.9, 0.0, 2.0 ** -25, 2.0 ** -24 * 1.5], dtype=np.float32),
    ])
    want_bf = torch.from_numpy(xs).to(torch.bfloat16).to(torch.float64).numpy()
    with np.errstate(over="ignore"):
        want_f16 = xs.astype(np.float16).astype(np.float64)
    for x, wb, wh in zip(xs, want_bf, want_f16):
        assert OPS.round_kv(float(x), BF16) == wb, x
        assert OPS.round_kv(float(x), F16) == wh, x


def test_round_kv_fp8_against_the_code_table_brute_force_and_torch():
    """The 8-bit cache format (e4m3: 4 exponent bits with bias 7, 3 mantissa bits, no infinities, largest finite value
    448).  Three references that share nothing with the oracle's rounding: the value of every code written out from
    the format definition, a brute-force search for the nearest finite value (ties to the even mantissa), and
    torch's float8_e4m3fn cast (which saturates nothing: compared inside the finite range only)."""
    FP8 = synth.FP8
    values = []
    for code in range(256):
        e, m = (code >> 3) & 15, code & 7
        if e == 15 and m == 7:
            assert np.isnan(OPS.upcast(code, FP8))
            continue
        v = (m * 2.0 ** -9) if e == 0 else (8 + m) * 2.0 ** (e - 10)
        v = -v if code & 0x80 else v
        assert OPS.upcast(code, FP8) == v
        assert OPS.round_kv(v, FP8) == v                    # representable values are fixed points
        values.append((v, m))
    assert max(v for v, _ in values) == 448.0 and min(abs(v) for v, _ in values if v != 0) == 2.0 ** -9
    finite = sorted(set(v for v, _ in values))
    even = {v: (m % 2 == 0) for v, m in values}
    xs = np.concatenate([RNG.standard_normal(3000) * 2, RNG.standard_normal(500) * 200, RNG.standard_normal(500) * 0.01,
                         np.array([1.0625, 1.1875, -1.0625, 0.0009765625, 0.0029296875, 464.0, 463.9, 1e6, -1e6, 0.0,
                                   2.0 ** -10, 3 * 2.0 ** -10, 17.0, 19.0])])
    for x in xs:
        got = OPS.round_kv(float(x), FP8)
        d = [abs(v - x) for v in finite]
        best = min(d)
        near = [v for v, dd in zip(finite, d) if dd == best]
        want = near[0] if len(near) == 1 else [v for v in near if even[v]][0]
        assert got == want, (x, got, want)
        assert synth.fp8_bits_to_f32(synth.f32_to_fp8_bits(np.array([x], np.float32)))[0] == OPS.round_kv(float(np.float32(x)), FP8)
    inside = np.array([x for x in xs if abs(x) <= 448.0], np.float32)
    want_t = torch.from_numpy(inside).to(torch.float8_e4m3fn).to(torch.float64).numpy()
    for x, w in zip(inside, want_t):
        assert OPS.round_kv(float(x), FP8) == w, x


# --------------------------------------------------------------------------- operators
@pytest.mark.parametrize("dtype", [F16, BF16])
def test_rmsnorm_vs_torch_and_closed_form(dtype):
    n = 96
    x = RNG.standard_normal(n) * 2.5
    g_bits = synth.to_bits((1 + 0.1 * RNG.standard_normal(n)).astype(np.float32), dtype)
    g = synth.from_bits(g_bits, dtype).astype(np.float64)
    want = torch.nn.functional.rms_norm(torch.from_numpy(x), (n,), torch.from_numpy(g), eps=1e-3).numpy()
    got = OPS.rmsnorm(x, g_bits, dtype, 1e-3)
    assert rel_l2(got, want) < 1e-14
    # constant vector, unit gain: c / sqrt(c^2 + eps) -- eps sits inside the root, added to the mean square
    one = synth.to_bits(np.ones(n, np.float32), dtype)
    c, eps = 0.01, 1e-4
    got = OPS.rmsnorm(np.full(n, c), one, dtype, eps)
    assert np.allclose(got, c / np.sqrt(c * c + eps), rtol=1e-14)


def test_matvec_vs_numpy_nonsquare_with_bias():
    W = synth.to_bits(RNG.standard_normal((37, 50)).astype(np.float32), BF16)
    b = synth.to_bits(RNG.standard_normal(37).astype(np.float32), BF16)
    a = RNG.standard_normal(50)
    want = synth.from_bits(W, BF16).astype(np.float64) @ a + synth.from_bits(b, BF16).astype(np.float64)
    assert rel_l2(OPS.matvec(W, b, BF16, a), want) < 1e-14
    assert rel_l2(OPS.matvec(W, None, BF16, a), want - synth.from_bits(b, BF16)) < 1e-14


def test_rope_invariants_and_closed_forms():
    d, theta = 64, 1e6
    x = RNG.standard_normal(d)
    assert np.array_equal(OPS.rope(x, 0, theta), x)                      # position 0 is the identity
    for pos in (1, 7, 1000, 8191):
        y = OPS.rope(x, pos, theta)
        # each (i, i+d/2) pair is rotated: pair norms (hence the head norm) are preserved
        assert np.allclose(x[: d // 2] ** 2 + x[d // 2:] ** 2, y[: d // 2] ** 2 + y[d // 2:] ** 2, rtol=1e-12)
        # closed form: complex multiplication of (x_i + j x_{i+d/2}) by exp(j pos theta^(-2i/d))
        ang = pos * theta ** (-2.0 * np.arange(d // 2) / d)
        z = (x[: d // 2] + 1j * x[d // 2:]) * np.exp(1j * ang)
        assert np.allclose(y, np.concatenate([z.real, z.imag]), rtol=1e-12, atol=1e-13)
    # d = 2: the unit vector (1, 0) at position p goes to (cos p, sin p): fixes the rotation's sign
    y = OPS.rope(np.array([1.0, 0.0]), 3, theta)
    assert np.allclose(y, [np.cos(3.0), np.sin(3.0)], rtol=1e-14)
    # relative-position property: <R_m q, R_n k> depends on m - n only
    q, k = RNG.standard_normal(d), RNG.standard_normal(d)
    a = OPS.rope(q, 40, theta) @ OPS.rope(k, 25, theta)
    b = OPS.rope(q, 140, theta) @ OPS.rope(k, 125, theta)
    assert abs(a - b) < 1e-10


def test_rope_vs_transformers_rotate_half():
    from transformers.models.qwen2.modeling_qwen2 import apply_rotary_pos_emb
    d, theta, pos = 128, 1e6, 517
    q = RNG.standard_normal(d); k = RNG.standard_normal(d)
    inv = theta ** (-2.0 * np.arange(d // 2) / d)
    ang = torch.from_numpy(np.concatenate([pos * inv, pos * inv]))[None, None, :]
    qt = torch.from_numpy(q)[None, None, None, :]; kt = torch.from_numpy(k)[None, None, None, :]
    qe, ke = apply_rotary_pos_emb(qt, kt, ang.cos(), ang.sin())
    assert rel_l2(OPS.rope(q, pos, theta), qe.numpy().ravel()) < 1e-14
    assert rel_l2(OPS.rope(k, pos, theta), ke.numpy().ravel()) < 1e-14


def test_attend_vs_sdpa_and_closed_forms():
    n, d = 53, 64
    q = RNG.standard_normal(d); K = RNG.standard_normal((n, d)); V = RNG.standard_normal((n, d))
    o, p = OPS.attend(q, K, V)
    want = torch.nn.functional.scaled_dot_product_attention(
        torch.from_numpy(q)[None, None, None], torch.from_numpy(K)[None, None], torch.from_numpy(V)[None, None])
    assert rel_l2(o, want.numpy().ravel()) < 1e-13
    assert abs(p.sum() - 1) < 1e-12 and (p >= 0).all()           # softmax row sums to one
    o1, p1 = OPS.attend(q, K[:1], V[:1])                            # one key: output is that V row
    assert np.allclose(o1, V[0], rtol=1e-15) and p1[0] == 1.0
    Ke = np.tile(K[:1], (n, 1))                                      # equal keys: uniform weights, mean of V
    oe, pe = OPS.attend(q, Ke, V)
    assert np.allclose(pe, 1.0 / n, rtol=1e-12) and np.allclose(oe, V.mean(0), rtol=1e-11, atol=1e-13)
    # large scores must not overflow (max subtraction)
    ob, pb = OPS.attend(q * 1e3, K, V)
    assert np.isfinite(ob).all() and abs(pb.sum() - 1) < 1e-12


def test_swiglu_vs_torch():
    g = RNG.standard_normal(200) * 4; u = RNG.standard_normal(200)
    want = (torch.nn.functional.silu(torch.from_numpy(g)) * torch.from_numpy(u)).numpy()
    assert rel_l2(OPS.swiglu(g, u), want) < 1e-14
    assert OPS.swiglu(np.zeros(3), np.ones(3)).tolist() == [0, 0, 0]


def test_argmax_lowest_index_on_ties():
    x = np.array([0.5, 2.0, -1.0, 2.0, 2.0, 1.0])
    assert OPS.argmax(x) == 1 == int(np.argmax(x))
    y = RNG.standard_normal(1000)
    assert OPS.argmax(y) == int(np.argmax(y))


# --------------------------------------------------------------------------- whole decoder
SMALL = synth.TINY.with_(name="pin-small", vocab=320, hidden=64, n_q_heads=4, n_kv_heads=2, head_dim=16,
                         intermediate=88, max_seq_len=40)
SMALL_BIAS = SMALL.with_(name="pin-small-bias", weight_dtype=BF16, kv_dtype=BF16, qkv_bias=True,
                         tie_embeddings=True, n_q_heads=6, n_kv_heads=2, hidden=96, rope_theta=1e4)


def _hf_logits(shape, w, tokens):
    """Run the transformers library's Qwen2 decoder in fp64 on the same weights (no KV rounding there)."""
    from transformers import Qwen2Config, Qwen2ForCausalLM
    cfg = Qwen2Config(vocab_size=shape.vocab, hidden_size=shape.hidden, intermediate_size=shape.intermediate,
                      num_hidden_layers=len(w["layers"]), num_attention_heads=shape.n_q_heads,
                      num_key_value_heads=shape.n_kv_heads, head_dim=shape.head_dim, rms_norm_eps=shape.rms_eps,
                      rope_theta=shape.rope_theta, max_position_embeddings=shape.max_seq_len,
                      tie_word_embeddings=shape.tie_embeddings, attn_implementation="eager",
                      use_sliding_window=False)
    cfg.rope_parameters = {"rope_type": "default", "rope_theta": shape.rope_theta}
    m = Qwen2ForCausalLM(cfg).double().eval()
    up = lambda b: torch.from_numpy(synth.from_bits(b, shape.weight_dtype).astype(np.float64))
    qd, kvd, I = shape.q_dim, shape.kv_dim, shape.intermediate
    sd = {"model.embed_tokens.weight": up(w["embed"]), "model.norm.weight": up(w["final_norm"])}
    sd["lm_head.weight"] = sd["model.embed_tokens.weight"] if shape.tie_embeddings else up(w["lm_head"])
    for l, lw in enumerate(w["layers"]):
        p = f"model.layers.{l}."
        W = up(lw["wqkv"])
        b = up(lw["bqkv"]) if lw["bqkv"] is not None else torch.zeros(shape.qkv_rows, dtype=torch.float64)
        for nm, lo, hi in (("q", 0, qd), ("k", qd, qd + kvd), ("v", qd + kvd, qd + 2 * kvd)):
            sd[p + f"self_attn.{nm}_proj.weight"] = W[lo:hi]
            sd[p + f"self_attn.{nm}_proj.bias"] = b[lo:hi]
        sd[p + "self_attn.o_proj.weight"] = up(lw["wo"])
        sd[p + "input_layernorm.weight"] = up(lw["attn_norm"])
        sd[p + "post_attention_layernorm.weight"] = up(lw["mlp_norm"])
        gu = up(lw["w_gate_up"])
        sd[p + "mlp.gate_proj.weight"] = gu[:I]
        sd[p + "mlp.up_proj.weight"] = gu[I:]
        sd[p + "mlp.down_proj.weight"] = up(lw["w_down"])
    missing, unexpected = m.load_state_dict(sd, strict=False)
    assert not unexpected and all("rotary" in k or k == "lm_head.weight" for k in missing), (missing, unexpected)
    with torch.no_grad():
        out = m(torch.from_numpy(np.asarray(tokens, dtype=np.int64))[None])
    return out.logits[0].numpy()


@pytest.mark.parametrize("shape", [SMALL, SMALL_BIAS], ids=lambda s: s.name)
def test_forward_vs_transformers_qwen2_fp64(shape):
    w = synth.make_weights(shape, seed=11)
    tokens = synth.make_prompt(shape, 24, seed=5)
    want = _hf_logits(shape, w, tokens)
    m = oracle.OracleModel(shape, w, kv_round=False)
    r1 = m.prefill(tokens[:17], logits="all")
    got = [r1["logits"]]
    for t in tokens[17:]:
        got.append(m.decode_step(int(t))["logits"][None])
    got = np.concatenate(got, 0)
    assert got.shape == want.shape
    # the library builds its rotary cos/sin table in fp32 even when the model is cast to fp64, which
    # limits the agreement to ~1e-7; any structural mistake (pairing, head map, eps, order) is >= 1e-3
    assert rel_l2(got, want) < 1e-6
    assert (got.argmax(1) == want.argmax(1)).all()


def _brute_force(shape, w, tokens, round_kv=True):
    """Independent full-sequence evaluation: float64 numpy, materialised T x T score matrix with an explicit
    causal mask, KV heads expanded with np.repeat (plain multi-head attention), cache rounding through
    the library casts."""
    wd, kd = shape.weight_dtype, shape.kv_dtype
    up = lambda b: synth.from_bits(b, wd).astype(np.float64)
    T, H, d, nq, nkv = len(tokens), shape.hidden, shape.head_dim, shape.n_q_heads, shape.n_kv_heads
    X = up(w["embed"])[tokens]

    def norm(X, g):
        return X / np.sqrt((X * X).mean(-1, keepdims=True) + shape.rms_eps) * up(g)

    def rnd(A):
        if not round_kv:
            return A
        if kd == BF16:
            # torch casts double -> bf16 through fp32; that double rounding can flip a value that sits within
            # 2^-29 relative of a bf16 tie (probability ~1e-6 per element), which the tolerance below absorbs
            return torch.from_numpy(A).to(torch.bfloat16).to(torch.float64).numpy()
        return A.astype(np.float16).astype(np.float64)  # numpy rounds double -> half directly

    pos = np.arange(T)[:, None]
    ang = pos * shape.rope_theta ** (-2.0 * np.arange(d // 2) / d)[None, :]
    cos = np.cos(np.concatenate([ang, ang], -1))[:, None, :]
    sin = np.sin(np.concatenate([ang, ang], -1))[:, None, :]
    rot = lambda A: np.concatenate([-A[..., d // 2:], A[..., : d // 2]], -1)
    mask = np.tril(np.ones((T, T), bool))
    for lw in w["layers"]:
        A = norm(X, lw["attn_norm"])
        QKV = A @ up(lw["wqkv"]).T
        if lw["bqkv"] is not None:
            QKV = QKV + up(lw["bqkv"])
        Q = QKV[:, : nq * d].reshape(T, nq, d)
        K = QKV[:, nq * d: (nq + nkv) * d].reshape(T, nkv, d)
        V = QKV[:, (nq + nkv) * d:].reshape(T, nkv, d)
        Q = Q * cos + rot(Q) * sin
        K = rnd(K * cos + rot(K) * sin)
        V = rnd(V)
        K = np.repeat(K, nq // nkv, axis=1); V = np.repeat(V, nq // nkv, axis=1)
        S = np.einsum("thd,shd->hts", Q, K) / np.sqrt(d)
        S = np.where(mask[None], S, -np.inf)
        P = np.exp(S - S.max(-1, keepdims=True)); P /= P.sum(-1, keepdims=True)
        O = np.einsum("hts,shd->thd", P, V).reshape(T, nq * d)
        X = X + O @ up(lw["wo"]).T
        B = norm(X, lw["mlp_norm"])
        GU = B @ up(lw["w_gate_up"]).T
        G, U = GU[:, : shape.intermediate], GU[:, shape.intermediate:]
        X = X + (G / (1 + np.exp(-G)) * U) @ up(lw["w_down"]).T
    F = norm(X, w["final_norm"])
    lm = w["embed"] if shape.tie_embeddings else w["lm_head"]
    return F, F @ up(lm).T


@pytest.mark.parametrize("shape", [synth.TINY, SMALL_BIAS], ids=lambda s: s.name)
def test_forward_with_rounded_cache_vs_numpy_brute_force(shape):
    w = synth.make_weights(shape, seed=21)
    tokens = synth.make_prompt(shape, 36 if shape is SMALL_BIAS else 48, seed=6)
    m = oracle.OracleModel(shape, w, kv_round=True)
    r = m.prefill(tokens, logits="all")
    F, LG = _brute_force(shape, w, tokens, round_kv=True)
    assert rel_l2(r["hidden"], F) < 1e-5 and rel_l2(r["logits"], LG) < 1e-5
    # and the rounding is really applied: the unrounded evaluation differs measurably
    F0, _ = _brute_force(shape, w, tokens, round_kv=False)
    assert rel_l2(r["hidden"], F0) > 20 * rel_l2(r["hidden"], F)
    # cache contents are exactly representable in the cache dtype
    k, v = m.kv_read(1, 5)
    assert np.array_equal(synth.from_bits(synth.to_bits(k.astype(np.float32), shape.kv_dtype), shape.kv_dtype), k)
    assert np.array_equal(synth.from_bits(synth.to_bits(v.astype(np.float32), shape.kv_dtype), shape.kv_dtype), v)


@pytest.mark.parametrize("shape", [synth.TINY, SMALL_BIAS], ids=lambda s: s.name)
def test_prefill_then_decode_equals_full_prefill(shape):
    """Eq. 3-4: the KV cache is exact -- any split of the sequence into blocks gives the same result."""
    w = synth.make_weights(shape, seed=31)
    n = 30
    tokens = synth.make_prompt(shape, n, seed=7)
    full = oracle.OracleModel(shape, w).prefill(tokens, logits="all")
    m = oracle.OracleModel(shape, w)
    hs = [m.prefill(tokens[:9], logits="all")]
    hs.append(m.prefill(tokens[9:14], logits="all"))  # appended block
    for t in tokens[14:]:
        hs.append(m.decode_step(int(t), logits="all"))
    H = np.concatenate([h["hidden"] for h in hs]); LG = np.concatenate([h["logits"] for h in hs])
    assert m.kv_len == n
    assert rel_l2(H, full["hidden"]) < 1e-13 and rel_l2(LG, full["logits"]) < 1e-13


def test_zero_output_projections_reduce_to_lm_head_of_embedding():
    shape = SMALL
    w = synth.make_weights(shape, seed=41)
    for lw in w["layers"]:
        lw["wo"] = np.zeros_like(lw["wo"]); lw["w_down"] = np.zeros_like(lw["w_down"])
    tokens = synth.make_prompt(shape, 6, seed=8)
    r = oracle.OracleModel(shape, w).prefill(tokens, logits="all")
    E = synth.from_bits(w["embed"], shape.weight_dtype).astype(np.float64)
    g = synth.from_bits(w["final_norm"], shape.weight_dtype).astype(np.float64)
    x = E[tokens]
    f = torch.nn.functional.rms_norm(torch.from_numpy(x), (shape.hidden,), torch.from_numpy(g), eps=shape.rms_eps).numpy()
    lm = synth.from_bits(w["lm_head"], shape.weight_dtype).astype(np.float64)
    assert rel_l2(r["hidden"], f) < 1e-14 and rel_l2(r["logits"], f @ lm.T) < 1e-14


def test_symmetries_neuron_and_kv_group_permutations():
    shape = SMALL_BIAS
    w = synth.make_weights(shape, seed=51)
    tokens = synth.make_prompt(shape, 12, seed=9)
    base = oracle.OracleModel(shape, w).prefill(tokens, logits="all")
    I, d, nq, nkv = shape.intermediate, shape.head_dim, shape.n_q_heads, shape.n_kv_heads
    g = nq // nkv
    perm = RNG.permutation(I)
    grp = np.arange(nkv)[::-1]
    qrows = np.concatenate([np.arange(h * g * d, (h + 1) * g * d) for h in grp])
    krows = nq * d + np.concatenate([np.arange(h * d, (h + 1) * d) for h in grp])
    vrows = krows + nkv * d
    rows = np.concatenate([qrows, krows, vrows])
    w2 = {**w, "layers": []}
    for lw in w["layers"]:
        w2["layers"].append({**lw,
                             "w_gate_up": np.ascontiguousarray(np.concatenate([lw["w_gate_up"][:I][perm], lw["w_gate_up"][I:][perm]])),
                             "w_down": np.ascontiguousarray(lw["w_down"][:, perm]),
                             "wqkv": np.ascontiguousarray(lw["wqkv"][rows]),
                             "bqkv": np.ascontiguousarray(lw["bqkv"][rows]),
                             "wo": np.ascontiguousarray(lw["wo"][:, qrows])})
    got = oracle.OracleModel(shape, w2).prefill(tokens, logits="all")
    assert rel_l2(got["logits"], base["logits"]) < 1e-12


def test_embedding_rows_input_equals_token_input_and_positions_follow():
    shape = SMALL
    w = synth.make_weights(shape, seed=61)
    tokens = synth.make_prompt(shape, 10, seed=10)
    a = oracle.OracleModel(shape, w).prefill(tokens, logits="all")
    emb = np.ascontiguousarray(w["embed"][tokens[:6]])
    b = oracle.OracleModel(shape, w).prefill(tokens[6:], embeds=emb, logits="all")
    assert np.array_equal(a["logits"], b["logits"])


def test_kv_reset_keeps_prefix_and_replays_suffix():
    """Section 3.9 / Eq. 5: KV = Concat(KV_p, KV_u) -- after recycling the slot to the prefix length
    only the suffix has to be evaluated again."""
    shape = SMALL
    w = synth.make_weights(shape, seed=71)
    tokens = synth.make_prompt(shape, 20, seed=11)
    m = oracle.OracleModel(shape, w)
    m.prefill(tokens[:12], logits="none")
    first = m.prefill(tokens[12:], logits="all")
    m.kv_reset(12)
    assert m.kv_len == 12
    again = m.prefill(tokens[12:], logits="all")
    assert np.array_equal(first["logits"], again["logits"])
    m.kv_reset(0)
    full = m.prefill(tokens, logits="all")
    assert np.array_equal(full["logits"][12:], first["logits"])
    with pytest.raises(ValueError):
        m.kv_reset(21)


def test_error_codes():
    shape = SMALL
    w = synth.make_weights(shape, seed=81)
    m = oracle.OracleModel(shape, w)
    with pytest.raises(ValueError, match="overflow"):
        m.prefill(np.zeros(shape.max_seq_len + 1, np.int32))
    with pytest.raises(ValueError, match="token"):
        m.prefill(np.array([shape.vocab], np.int32))
    with pytest.raises(ValueError, match="token"):
        m.prefill(np.array([-1], np.int32))
    assert m.kv_len == 0


def test_kv_injection_roundtrip_and_attention_over_injected_rows():
    shape = SMALL
    w = synth.make_weights(shape, seed=91)
    m = oracle.OracleModel(shape, w)
    rows = [synth.make_kv_rows(shape, l, 17) for l in range(shape.n_layers)]
    m.kv_inject(rows)
    assert m.kv_len == 17
    k, v = m.kv_read(1, 16)
    assert np.array_equal(k, synth.from_bits(rows[1][0][16], shape.kv_dtype))
    assert np.array_equal(v, synth.from_bits(rows[1][1][16], shape.kv_dtype))
    r = m.decode_step(3)
    assert m.kv_len == 18 and np.isfinite(r["logits"]).all()


def test_fp32_build_of_same_source_is_close():
    """How much does evaluation precision matter?  The fp32 build of the oracle source must agree with the
    fp64 oracle far inside the 2e-3 parity tolerance."""
    shape = synth.TINY
    w = synth.make_weights(shape)
    tokens = synth.make_prompt(shape, 32)
    a = oracle.OracleModel(shape, w, kind="f64").prefill(tokens, logits="all")
    b = oracle.OracleModel(shape, w, kind="f32").prefill(tokens, logits="all")
    assert rel_l2(b["hidden"], a["hidden"]) < 2e-5 and rel_l2(b["logits"], a["logits"]) < 2e-5


def test_restricted_argmax_is_the_brute_force_choice():
    """Vocabulary pruning as the library documents it: the argmax over the candidate ids, lowest id on ties.
    Pinned against numpy on random logits and on planted ties."""
    rng = np.random.default_rng(5)
    for trial in range(50):
        V = int(rng.integers(5, 400))
        logits = rng.standard_normal(V).astype(np.float32)
        n = int(rng.integers(1, V + 1))
        subset = np.sort(rng.choice(V, size=n, replace=False))
        if trial % 3 == 0 and n >= 2:  # plant a tie at the maximum between two candidates
            a, b = rng.choice(n, size=2, replace=False)
            logits[subset[a]] = logits[subset[b]] = logits.max() + 1.0
        tok, cand = oracle.restricted_argmax(logits, subset)
        np.testing.assert_array_equal(cand, logits[subset])
        assert tok == int(subset[int(np.argmax(logits[subset]))])  # numpy's argmax also takes the first maximum
        assert tok in subset and logits[tok] == logits[subset].max()
    full = np.arange(17)
    lg = rng.standard_normal(17)
    assert oracle.restricted_argmax(lg, full)[0] == int(np.argmax(lg))
