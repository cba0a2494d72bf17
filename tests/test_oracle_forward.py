"""Pins for the checker's forward pass: closed forms, a library Llama
implementation, a loop-level brute force, and structural properties
(causality, prefix purity, KV overwrite, stream invariance of the
decode-verify-rollback loop; paper Sections 3, 4.1, 4.2)."""
import math

import numpy as np
import pytest
import torch

from helpers import orc, wl, oracle_cfg, randomize_gains, oracle_prefill, oracle_greedy_decode

F64 = torch.float64


# ---------------------------------------------------------------- scalars ----
def test_bf16_round_matches_library_and_ties_to_even():
    g = torch.Generator().manual_seed(0)
    x = torch.randn(100000, generator=g, dtype=torch.float32) * 3
    assert torch.equal(orc.bf16_round(x), x.to(torch.bfloat16).to(torch.float32))
    # 1 + 2^-8 lies exactly between bf16(1) and bf16(1 + 2^-7): ties go to the even mantissa (1.0);
    # 1 + 3*2^-8 lies between 1+2^-7 (odd) and 1+2^-6 (even) -> 1 + 2^-6
    t = torch.tensor([1 + 2.0 ** -8, 1 + 3 * 2.0 ** -8, -(1 + 2.0 ** -8), 1 + 2.0 ** -8 + 2.0 ** -20], dtype=F64)
    assert orc.bf16_round(t).tolist() == [1.0, 1 + 2.0 ** -6, -1.0, 1 + 2.0 ** -7]
    assert orc.bf16_round(t).dtype == F64


def test_rmsnorm_constant_vector_closed_form():
    d, c, eps = 64, -3.0, 1e-5
    gain = torch.linspace(0.5, 2.0, d, dtype=F64)
    y = orc.rmsnorm(torch.full((2, d), c, dtype=F64), gain, eps)
    expect = -gain / math.sqrt(1 + eps / c ** 2)
    assert torch.allclose(y[0], expect, rtol=1e-14, atol=0)
    # scale invariance up to eps: rmsnorm(a x) = rmsnorm(x) for eps -> 0
    x = torch.randn(3, d, dtype=F64)
    assert torch.allclose(orc.rmsnorm(5 * x, gain, 0.0), orc.rmsnorm(x, gain, 0.0), rtol=1e-13)
    # unit mean square of y / gain
    z = orc.rmsnorm(x, torch.ones(d, dtype=F64), 0.0)
    assert torch.allclose((z * z).mean(-1), torch.ones(3, dtype=F64), rtol=1e-13)


def test_rope_closed_forms():
    hd, theta = 8, 1e4
    x = torch.randn(5, 3, hd, dtype=F64)
    pos = torch.tensor([0, 1, 2, 7, 100])
    cos, sin = orc.rope_angles(pos, hd, theta, F64)
    y = orc.apply_rope(x, cos, sin)
    assert torch.equal(y[0], x[0])                                   # position 0: identity
    assert torch.allclose(y.norm(dim=-1), x.norm(dim=-1), rtol=1e-13)  # a rotation
    # pair (j, j + hd/2) turns by pos * theta^(-2j/hd): check pair j = 1 at pos 7 by hand
    a = 7 * theta ** (-2 * 1 / hd)
    assert math.isclose(y[3, 0, 1], x[3, 0, 1] * math.cos(a) - x[3, 0, 5] * math.sin(a), rel_tol=1e-12)
    assert math.isclose(y[3, 0, 5], x[3, 0, 5] * math.cos(a) + x[3, 0, 1] * math.sin(a), rel_tol=1e-12)
    # j = 0 has frequency 1: angle = position
    assert math.isclose(cos[4, 0], math.cos(100.0), rel_tol=1e-12)
    # relative-position property: <rope(q, m), rope(k, n)> depends on m - n only
    q, k = torch.randn(1, 1, hd, dtype=F64), torch.randn(1, 1, hd, dtype=F64)

    def dot(m, n):
        cm, sm = orc.rope_angles(torch.tensor([m]), hd, theta, F64)
        cn, sn = orc.rope_angles(torch.tensor([n]), hd, theta, F64)
        return float((orc.apply_rope(q, cm, sm) * orc.apply_rope(k, cn, sn)).sum())
    assert math.isclose(dot(9, 4), dot(105, 100), rel_tol=1e-10)
    assert not math.isclose(dot(9, 4), dot(9, 5), rel_tol=1e-3)


def test_silu_closed_forms():
    z = torch.tensor([0.0, 1.0, -1.0, 40.0, -40.0], dtype=F64)
    s = orc.silu(z)
    assert s[0] == 0.0
    assert math.isclose(s[1], 1 / (1 + math.exp(-1)), rel_tol=1e-15)      # 0.7310585786...
    assert math.isclose(s[2], -1 / (1 + math.exp(1)), rel_tol=1e-15)
    assert math.isclose(s[3], 40.0, rel_tol=1e-15) and abs(s[4]) < 1e-15


# ------------------------------------------------------- library Llama ------
def _hf_model(shape, w):
    from transformers import LlamaConfig, LlamaForCausalLM
    cfg = LlamaConfig(vocab_size=shape.vocab, hidden_size=shape.d_model, intermediate_size=shape.d_ffn,
                      num_hidden_layers=shape.n_layers, num_attention_heads=shape.n_q_heads,
                      num_key_value_heads=shape.n_kv_heads, head_dim=shape.head_dim, hidden_act="silu",
                      max_position_embeddings=512, rms_norm_eps=shape.rms_eps, rope_theta=shape.rope_theta,
                      attention_bias=False, mlp_bias=False, tie_word_embeddings=False,
                      attn_implementation="eager")
    m = LlamaForCausalLM(cfg).double().eval()
    sd = {"model.embed_tokens.weight": w["embed"], "model.norm.weight": w["final_norm"],
          "lm_head.weight": w["lm_head"]}
    names = {"attn_norm": "input_layernorm", "ffn_norm": "post_attention_layernorm",
             "wq": "self_attn.q_proj", "wk": "self_attn.k_proj", "wv": "self_attn.v_proj",
             "wo": "self_attn.o_proj", "w_gate": "mlp.gate_proj", "w_up": "mlp.up_proj",
             "w_down": "mlp.down_proj"}
    for li, lw in enumerate(w["layers"]):
        for k, v in lw.items():
            sd[f"model.layers.{li}.{names[k]}.weight"] = v
    m.load_state_dict({k: v.to(F64) for k, v in sd.items()}, strict=True)
    return m


def test_forward_matches_library_llama_fp64():
    """round_points off: the checker is the textbook real-number forward and must
    agree with an independent library implementation of the same architecture,
    both for a full pass and for a window replayed on top of a cached prefix."""
    shape = wl.TINY
    w = randomize_gains(wl.make_weights(shape, seed=42, std=0.08))   # larger std: sharper softmax
    cfg = oracle_cfg(shape)
    ids = wl.random_tokens(wl.rng_for(3), 29, shape.vocab)
    with torch.no_grad():
        ref = _hf_model(shape, w)(torch.tensor(ids[None].astype(np.int64))).logits[0]
    kv = orc.OracleKV(cfg, 64)
    full = orc.forward_window(cfg, w, kv, 0, ids, round_points=False)
    # the library evaluates its rotary cos/sin in float32 whatever the model dtype, which
    # bounds the agreement near 1e-6; any structural mistake shows at the 1e-1 level
    assert torch.allclose(full, ref, rtol=0, atol=2e-5), float((full - ref).abs().max())
    kv2 = orc.OracleKV(cfg, 64)
    orc.forward_window(cfg, w, kv2, 0, ids[:21], round_points=False)
    tail = orc.forward_window(cfg, w, kv2, 21, ids[21:], round_points=False)
    assert torch.allclose(tail, ref[21:], rtol=0, atol=2e-5)
    assert ref.abs().max() > 0.5          # the comparison is not between zeros


# ------------------------------------------------------- brute force --------
def _bf16_np(x):
    """Independent bf16 rounding (numpy integer arithmetic on the float32 bits)."""
    b = np.asarray(x, dtype=np.float32).view(np.uint32).astype(np.uint64)
    b = (b + 0x7FFF + ((b >> 16) & 1)) & 0xFFFF0000
    return b.astype(np.uint32).view(np.float32).astype(np.float64)


def _brute_force_logits(shape, w, ids, rnd, round_p=False):
    """Scalar-loop forward without any cache: every row recomputes attention over
    the whole token list.  Written separately from the checker on purpose."""
    R = _bf16_np if rnd else (lambda a: np.asarray(a, dtype=np.float64))
    f = lambda t: t.to(torch.float64).numpy()
    H, G, hd, d = shape.n_q_heads, shape.n_kv_heads, shape.head_dim, shape.d_model
    n = len(ids)
    x = np.stack([f(w["embed"][int(t)]) for t in ids])

    def norm(v, g):
        out = np.empty_like(v)
        for i in range(v.shape[0]):
            ms = sum(float(a) * float(a) for a in v[i]) / d
            out[i] = v[i] / math.sqrt(ms + shape.rms_eps) * g
        return out

    def rope(vec, p):
        out = np.empty_like(vec)
        for j in range(hd // 2):
            a = p * shape.rope_theta ** (-2.0 * j / hd)
            out[j] = vec[j] * math.cos(a) - vec[j + hd // 2] * math.sin(a)
            out[j + hd // 2] = vec[j + hd // 2] * math.cos(a) + vec[j] * math.sin(a)
        return out

    for lw in w["layers"]:
        y = R(norm(x, f(lw["attn_norm"])))
        q = y @ f(lw["wq"]).T
        k = y @ f(lw["wk"]).T
        v = R(y @ f(lw["wv"]).T)
        qr = np.empty_like(q)
        kr = np.empty_like(k)
        for i in range(n):
            for h in range(H):
                qr[i, h * hd:(h + 1) * hd] = rope(q[i, h * hd:(h + 1) * hd], i)
            for g in range(G):
                kr[i, g * hd:(g + 1) * hd] = rope(k[i, g * hd:(g + 1) * hd], i)
        qr, kr = R(qr), R(kr)
        att = np.zeros((n, H * hd))
        for i in range(n):
            for h in range(H):
                g = h // (H // G)
                sc = [float(qr[i, h * hd:(h + 1) * hd] @ kr[t, g * hd:(g + 1) * hd]) / math.sqrt(hd)
                      for t in range(i + 1)]
                mx = max(sc)
                e = [math.exp(s - mx) for s in sc]
                z = sum(e)
                for t in range(i + 1):
                    if round_p:     # rounded weight in the numerator, unrounded weights in the denominator
                        att[i, h * hd:(h + 1) * hd] += float(_bf16_np(e[t])) * v[t, g * hd:(g + 1) * hd] / z
                    else:
                        att[i, h * hd:(h + 1) * hd] += e[t] / z * v[t, g * hd:(g + 1) * hd]
        x = x + R(att) @ f(lw["wo"]).T
        y = R(norm(x, f(lw["ffn_norm"])))
        ga, up = y @ f(lw["w_gate"]).T, y @ f(lw["w_up"]).T
        hdn = R(ga / (1 + np.exp(-ga)) * up)
        x = x + hdn @ f(lw["w_down"]).T
    return R(norm(x, f(w["final_norm"]))) @ f(w["lm_head"]).T


@pytest.mark.parametrize("rnd", [False, True])
def test_forward_matches_scalar_brute_force(rnd):
    shape = wl.ModelShape(n_layers=2, d_model=32, n_q_heads=4, n_kv_heads=2, head_dim=8, d_ffn=48,
                          vocab=64, rope_theta=100.0)
    w = randomize_gains(wl.make_weights(shape, seed=5, std=0.3))
    ids = wl.random_tokens(wl.rng_for(6), 11, shape.vocab)
    cfg = oracle_cfg(shape)
    kv = orc.OracleKV(cfg, 16)
    orc.forward_window(cfg, w, kv, 0, ids[:6], round_points=rnd)
    got = orc.forward_window(cfg, w, kv, 6, ids[6:], round_points=rnd).numpy()
    ref = _brute_force_logits(shape, w, ids, rnd)[6:]
    # with rounding on, a last-bit difference before a rounding point can flip one bf16 ulp
    tol = 2e-2 if rnd else 1e-11
    assert np.abs(got - ref).max() < tol * max(1.0, np.abs(ref).max()), np.abs(got - ref).max()
    if rnd:
        # such flips are rare: the bulk must agree to fp64 accuracy
        assert np.median(np.abs(got - ref)) < 1e-9


def test_softmax_weight_rounding_option_matches_scalar_brute_force():
    """round_p: exp(s - max) rounded to bf16 where it multiplies V, the denominator from the unrounded weights.
    With every other rounding point off the two implementations must agree to fp64 accuracy, and the option
    must move the result by about one bf16 rounding of the attention output, no more."""
    shape = wl.ModelShape(n_layers=2, d_model=32, n_q_heads=4, n_kv_heads=2, head_dim=8, d_ffn=48,
                          vocab=64, rope_theta=100.0)
    w = randomize_gains(wl.make_weights(shape, seed=5, std=0.3))
    ids = wl.random_tokens(wl.rng_for(6), 11, shape.vocab)
    cfg = oracle_cfg(shape)
    kv = orc.OracleKV(cfg, 16)
    orc.forward_window(cfg, w, kv, 0, ids[:6], round_points=False, round_p=True)
    got = orc.forward_window(cfg, w, kv, 6, ids[6:], round_points=False, round_p=True).numpy()
    ref = _brute_force_logits(shape, w, ids, False, round_p=True)[6:]
    plain = _brute_force_logits(shape, w, ids, False)[6:]
    scale = max(1.0, np.abs(ref).max())
    assert np.abs(got - ref).max() < 1e-11 * scale
    moved = np.abs(ref - plain).max() / scale
    assert 1e-6 < moved < 2.0 ** -7, moved
    # a softmax over one key has weight exactly 1: nothing to round, the option changes nothing
    kv1 = orc.OracleKV(cfg, 4)
    a = orc.forward_window(cfg, w, kv1, 0, ids[:1], round_p=True)
    b = orc.forward_window(cfg, w, orc.OracleKV(cfg, 4), 0, ids[:1], round_p=False)
    assert torch.equal(a, b)


# ------------------------------------------------------- structure ----------
@pytest.fixture(scope="module")
def tiny():
    shape = wl.TINY
    w = randomize_gains(wl.make_weights(shape, seed=42))
    return shape, oracle_cfg(shape), w


def test_row_by_row_equals_batched(tiny):
    shape, cfg, w = tiny
    ids = wl.random_tokens(wl.rng_for(11), 24, shape.vocab)
    kv_a, kv_b = orc.OracleKV(cfg, 32), orc.OracleKV(cfg, 32)
    a = orc.forward_window(cfg, w, kv_a, 0, ids)
    b = torch.cat([orc.forward_window(cfg, w, kv_b, i, ids[i:i + 1]) for i in range(len(ids))])
    assert torch.allclose(a, b, rtol=0, atol=1e-9)
    assert torch.equal(orc.greedy_argmax(a), orc.greedy_argmax(b))
    assert torch.equal(kv_a.k, kv_b.k) and torch.equal(kv_a.v, kv_b.v)


def test_prefix_purity_and_causality(tiny):
    """Logits at a position depend on the tokens up to it only: not on how the
    positions were cut into windows and not on later inputs."""
    shape, cfg, w = tiny
    ids = wl.random_tokens(wl.rng_for(12), 30, shape.vocab)
    kv = orc.OracleKV(cfg, 32)
    orc.forward_window(cfg, w, kv, 0, ids[:14])
    one = orc.forward_window(cfg, w, kv, 14, ids[14:30])
    kv2 = orc.OracleKV(cfg, 32)
    orc.forward_window(cfg, w, kv2, 0, ids[:9])
    orc.forward_window(cfg, w, kv2, 9, ids[9:14])
    two = torch.cat([orc.forward_window(cfg, w, kv2, 14, ids[14:19]),
                     orc.forward_window(cfg, w, kv2, 19, ids[19:30])])
    assert torch.allclose(one, two, rtol=0, atol=1e-9)
    changed = ids.copy()
    changed[22:] = (changed[22:] + 1) % shape.vocab
    kv3 = orc.OracleKV(cfg, 32)
    orc.forward_window(cfg, w, kv3, 0, ids[:14])
    other = orc.forward_window(cfg, w, kv3, 14, changed[14:30])
    assert torch.equal(other[:8], one[:8])           # rows 14..21 see no changed input
    assert not torch.allclose(other[8:], one[8:], atol=1e-3)


def test_window_kv_is_overwritten_and_the_rest_untouched(tiny):
    shape, cfg, w = tiny
    ids = wl.random_tokens(wl.rng_for(13), 20, shape.vocab)
    kv = orc.OracleKV(cfg, 32)
    orc.forward_window(cfg, w, kv, 0, ids[:12])
    clean = orc.forward_window(cfg, w, kv, 12, ids[12:20])
    k_clean = kv.k.clone()
    kv.k[:, 12:] = 777.0          # stale fast-path entries and never-written slots
    kv.v[:, 12:] = -777.0
    again = orc.forward_window(cfg, w, kv, 12, ids[12:20])
    assert torch.equal(again, clean)
    assert torch.equal(kv.k[:, :20], k_clean[:, :20])
    assert bool((kv.k[:, 20:] == 777.0).all()) and bool((kv.v[:, 20:] == -777.0).all())
    # stored K/V are bf16 values
    assert torch.equal(orc.bf16_round(kv.k[:, :20]), kv.k[:, :20])


def test_fp32_accumulation_mode_is_close(tiny):
    shape, cfg, w = tiny
    ids = wl.random_tokens(wl.rng_for(14), 24, shape.vocab)
    a = orc.forward_window(cfg, w, orc.OracleKV(cfg, 32), 0, ids)
    b = orc.forward_window(cfg, w, orc.OracleKV(cfg, 32), 0, ids, acc_dtype=torch.float32)
    assert b.dtype == torch.float32
    assert float((a - b.double()).abs().max()) < 5e-3


# ------------------------------------------------------- the DVR loop -------
def _dvr_stream(cfg, w, shape, prompt, total, window, rate, seed):
    """Decode-verify-rollback with a simulated fast path: candidates are the true
    greedy continuation with a fraction replaced at random (Section 4.2)."""
    kv = orc.OracleKV(cfg, len(prompt) + total + window + 1)
    last = oracle_prefill(cfg, w, kv, prompt)
    L, stream, passes = len(prompt), [last], 0
    rng = wl.rng_for(seed)
    while len(stream) < total:
        scratch = orc.OracleKV(cfg, kv.capacity)
        scratch.k[:, :L] = kv.k[:, :L]
        scratch.v[:, :L] = kv.v[:, :L]
        chain = oracle_greedy_decode(cfg, w, scratch, L, last, window - 1)
        inputs = wl.replace_candidates(rng, np.array([last] + chain), rate, shape.vocab)
        outs, _ = orc.verify_window(cfg, w, [kv], [L], [inputs])
        committed, toks, rolled = orc.commit_rollback(inputs, outs[0], window)
        assert 1 <= committed <= window and committed + rolled == window
        stream += toks
        L += committed
        last = toks[-1]
        passes += 1
    return stream[:total], passes


def test_dvr_stream_is_invariant_to_the_fast_path(tiny):
    """The paper's claim: whatever the fast path proposes, the released stream is
    the one plain greedy decoding from the consistent state produces."""
    shape, cfg, w = tiny
    prompt = wl.random_tokens(wl.rng_for(15), 19, shape.vocab)
    total, window = 25, 8
    kv = orc.OracleKV(cfg, 64)
    first = oracle_prefill(cfg, w, kv, prompt)
    plain = [first] + oracle_greedy_decode(cfg, w, kv, len(prompt), first, total - 1)
    s0, p0 = _dvr_stream(cfg, w, shape, prompt, total, window, 0.0, 1)
    s1, p1 = _dvr_stream(cfg, w, shape, prompt, total, window, 0.1, 2)
    s5, p5 = _dvr_stream(cfg, w, shape, prompt, total, window, 0.5, 3)
    assert s0 == plain and s1 == plain and s5 == plain
    assert p0 == 3                      # 24 new tokens at 8 per pass: no rollbacks
    assert p5 > p0                      # rollbacks cost extra passes, not correctness


def test_replacement_at_j_commits_exactly_j(tiny):
    shape, cfg, w = tiny
    prompt = wl.random_tokens(wl.rng_for(16), 17, shape.vocab)
    window = 8
    kv = orc.OracleKV(cfg, 64)
    last = oracle_prefill(cfg, w, kv, prompt)
    chain = oracle_greedy_decode(cfg, w, kv, len(prompt), last, window - 1)
    base = [last] + chain
    outs, _ = orc.verify_window(cfg, w, [kv], [len(prompt)], [base])
    assert orc.commit_rollback(base, outs[0], window)[0] == window
    for j in range(1, window):
        bad = list(base)
        bad[j] = (bad[j] + 1) % shape.vocab
        outs, _ = orc.verify_window(cfg, w, [kv], [len(prompt)], [bad])
        committed, toks, _ = orc.commit_rollback(bad, outs[0], window)
        assert committed == j and toks == base[1:j] + [chain[j - 1]]
