"""Pins of the model oracle against things other than itself: closed forms, invariants,
library routines (torch CPU, fp64) and an independent library implementation of the
same decoder family (transformers' LLaMA model in fp64 with the same weights)."""
import math

import numpy as np
import pytest
import torch

from paper_2305_13144_amd import synth
from oracle.model_oracle import Components, OracleModel


@pytest.fixture(scope="module")
def comp(oracle_built):
    return Components("f64")


def _bits(x):
    return synth.f32_to_bf16_bits(np.asarray(x, np.float32))


def _wide(b):
    return synth.bf16_bits_to_f32(b).astype(np.float64)


# ------------------------------------------------------------------ bf16 helper (generator side)
def test_bf16_rounding_matches_torch():
    rng = np.random.default_rng(0)
    x = (rng.standard_normal(10000) * 0.02).astype(np.float32)
    ours = synth.f32_to_bf16_bits(x)
    ref = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(ours, ref)
    # ties go to even: 1 + 2^-8 is exactly half way between 1 and 1 + 2^-7
    assert synth.f32_to_bf16_bits(np.array([1.0 + 2.0 ** -8], np.float32))[0] == 0x3F80
    assert synth.f32_to_bf16_bits(np.array([1.0 + 3 * 2.0 ** -8], np.float32))[0] == 0x3F82


# ------------------------------------------------------------------ RMSNorm
def test_rmsnorm_constant_vector_closed_form(comp):
    d, c, eps = 64, 3.0, 1e-6
    w = _bits(np.full(d, 0.5))
    out = comp.rmsnorm(np.full(d, c), w, eps)
    assert np.allclose(out, 0.5 * c / math.sqrt(c * c + float(np.float32(eps))), rtol=1e-13)


def test_rmsnorm_vs_torch(comp):
    rng = np.random.default_rng(1)
    x = rng.standard_normal(256)
    wb = _bits(1.0 + 0.1 * rng.standard_normal(256))
    ref = torch.nn.functional.rms_norm(torch.from_numpy(x), (256,), torch.from_numpy(_wide(wb)),
                                       eps=float(np.float32(1e-6))).numpy()
    assert np.allclose(comp.rmsnorm(x, wb, 1e-6), ref, rtol=1e-12, atol=1e-14)


# ------------------------------------------------------------------ matvec
def test_matvec_vs_numpy_and_orientation(comp):
    rng = np.random.default_rng(2)
    W = _bits(rng.standard_normal((48, 80)) * 0.02)     # [out, in]
    x = rng.standard_normal(80)
    assert np.allclose(comp.matvec(x, W), _wide(W) @ x, rtol=1e-12, atol=1e-15)
    # a one-hot input picks a column of W (fails if the operand were transposed)
    e = np.zeros(80)
    e[7] = 1.0
    assert np.array_equal(comp.matvec(e, W), _wide(W)[:, 7])


# ------------------------------------------------------------------ RoPE
def test_rope_invariants(comp):
    rng = np.random.default_rng(3)
    hd = 64
    q, k = rng.standard_normal(hd), rng.standard_normal(hd)
    assert np.array_equal(comp.rope(q, 0), q)                                    # position 0 is the identity
    assert np.isclose(np.linalg.norm(comp.rope(q, 17)), np.linalg.norm(q), rtol=1e-13)   # a rotation
    a = comp.rope(q, 9) @ comp.rope(k, 4)
    b = comp.rope(q, 105) @ comp.rope(k, 100)
    c = comp.rope(q, 5) @ comp.rope(k, 0)
    assert np.isclose(a, b, rtol=1e-10) and np.isclose(a, c, rtol=1e-10)         # depends on m - n only
    assert not np.isclose(a, comp.rope(q, 9) @ comp.rope(k, 5), rtol=1e-6)


def test_rope_pairing_and_frequency(comp):
    hd, base = 8, 1.0e4
    # unit vector on element j rotates into element j + hd/2 by angle pos * base^(-2j/hd)
    for j in range(hd // 2):
        e = np.zeros(hd)
        e[j] = 1.0
        out = comp.rope(e, 3, base)
        ang = 3.0 * base ** (-2.0 * j / hd)
        want = np.zeros(hd)
        want[j], want[j + hd // 2] = math.cos(ang), math.sin(ang)
        assert np.allclose(out, want, atol=1e-15)


# ------------------------------------------------------------------ attention
def test_attention_special_cases(comp):
    rng = np.random.default_rng(4)
    hd = 32
    q = rng.standard_normal(hd)
    V = rng.standard_normal((5, hd))
    K_same = np.tile(rng.standard_normal(hd), (5, 1))
    assert np.allclose(comp.attention(q, K_same, V), V.mean(axis=0), rtol=1e-12)   # equal scores -> mean of values
    assert np.allclose(comp.attention(q, K_same[:1], V[:1]), V[0], rtol=1e-14)     # one key -> its value


def test_attention_vs_torch_sdpa(comp):
    rng = np.random.default_rng(5)
    T, hd = 37, 64
    q = rng.standard_normal((T, hd))
    K = rng.standard_normal((T, hd))
    V = rng.standard_normal((T, hd))
    ref = torch.nn.functional.scaled_dot_product_attention(
        torch.from_numpy(q)[None, None], torch.from_numpy(K)[None, None], torch.from_numpy(V)[None, None],
        is_causal=True)[0, 0].numpy()
    for t in (0, 1, 17, T - 1):
        assert np.allclose(comp.attention(q[t], K[:t + 1], V[:t + 1]), ref[t], rtol=1e-11, atol=1e-13)


def test_attention_large_scores_do_not_overflow(comp):
    hd = 16
    q = np.full(hd, 100.0)
    K = np.stack([np.full(hd, 100.0), np.full(hd, -100.0)])
    V = np.stack([np.ones(hd), -np.ones(hd)])
    assert np.allclose(comp.attention(q, K, V), np.ones(hd))


# ------------------------------------------------------------------ SiLU, argmax
def test_silu_vs_torch(comp):
    for z in (-30.0, -2.5, -1e-3, 0.0, 0.7, 4.0, 30.0):
        ref = float(torch.nn.functional.silu(torch.tensor(z, dtype=torch.float64)))
        assert math.isclose(comp.silu(z), ref, rel_tol=1e-13, abs_tol=1e-300)


def test_argmax_ties_and_margin(comp):
    i, mg = comp.argmax([0.1, 0.9, 0.3, 0.9, -1.0])
    assert i == 1 and mg == 0.0                 # duplicated maximum: lowest index, zero margin
    i, mg = comp.argmax([0.1, 0.2, 0.95, 0.9])
    assert i == 2 and math.isclose(mg, 0.05, rel_tol=1e-12)
    i, _ = comp.argmax([-3.0, -2.0, -5.0])
    assert i == 1


# ------------------------------------------------------------------ whole model vs an independent library model
def _hf_model(shape, tensors):
    from transformers import LlamaConfig, LlamaForCausalLM
    cfg = LlamaConfig(vocab_size=shape.vocab, hidden_size=shape.d_model, intermediate_size=shape.d_ffn,
                      num_hidden_layers=shape.n_layers, num_attention_heads=shape.n_heads,
                      num_key_value_heads=shape.n_heads, head_dim=shape.head_dim,
                      rms_norm_eps=float(np.float32(shape.rms_eps)), rope_theta=shape.rope_base,
                      tie_word_embeddings=False, attention_bias=False, mlp_bias=False,
                      max_position_embeddings=4096, hidden_act="silu")
    cfg._attn_implementation = "eager"
    m = LlamaForCausalLM(cfg).double().eval()
    names = dict(embed="model.embed_tokens.weight", final_norm="model.norm.weight", lm_head="lm_head.weight")
    per = dict(attn_norm="input_layernorm.weight", wq="self_attn.q_proj.weight", wk="self_attn.k_proj.weight",
               wv="self_attn.v_proj.weight", wo="self_attn.o_proj.weight", mlp_norm="post_attention_layernorm.weight",
               wg="mlp.gate_proj.weight", wu="mlp.up_proj.weight", wd="mlp.down_proj.weight")
    sd = {}
    for (name, _), t in zip(shape.tensor_specs(), tensors):
        if name in names:
            key = names[name]
        else:
            l, k = name.split(".")
            key = f"model.layers.{int(l[1:])}.{per[k]}"
        sd[key] = torch.from_numpy(_wide(t))
    missing, unexpected = m.load_state_dict(sd, strict=False)
    assert not unexpected and all("rotary" in k or "inv_freq" in k for k in missing), (missing, unexpected)
    return m


@pytest.fixture(scope="module")
def tiny(oracle_built):
    W = synth.make_weights(synth.TINY, seed=11, norm_jitter=0.1, threads=1)
    return W, OracleModel(synth.TINY, W, "f64"), _hf_model(synth.TINY, W)


def test_logits_match_independent_llama(tiny):
    W, om, hf = tiny
    rng = np.random.default_rng(6)
    toks = rng.integers(0, synth.TINY.vocab, size=41).astype(np.int32)
    with torch.no_grad():
        ref = hf(torch.from_numpy(toks.astype(np.int64))[None]).logits[0].numpy()
    full = om.teacher_forced(toks, first=0)
    # the library model evaluates its rotary cos/sin tables in fp32, which bounds the agreement near 1e-7
    assert np.abs(full - ref).max() <= 1e-6 * np.abs(ref).max()
    # key/value history extended one position at a time gives the same logits as the full causal forward
    inc = om.teacher_forced(toks, first=9, incremental=True)
    assert np.abs(inc - ref[9:]).max() <= 1e-6 * np.abs(ref).max()


def test_fp32_build_is_the_same_function(tiny, oracle_built):
    W, om, _ = tiny
    toks = np.random.default_rng(7).integers(0, synth.TINY.vocab, size=30).astype(np.int32)
    a = om.teacher_forced(toks, first=0)
    b = OracleModel(synth.TINY, W, "f32").teacher_forced(toks, first=0)
    assert np.abs(a - b).max() <= 2e-5 * np.abs(a).max()


def test_greedy_microbatch_semantics(tiny):
    W, om, hf = tiny
    w = synth.make_workload(1)
    cap = 20
    r = om.greedy_microbatch(w.prompt_tokens, w.prompt_offsets, cap, w.target_lens)
    t = w.target_lens
    assert np.array_equal(r["lens"], np.minimum(t, cap))
    assert np.array_equal(r["failed"].astype(bool), t > cap)
    assert r["steps"] == min(cap, int(t.max()))
    for i in range(w.n):
        L = int(r["lens"][i])
        assert (r["tokens"][i, :L] >= 0).all() and (r["tokens"][i, L:] == -1).all()
    # every emitted token is the argmax of the independent model's logits on the same prefix
    for i in (0, 3, 7):
        L = int(r["lens"][i])
        seq = np.concatenate([w.prompt(i), r["tokens"][i, :L]]).astype(np.int64)
        with torch.no_grad():
            lg = hf(torch.from_numpy(seq)[None]).logits[0].numpy()
        p = len(w.prompt(i))
        for g in range(L):
            if r["margins"][i, g] > 1e-5:
                assert int(np.argmax(lg[p - 1 + g])) == int(r["tokens"][i, g])
            top2 = np.sort(lg[p - 1 + g])[-2:]
            assert math.isclose(top2[1] - top2[0], r["margins"][i, g], rel_tol=1e-3, abs_tol=2e-6)


def test_a_row_that_ends_exactly_at_the_cap_has_not_failed(tiny):
    """Sec. 4.1, FCR: a row fails when it is still unfinished at the cap.  A response of exactly `cap` tokens is complete;
    one token more is a failure whose first `cap` tokens are the same."""
    W, om, hf = tiny
    w = synth.make_workload(1)
    toks, offs = w.prompt_tokens[:w.prompt_offsets[3]], w.prompt_offsets[:4]
    r = om.greedy_microbatch(toks, offs, 6, [6, 7, 5])
    assert r["failed"].tolist() == [0, 1, 0] and r["lens"].tolist() == [6, 6, 5] and r["steps"] == 6
    r1 = om.greedy_microbatch(toks, offs, 7, [6, 7, 5])
    assert r1["failed"].tolist() == [0, 0, 0] and r1["lens"].tolist() == [6, 7, 5] and r1["steps"] == 7
    assert np.array_equal(r["tokens"][1, :6], r1["tokens"][1, :6])


def test_query_output_independent_of_batch(tiny):
    """A query's tokens are the same alone, in a micro-batch, and after a capped (failed) first try."""
    W, om, _ = tiny
    w = synth.make_workload(1)
    full = om.greedy_microbatch(w.prompt_tokens, w.prompt_offsets, w.l_max, w.target_lens)
    for i in (1, 5, 12):
        t = int(w.target_lens[i])
        alone, _ = om.greedy_query(w.prompt(i), t)
        assert np.array_equal(alone[:t], full["tokens"][i, :t])
    capped = om.greedy_microbatch(w.prompt_tokens, w.prompt_offsets, 5, w.target_lens)
    for i in range(w.n):
        L = int(capped["lens"][i])
        assert np.array_equal(capped["tokens"][i, :L], full["tokens"][i, :L])


def test_bad_arguments_rejected(tiny):
    W, om, _ = tiny
    with pytest.raises(ValueError):
        om.greedy_microbatch([1, 2, 3], [0, 3], 0, [4])
    with pytest.raises(ValueError):
        om.greedy_microbatch([1, 2, synth.TINY.vocab], [0, 3], 4, [4])
