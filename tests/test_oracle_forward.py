"""Pins for the oracle's decoder forward pass (CPU only).

The paper fixes the architecture only by naming the model family (Section 4.1 "Models": LLaMA-68M /
LLaMA-2-7B ...), and prints no worked numbers.  The forward pass is therefore pinned to an independent
library implementation of that family, plus structural invariants that a dropped term, a wrong sign, a
wrong index or a transposed operand would break.
"""
import numpy as np
import pytest
import torch

import oracle
import workloads as wl


@pytest.fixture(scope="module")
def tiny():
    w = wl.get_workload("c1")
    return w, wl.Weights(w.model, w.seed)


def _hf_model(m, W):
    from transformers import LlamaConfig, LlamaForCausalLM
    cfg = LlamaConfig(vocab_size=m.vocab, hidden_size=m.d_model, intermediate_size=m.d_ff,
                      num_hidden_layers=m.n_layers, num_attention_heads=m.n_heads,
                      num_key_value_heads=m.n_heads, head_dim=m.head_dim, rms_norm_eps=m.rms_eps,
                      rope_theta=m.rope_theta, attention_bias=False, mlp_bias=False,
                      tie_word_embeddings=False, max_position_embeddings=512, attn_implementation="eager")
    model = LlamaForCausalLM(cfg).double().eval()
    names = {"wq": "self_attn.q_proj", "wk": "self_attn.k_proj", "wv": "self_attn.v_proj",
             "wo": "self_attn.o_proj", "wgate": "mlp.gate_proj", "wup": "mlp.up_proj",
             "wdown": "mlp.down_proj", "norm_attn": "input_layernorm", "norm_ffn": "post_attention_layernorm"}
    sd = {"model.embed_tokens.weight": W.tok_emb(), "model.norm.weight": W.norm_final(),
          "lm_head.weight": W.lm_head()}
    for l in range(m.n_layers):
        for k, v in W.layer(l).items():
            sd[f"model.layers.{l}.{names[k]}.weight"] = v
    model.load_state_dict({k: torch.from_numpy(np.array(v)).double() for k, v in sd.items()}, strict=True)
    return model


def test_forward_matches_library_llama(tiny):
    """Plain causal forward == transformers' LlamaForCausalLM in float64 with the same weights (the
    library evaluates the rotary cos/sin tables in float32, hence 1e-6 rather than 1e-12)."""
    w, W = tiny
    toks = wl.prefix_tokens(w)[:48]
    model = _hf_model(w.model, W)
    with torch.no_grad():
        ref = model(torch.from_numpy(toks.astype(np.int64))[None]).logits[0].numpy()
    got, _, _ = oracle.decode_rows(w.model, W, toks)
    assert got.shape == ref.shape
    assert np.abs(got - ref).max() < 1e-6 * max(1.0, np.abs(ref).max())


def test_library_llama_with_cache_matches_rows_against_context(tiny):
    """Rows decoded against a context KV == the library model run with its own KV cache."""
    w, W = tiny
    toks = wl.prefix_tokens(w)
    ctx, new = toks[:40], toks[40:47]
    model = _hf_model(w.model, W)
    with torch.no_grad():
        out = model(torch.from_numpy(ctx.astype(np.int64))[None], use_cache=True)
        ref = model(torch.from_numpy(new.astype(np.int64))[None], past_key_values=out.past_key_values,
                    use_cache=True).logits[0].numpy()
    _, ks, vs = oracle.decode_rows(w.model, W, ctx)
    got, _, _ = oracle.decode_rows(w.model, W, new, ctx_kv=lambda l: (ks[l], vs[l]), pos0=len(ctx))
    assert np.abs(got - ref).max() < 1e-6 * max(1.0, np.abs(ref).max())


def test_verify_rows_equal_separate_plain_forwards(tiny):
    """Batched verify over (shared prefix + private context + draft rows) == N ordinary causal forwards
    of the concatenated sequences without any cache (Section 3.1: the verify phase returns the plain
    model's distributions given (c, x_<j))."""
    w, W = tiny
    m = w.model
    rng = np.random.default_rng(7)
    shared = wl.prefix_tokens(w)[:20]
    priv = [rng.integers(0, m.vocab, size=r).astype(np.int32) for r in (0, 3, 5)]
    rows = rng.integers(0, m.vocab, size=(3, 4)).astype(np.int32)
    _, ks, vs = oracle.decode_rows(m, W, shared)
    pk, pv = [], []
    for b in range(3):       # private context KV per branch, computed against the shared prefix
        _, kb, vb = oracle.decode_rows(m, W, priv[b], ctx_kv=lambda l: (ks[l], vs[l]), pos0=len(shared))
        pk.append(kb)
        pv.append(vb)

    def ctx(l):
        return [(np.concatenate([ks[l], pk[b][l]], axis=1), np.concatenate([vs[l], pv[b][l]], axis=1))
                for b in range(3)]
    pos0 = [len(shared) + len(priv[b]) for b in range(3)]
    got = oracle.verify_forward(m, W, rows, ctx, pos0)
    for b in range(3):
        seq = np.concatenate([shared, priv[b], rows[b]])
        full, _, _ = oracle.decode_rows(m, W, seq)
        assert np.abs(got[b] - full[-4:]).max() < 1e-10


def test_branches_do_not_interfere(tiny):
    """Permuting branches permutes the outputs bit for bit; changing one branch's rows leaves the
    others bit-identical (Section 3: branches are independent of each other)."""
    w, W = tiny
    m = w.model
    rng = np.random.default_rng(11)
    shared = wl.prefix_tokens(w)[:16]
    rows = rng.integers(0, m.vocab, size=(3, 4)).astype(np.int32)
    _, ks, vs = oracle.decode_rows(m, W, shared)
    ctx = lambda l: [(ks[l], vs[l])] * 3
    base = oracle.verify_forward(m, W, rows, ctx, [16] * 3)
    perm = [2, 0, 1]
    assert np.array_equal(oracle.verify_forward(m, W, rows[perm], ctx, [16] * 3), base[perm])
    rows2 = rows.copy()
    rows2[1] = (rows2[1] + 1) % m.vocab
    other = oracle.verify_forward(m, W, rows2, ctx, [16] * 3)
    assert np.array_equal(other[0], base[0]) and np.array_equal(other[2], base[2])
    assert not np.array_equal(other[1], base[1])


def test_rope_is_a_rotation_by_relative_offset():
    """Rotary scores depend only on the position difference; position 0 is the identity; norms are kept."""
    rng = np.random.default_rng(3)
    q = rng.standard_normal((5, 2, 64))
    k = rng.standard_normal((5, 2, 64))
    pq, pk = np.array([3, 9, 4, 100, 7]), np.array([1, 2, 4, 60, 0])
    s0 = np.einsum("thd,thd->th", oracle.rope_rotate(q, pq, 10000.0), oracle.rope_rotate(k, pk, 10000.0))
    s1 = np.einsum("thd,thd->th", oracle.rope_rotate(q, pq + 37, 10000.0), oracle.rope_rotate(k, pk + 37, 10000.0))
    assert np.abs(s0 - s1).max() < 1e-10
    assert np.array_equal(oracle.rope_rotate(q, np.zeros(5, int), 10000.0), q)
    assert np.allclose(np.linalg.norm(oracle.rope_rotate(q, pq, 10000.0), axis=-1), np.linalg.norm(q, axis=-1))
    # first pair (i=0, frequency 1) at position 1 is a rotation by exactly one radian
    x = np.zeros((1, 1, 64)); x[0, 0, 0] = 1.0
    y = oracle.rope_rotate(x, np.array([1]), 10000.0)
    assert abs(y[0, 0, 0] - np.cos(1.0)) < 1e-15 and abs(y[0, 0, 32] - np.sin(1.0)) < 1e-15


def test_rms_norm_closed_form():
    x = np.array([[3.0, 4.0, 0.0, 0.0]])
    out = oracle.rms_norm(x, np.array([1.0, 2.0, 1.0, 1.0]), 0.0)
    assert np.allclose(out, [[3 / 2.5, 2 * 4 / 2.5, 0, 0]])     # rms = sqrt(25/4) = 2.5
