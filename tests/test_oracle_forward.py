"""Pins of the oracle's target forward and draft head.

The reference here is an independent full-sequence causal forward built from PyTorch CPU
library routines in fp64 (rms_norm, scaled_dot_product_attention with a causal mask,
silu, complex-number rotary embedding): batched over all positions at once, whereas the
oracle feeds one row at a time through a KV cache.  Agreement pins the layer arithmetic,
the cache indexing and the equivalence "k+1 rows in one pass == token by token"
(Preliminary, "Speculative Sampling": one target pass verifies the drafted positions in
parallel).
"""
import numpy as np
import pytest
import torch
import torch.nn.functional as F

import oracle
import synth


def torch_forward(shape, blob, x):
    """x: [T, d] fp64 input embeddings -> (hidden before final norm [T, d], logits [T, V_s])."""
    W = lambda name: torch.from_numpy(synth.blob_tensor(shape, blob, name)).double()
    T, d = x.shape
    H, hd = shape.n_heads, shape.head_dim
    pos = torch.arange(T, dtype=torch.float64)
    inv = shape.rope_theta ** (-torch.arange(0, hd, 2, dtype=torch.float64) / hd)
    rot = torch.polar(torch.ones(T, hd // 2, dtype=torch.float64), pos[:, None] * inv[None, :])

    def rope(t):  # t: [T, H, hd]
        c = torch.view_as_complex(t.reshape(T, H, hd // 2, 2).contiguous())
        return torch.view_as_real(c * rot[:, None, :]).reshape(T, H, hd)

    h = x.clone()
    for l in range(shape.n_layers):
        a = F.rms_norm(h, (d,), W(f"l{l}.g1"), eps=shape.rms_eps)
        q = rope((a @ W(f"l{l}.Wq").T).reshape(T, H, hd)).transpose(0, 1)
        k = rope((a @ W(f"l{l}.Wk").T).reshape(T, H, hd)).transpose(0, 1)
        v = (a @ W(f"l{l}.Wv").T).reshape(T, H, hd).transpose(0, 1)
        o = F.scaled_dot_product_attention(q[None], k[None], v[None], is_causal=True)[0]
        h = h + o.transpose(0, 1).reshape(T, d) @ W(f"l{l}.Wo").T
        b = F.rms_norm(h, (d,), W(f"l{l}.g2"), eps=shape.rms_eps)
        h = h + (F.silu(b @ W(f"l{l}.W1").T) * (b @ W(f"l{l}.W3").T)) @ W(f"l{l}.W2").T
    f = F.rms_norm(h, (d,), W("g_f"), eps=shape.rms_eps)
    lo = shape.samp_lo
    logits = f @ W("W_out")[lo:lo + shape.v_s].T
    return h, logits


@pytest.mark.parametrize("dtype,samp", [("fp32", (0, 0)), ("bf16", (0, 0)), ("bf16", (6, 24))])
def test_incremental_forward_matches_torch_full_causal(micro_shape, dtype, samp):
    s = micro_shape.replace(dtype=dtype, samp_lo=samp[0], samp_n=samp[1])
    blob = synth.make_weights(s, seed=5, std=0.2)  # larger weights: attention far from uniform
    o = oracle.Oracle.from_shape(s, blob)
    T = s.n_cond + s.n_img
    rng = np.random.default_rng(0)
    x = rng.standard_normal((T, s.d_model))
    h_ref, lg_ref = torch_forward(s, blob, torch.from_numpy(x))
    for t in range(T):
        h, lg = o.forward_row(0, t, x[t])
        np.testing.assert_allclose(h, h_ref[t].numpy(), rtol=1e-10, atol=1e-11)
        np.testing.assert_allclose(lg, lg_ref[t].numpy().astype(np.float32), rtol=2e-6, atol=1e-6)
    # re-feeding a suffix over the existing cache reproduces the same rows bit for bit
    h_a, lg_a = o.forward_row(0, T - 3, x[T - 3])
    h_b, lg_b = o.forward_row(0, T - 3, x[T - 3])
    assert (h_a == h_b).all() and (lg_a == lg_b).all()
    np.testing.assert_allclose(h_a, h_ref[T - 3].numpy(), rtol=1e-10, atol=1e-11)


def test_draft_head_hand_computed():
    s = synth.HawkShape("hand", 1, 4, 2, 6, 8, 2, 2, 3, 2, dtype="fp32", top_k=8)
    blob = synth.make_weights(s, seed=7, std=0.5)
    o = oracle.Oracle.from_shape(s, blob)
    E = synth.blob_tensor(s, blob, "E").astype(np.float64)
    Wd = synth.blob_tensor(s, blob, "W_d").astype(np.float64)
    Wout = synth.blob_tensor(s, blob, "W_out").astype(np.float64)
    g = np.array([0.5, -1.0, 2.0, 0.25])
    for left, up in ((3, 5), (0, -1), (7, 7)):
        cat = np.concatenate([g, E[left], E[up] if up >= 0 else np.zeros(4)])
        want_g = Wd @ cat
        got_g, lg = o.draft_head(g, left, up)
        np.testing.assert_allclose(got_g, want_g, rtol=1e-14, atol=1e-15)
        nrm = want_g / np.sqrt(np.mean(want_g ** 2) + s.rms_eps)
        np.testing.assert_allclose(lg, (Wout @ nrm).astype(np.float32), rtol=2e-6, atol=1e-7)
    # the three input blocks are read in the order [hidden | left | up]
    got_g, _ = o.draft_head(np.zeros(4), 2, -1, want_logits=False)
    np.testing.assert_allclose(got_g, Wd[:, 4:8] @ E[2], rtol=1e-14, atol=1e-15)
    got_g, _ = o.draft_head(np.zeros(4), 2, 6, want_logits=False)
    np.testing.assert_allclose(got_g, Wd[:, 4:8] @ E[2] + Wd[:, 8:12] @ E[6], rtol=1e-14, atol=1e-15)


def test_bf16_blob_values_are_exact_bf16_of_the_fp32_draw():
    s32 = synth.HawkShape("a", 1, 8, 2, 16, 32, 2, 2, 2, 1, dtype="fp32")
    s16 = s32.replace(dtype="bf16")
    w32 = synth.blob_tensor(s32, synth.make_weights(s32, 3), "l0.W1")
    w16 = synth.blob_tensor(s16, synth.make_weights(s16, 3), "l0.W1")
    ref = torch.from_numpy(w32).to(torch.bfloat16).float().numpy()  # torch rounds to nearest even
    assert (w16 == ref).all()
    assert np.all(synth.blob_tensor(s16, synth.make_weights(s16, 3), "g_f") == 1.0)


@pytest.mark.parametrize("guided", [False, True])
def test_prefill_hands_over_the_last_condition_rows_hidden_state(micro_shape, guided):
    # The hidden state the draft head continues from after the prefill (Preliminary, "Utilization of
    # Draft Heads Structure": heads read the final hidden layer) is the last condition row's output of
    # the last layer, before the final norm - per stream under guidance.  Pinned against the full causal
    # PyTorch forward over the condition vectors, which shares nothing with the oracle's prefill.
    s = micro_shape.replace(cfg_scale=2.5) if guided else micro_shape
    blob = synth.make_weights(s, seed=5, std=0.2)
    B = 2
    cond = synth.make_cond(s, seed=2, batch=B)
    unc = synth.make_cond(s, seed=3, batch=B) if guided else None
    o = oracle.Oracle.from_shape(s, blob, batch=B)
    o.prefill(cond, unc, 1.0, 10, s.cfg_scale, [0.3, 0.7])
    hp = o.h_prev()
    assert hp.shape == ((2 if guided else 1) * B, s.d_model)
    for b in range(B):
        h_ref, lg_ref = torch_forward(s, blob, torch.from_numpy(cond[b].astype(np.float64)))
        np.testing.assert_allclose(hp[b], h_ref[-1].numpy(), rtol=1e-10, atol=1e-11)
        if guided:   # the unconditional stream of prompt b is sequence B + b
            hu_ref, lu_ref = torch_forward(s, blob, torch.from_numpy(unc[b].astype(np.float64)))
            np.testing.assert_allclose(hp[B + b], hu_ref[-1].numpy(), rtol=1e-10, atol=1e-11)
            assert not np.allclose(hp[b], hp[B + b])
            lg_ref = lu_ref[-1] + s.cfg_scale * (lg_ref[-1] - lu_ref[-1])
        else:
            lg_ref = lg_ref[-1]
        # and the first token is the draw from that row's (guided) logits
        w, z = oracle.warp(lg_ref.numpy().astype(np.float32), 1.0, 10)
        assert o.grid()[b, 0] == s.samp_lo + oracle.inv_cdf(w, z, [0.3, 0.7][b])
