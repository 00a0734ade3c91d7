"""Pins for the CPU oracle: invariants, closed forms, textbook special cases, library routines and
values the paper prints.  None of these tests touches the HIP path."""
import os

import numpy as np
import pytest
import torch
import torch.nn.functional as F

import oracle as orc
from paper_2404_06709_amd import synth

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")
TINY = synth.SHAPES["tiny"]


def tiny_dims(max_seq=64, wdtype=orc.F32):
    return orc.Dims(TINY.d_model, TINY.n_heads, TINY.head_dim, TINY.d_ffn, max_seq, 10000.0, 1e-6, wdtype)


def tiny_layers(n, seed=1001, dtype=torch.float32, jitter=0.1, w_std=0.05):
    # larger std than the workload's 0.02 so that every branch contributes visibly
    tl = synth.make_layers(n, TINY, dtype, seed, w_std=w_std, gain_jitter=jitter)
    return tl, [synth.layer_to_numpy(L) for L in tl]


def hidden(B, T, seed=7):
    return synth.widen(synth.normal((B, T, TINY.d_model), 1.0, torch.float32, synth.generator(seed)))


# ----------------------------------------------------------------------------- library composition
def torch_rope(v, pos, base):
    """Rotary embedding through complex multiplication: (v[i] + j v[i+half]) * exp(j pos theta_i)."""
    half = v.shape[-1] // 2
    theta = base ** (-torch.arange(half, dtype=torch.float64) * 2.0 / v.shape[-1])
    rot = torch.polar(torch.ones(half, dtype=torch.float64), pos * theta)
    z = torch.complex(v[..., :half], v[..., half:]) * rot
    return torch.cat([z.real, z.imag], dim=-1)


def torch_attn(tl, x, kpast, vpast, eps=1e-6, base=10000.0):
    """ATTN_l for one sequence from torch library routines in fp64.
    x [T,dm]; kpast/vpast [n,S,dk] (K already rotated).  Returns (a [T,dm], k_all, v_all)."""
    W = {k: v.to(torch.float64) for k, v in tl.items()}
    T, dm = x.shape
    n, dk = TINY.n_heads, TINY.head_dim
    S = kpast.shape[1]
    nrm = F.rms_norm(x, (dm,), W["g_attn"], eps)
    q = F.linear(nrm, W["wq"]).view(T, n, dk).transpose(0, 1)
    k = F.linear(nrm, W["wk"]).view(T, n, dk).transpose(0, 1)
    v = F.linear(nrm, W["wv"]).view(T, n, dk).transpose(0, 1)
    pos = torch.arange(S, S + T, dtype=torch.float64)
    q = torch.stack([torch_rope(q[:, t], pos[t], base) for t in range(T)], dim=1)
    k = torch.stack([torch_rope(k[:, t], pos[t], base) for t in range(T)], dim=1)
    k_all = torch.cat([kpast, k], dim=1)
    v_all = torch.cat([vpast, v], dim=1)
    mask = torch.ones(T, S + T, dtype=torch.bool).tril(diagonal=S)
    ctx = F.scaled_dot_product_attention(q, k_all, v_all, attn_mask=mask)
    a = F.linear(ctx.transpose(0, 1).reshape(T, dm), W["wo"])
    return a, k_all, v_all


def torch_ffn(tl, h, eps=1e-6):
    W = {k: v.to(torch.float64) for k, v in tl.items()}
    nrm = F.rms_norm(h, (h.shape[-1],), W["g_ffn"], eps)
    return F.linear(F.silu(F.linear(nrm, W["wgate"])) * F.linear(nrm, W["wup"]), W["wdown"])


# ----------------------------------------------------------------------------- primitives (I8)
def test_linear_is_matrix_vector_product():
    gen = synth.generator(3)
    W = synth.normal((37, 53), 1.0, torch.float32, gen)
    x = synth.widen(synth.normal((53,), 1.0, torch.float32, gen))
    y = orc.linear(synth.to_numpy(W), x)
    np.testing.assert_allclose(y, W.double().numpy() @ x, rtol=1e-13, atol=1e-13)
    # a transposed operand would fail on a non-square matrix with distinct rows
    e3 = np.zeros(53); e3[3] = 1.0
    np.testing.assert_array_equal(orc.linear(synth.to_numpy(W), e3), W[:, 3].double().numpy())


def test_bf16_weights_are_widened_exactly():
    W = synth.normal((8, 16), 1.0, torch.bfloat16, synth.generator(5))
    e = np.zeros(16); e[5] = 1.0
    np.testing.assert_array_equal(orc.linear(synth.to_numpy(W), e), W[:, 5].double().numpy())


def test_rmsnorm_closed_form():
    x = hidden(1, 1)[0, 0]
    ones = np.ones(x.shape[0], dtype=np.float32)
    eps = 1e-2
    out = orc.rmsnorm(x, ones, eps)
    ms = np.mean(x * x)
    assert np.isclose(np.mean(out * out), ms / (ms + eps), rtol=1e-13)
    # gain multiplies element-wise; compare with the torch library routine
    g = synth.to_numpy(1.0 + synth.normal((x.shape[0],), 0.3, torch.float32, synth.generator(9)))
    ref = F.rms_norm(torch.from_numpy(x), (x.shape[0],), torch.from_numpy(g).double(), eps).numpy()
    np.testing.assert_allclose(orc.rmsnorm(x, g, eps), ref, rtol=1e-13)


def test_silu_values():
    assert orc.silu(0.0) == 0.0
    for z in (-20.0, -3.0, -0.5, 0.25, 1.0, 7.5):
        assert np.isclose(orc.silu(z), F.silu(torch.tensor(z, dtype=torch.float64)).item(), rtol=1e-14)


def test_rope_properties():
    gen = synth.generator(11)
    q = synth.widen(synth.normal((64,), 1.0, torch.float32, gen))
    k = synth.widen(synth.normal((64,), 1.0, torch.float32, gen))
    np.testing.assert_array_equal(orc.rope(q, 0), q)                     # position 0 is the identity
    r = orc.rope(q, 17)
    np.testing.assert_allclose(r[:32] ** 2 + r[32:] ** 2, q[:32] ** 2 + q[32:] ** 2, rtol=1e-13)
    # the score depends only on the distance between the positions
    d1 = orc.rope(q, 29) @ orc.rope(k, 12)
    d2 = orc.rope(q, 117) @ orc.rope(k, 100)
    assert np.isclose(d1, d2, rtol=1e-12)
    # direction and pairing: complex-multiplication formulation
    ref = torch_rope(torch.from_numpy(q), torch.tensor(23.0, dtype=torch.float64), 10000.0).numpy()
    np.testing.assert_allclose(orc.rope(q, 23), ref, rtol=1e-12, atol=1e-14)
    # pair 0 turns by exactly pos radians, the last pair by pos * base^(-(d-2)/d)
    e = np.zeros(64); e[0] = 1.0
    r = orc.rope(e, 2)
    assert np.isclose(r[0], np.cos(2.0)) and np.isclose(r[32], np.sin(2.0))
    e = np.zeros(64); e[31] = 1.0
    r = orc.rope(e, 1000)
    phi = 1000.0 * 10000.0 ** (-62.0 / 64.0)
    assert np.isclose(r[31], np.cos(phi)) and np.isclose(r[63], np.sin(phi))


def test_attention_single_slot_returns_wo_v():
    """KV length 1: softmax over one score is 1, so ATTN(x) = Wo (Wv Norm(x))."""
    D = tiny_dims()
    tl, nl = tiny_layers(1)
    x = hidden(1, 1)
    kc, vc = orc.new_cache(1, 1, D), orc.new_cache(1, 1, D)
    a = orc.attn_module(D, nl[0], 0, kc, vc, [0], x)
    n = orc.rmsnorm(x[0, 0], nl[0]["g_attn"], D.rms_eps)
    np.testing.assert_allclose(a[0, 0], orc.linear(nl[0]["wo"], orc.linear(nl[0]["wv"], n)), rtol=1e-12, atol=1e-15)


def test_attention_equal_keys_average_values():
    """All cached keys equal (and Wk = 0 so the new key is the zero vector like them):
    the softmax is uniform and the context is the mean of the values."""
    D = tiny_dims()
    tl, nl = tiny_layers(1)
    nl[0]["wk"] = np.zeros_like(nl[0]["wk"])
    S = 9
    kc, vc = orc.new_cache(1, 1, D), orc.new_cache(1, 1, D)
    vc[0, 0, :, :S, :] = synth.widen(synth.normal((D.n_heads, S, D.head_dim), 1.0, torch.float32, synth.generator(2)))
    x = hidden(1, 1)
    a = orc.attn_module(D, nl[0], 0, kc, vc, [S], x)
    ctx = vc[0, 0, :, : S + 1, :].mean(axis=1).reshape(-1)
    np.testing.assert_allclose(a[0, 0], orc.linear(nl[0]["wo"], ctx), rtol=1e-11, atol=1e-14)


# ----------------------------------------------------------------------------- I10: library composition
@pytest.mark.parametrize("S,T", [(0, 6), (5, 1), (3, 4)])
def test_seq_layer_matches_torch_library_composition(S, T):
    D = tiny_dims()
    tl, nl = tiny_layers(1)
    gen = synth.generator(21)
    kpast = synth.normal((D.n_heads, S, D.head_dim), 1.0, torch.float32, gen).double()
    vpast = synth.normal((D.n_heads, S, D.head_dim), 1.0, torch.float32, gen).double()
    x = hidden(1, T)
    kc, vc = orc.new_cache(1, 1, D), orc.new_cache(1, 1, D)
    kc[0, 0, :, :S] = kpast.numpy(); vc[0, 0, :, :S] = vpast.numpy()
    out = orc.seq_layer(D, nl[0], kc, vc, [S], x)
    xt = torch.from_numpy(x[0])
    a, k_all, v_all = torch_attn(tl[0], xt, kpast, vpast)
    h = xt + a
    ref = h + torch_ffn(tl[0], h)
    np.testing.assert_allclose(out[0], ref.numpy(), rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(kc[0, 0, :, : S + T], k_all.numpy(), rtol=1e-11, atol=1e-13)
    np.testing.assert_allclose(vc[0, 0, :, : S + T], v_all.numpy(), rtol=1e-11, atol=1e-13)
    assert not kc[0, 0, :, S + T:].any() and not vc[0, 0, :, S + T:].any()


@pytest.mark.parametrize("P,d", [(3, 1), (4, 2), (2, 0)])
def test_group_forward_matches_eq4_written_with_library_modules(P, d):
    D = tiny_dims()
    tl, nl = tiny_layers(P)
    S, T = 4, 3
    gen = synth.generator(33)
    kc, vc = orc.new_cache(P, 1, D), orc.new_cache(P, 1, D)
    kp = [synth.normal((D.n_heads, S, D.head_dim), 1.0, torch.float32, gen).double() for _ in range(P)]
    vp = [synth.normal((D.n_heads, S, D.head_dim), 1.0, torch.float32, gen).double() for _ in range(P)]
    for i in range(P):
        kc[i, 0, :, :S] = kp[i].numpy(); vc[i, 0, :, :S] = vp[i].numpy()
    x = hidden(1, T)
    out = orc.group_forward(D, nl, d, kc, vc, [S], x)
    xt = torch.from_numpy(x[0])
    attn = [torch_attn(tl[i], xt, kp[i], vp[i])[0] for i in range(P)]
    ref = xt + sum(attn)
    for l in range(P):
        ffn_in = xt + attn[l] + sum((attn[lp] for lp in range(P) if 1 <= l - lp <= d), torch.zeros_like(xt))
        ref = ref + torch_ffn(tl[l], ffn_in)
    np.testing.assert_allclose(out[0], ref.numpy(), rtol=1e-10, atol=1e-12)


# ----------------------------------------------------------------------------- Sec.3.1 input similarity
def test_input_similarity_textbook_cases():
    """Per-token cosine, mean over tokens: equal directions 1, opposite -1, orthogonal 0, scale-free, symmetric,
    and a hand-computed 45-degree pair; a mean over vectors instead of over cosines would fail the last check."""
    n = 8
    e0 = np.zeros(n); e0[0] = 1.0
    e1 = np.zeros(n); e1[1] = 1.0
    X = np.stack([
        np.stack([e0, e1]),                    # layer 0
        np.stack([3.0 * e0, -2.0 * e1]),       # layer 1: same direction, opposite direction
        np.stack([e1, e0 + e1]),               # layer 2: orthogonal, 45 degrees
    ])
    sim = orc.input_similarity(X)
    np.testing.assert_allclose(np.diag(sim), 1.0, rtol=0, atol=1e-15)
    np.testing.assert_allclose(sim, sim.T, rtol=0, atol=0)
    assert abs(sim[0, 1] - 0.0) < 1e-15                    # (1 + (-1)) / 2
    assert abs(sim[0, 2] - (0.0 + np.sqrt(0.5)) / 2) < 1e-15
    assert abs(sim[1, 2] - (0.0 - np.sqrt(0.5)) / 2) < 1e-15
    # scale invariance and agreement with the library routine on random data
    gen = synth.generator(91)
    Y = synth.widen(synth.normal((4, 5, 24), 1.0, torch.float32, gen))
    s1 = orc.input_similarity(Y)
    s2 = orc.input_similarity(Y * np.array([1.0, 7.0, 0.25, 3.0])[:, None, None])
    np.testing.assert_allclose(s1, s2, rtol=1e-13, atol=1e-14)
    t = torch.from_numpy(Y)
    ref = F.cosine_similarity(t[:, None], t[None, :], dim=-1).mean(dim=-1)
    np.testing.assert_allclose(s1, ref.numpy(), rtol=1e-12, atol=1e-13)


# ----------------------------------------------------------------------------- LoRA merge (alpha = rank)
def test_lora_merge_unit_vectors_touch_one_element():
    """Bm = e_i (column j0 of the rank axis), A = c e_k^T: only W[i,k] changes, by c.  A transposed operand or a
    swapped index would move the change elsewhere (the matrix is not square)."""
    gen = synth.generator(61)
    W = synth.to_numpy(synth.normal((5, 9), 1.0, torch.float32, gen))
    A = np.zeros((3, 9), dtype=np.float32); Bm = np.zeros((5, 3), dtype=np.float32)
    A[1, 7] = 0.25; Bm[4, 1] = 1.0
    out = orc.merge_lora(W, A, Bm)
    delta = out - W.astype(np.float64)
    expect = np.zeros((5, 9)); expect[4, 7] = 0.25
    np.testing.assert_array_equal(delta, expect)
    np.testing.assert_array_equal(orc.merge_lora(W, A, np.zeros_like(Bm)), W.astype(np.float64))   # Bm = 0: identity
    np.testing.assert_array_equal(orc.merge_lora(W, A, Bm, scale=-2.0) - W, -2.0 * expect)


@pytest.mark.parametrize("bf16", [False, True])
def test_lora_merged_matrix_acts_as_base_plus_low_rank_path(bf16):
    """(W + Bm A) x = W x + Bm (A x): the merged weights give what the adapter computes on the side."""
    gen = synth.generator(62)
    dt = torch.bfloat16 if bf16 else torch.float32
    W = synth.to_numpy(synth.normal((24, 40), 0.05, dt, gen))
    A = synth.to_numpy(synth.normal((4, 40), 0.3, dt, gen))
    Bm = synth.to_numpy(synth.normal((24, 4), 0.3, dt, gen))
    x = synth.widen(synth.normal((40,), 1.0, torch.float32, gen))
    merged = orc.merge_lora(W, A, Bm)
    side = orc.linear(W, x) + orc.linear(Bm, orc.linear(A, x))
    np.testing.assert_allclose(merged @ x, side, rtol=1e-12, atol=1e-13)


# ----------------------------------------------------------------------------- App. A, Eq.5 (d = -1)
@pytest.mark.parametrize("P", [1, 3])
def test_attention_ffn_parallel_form_matches_library_modules(P):
    """x_out = x + sum ATTN_l(x) + sum FFN_l(x): the feed-forward modules read the shared input, not x + a."""
    D = tiny_dims()
    tl, nl = tiny_layers(P)
    S, T = 4, 3
    gen = synth.generator(34)
    kc, vc = orc.new_cache(P, 1, D), orc.new_cache(P, 1, D)
    kp = [synth.normal((D.n_heads, S, D.head_dim), 1.0, torch.float32, gen).double() for _ in range(P)]
    vp = [synth.normal((D.n_heads, S, D.head_dim), 1.0, torch.float32, gen).double() for _ in range(P)]
    for i in range(P):
        kc[i, 0, :, :S] = kp[i].numpy(); vc[i, 0, :, :S] = vp[i].numpy()
    x = hidden(1, T)
    out, attn_dbg, h_dbg = orc.group_forward(D, nl, -1, kc, vc, [S], x, debug=True)
    xt = torch.from_numpy(x[0])
    ref = xt.clone()
    for l in range(P):
        ref = ref + torch_attn(tl[l], xt, kp[l], vp[l])[0] + torch_ffn(tl[l], xt)
    np.testing.assert_allclose(out[0], ref.numpy(), rtol=1e-10, atol=1e-12)
    for l in range(P):
        np.testing.assert_array_equal(h_dbg[l], x)          # FFN input is x itself
    # it differs from Eq.3 (d = 0) whenever the attention output is not zero
    kc2, vc2 = kc.copy(), vc.copy()
    eq3 = orc.group_forward(D, nl, 0, kc2, vc2, [S], x)
    assert np.abs(eq3 - out).max() > 1e-6


def test_attention_ffn_parallel_form_equals_eq1_when_attention_is_silent():
    """With W^O = 0 the attention output vanishes and Eq.5 and Eq.1 coincide bit for bit."""
    D = tiny_dims()
    _, nl = tiny_layers(1)
    nl[0] = dict(nl[0]); nl[0]["wo"] = np.zeros_like(nl[0]["wo"])
    S = [5]
    x = hidden(1, 2)
    kc, vc = _filled_caches(1, 1, D, S)
    a = orc.group_forward(D, nl, -1, kc.copy(), vc.copy(), S, x)
    b = orc.seq_layer(D, nl[0], kc.copy(), vc.copy(), S, x)
    np.testing.assert_array_equal(a, b)


def test_attention_ffn_parallel_form_is_additive_in_the_attention_branch():
    """x_out(W^O) - x_out(0) = ATTN(x): the feed-forward term does not see the attention output."""
    D = tiny_dims()
    _, nl = tiny_layers(2)
    S = [6]
    x = hidden(1, 3)
    kc, vc = _filled_caches(2, 1, D, S)
    full, attn, _ = orc.group_forward(D, nl, -1, kc.copy(), vc.copy(), S, x, debug=True)
    silent = [dict(l, wo=np.zeros_like(l["wo"])) for l in nl]
    base = orc.group_forward(D, silent, -1, kc.copy(), vc.copy(), S, x)
    np.testing.assert_allclose(full - base, attn.sum(axis=0), rtol=0, atol=1e-12)


# ----------------------------------------------------------------------------- invariants I1-I7
def _filled_caches(P, B, D, S, seed=55):
    gen = synth.generator(seed)
    kc, vc = orc.new_cache(P, B, D), orc.new_cache(P, B, D)
    for b in range(B):
        kc[:, b, :, : S[b]] = synth.widen(synth.normal((P, D.n_heads, S[b], D.head_dim), 1.0, torch.float32, gen))
        vc[:, b, :, : S[b]] = synth.widen(synth.normal((P, D.n_heads, S[b], D.head_dim), 1.0, torch.float32, gen))
    return kc, vc


@pytest.mark.parametrize("d", [0, 1, 3])
def test_I1_group_of_one_is_the_sequential_layer(d):
    D = tiny_dims()
    _, nl = tiny_layers(1)
    S = [3, 7]
    x = hidden(2, 2)
    kc1, vc1 = _filled_caches(1, 2, D, S)
    kc2, vc2 = kc1.copy(), vc1.copy()
    a = orc.group_forward(D, nl, d, kc1, vc1, S, x)
    b = orc.seq_layer(D, nl[0], kc2, vc2, S, x)
    np.testing.assert_array_equal(a, b)
    np.testing.assert_array_equal(kc1, kc2)
    np.testing.assert_array_equal(vc1, vc2)


@pytest.mark.parametrize("P,d", [(1, 0), (2, 1), (4, 2)])
def test_I2_zero_output_projections_give_identity(P, d):
    D = tiny_dims()
    _, nl = tiny_layers(P)
    for L in nl:
        L["wo"] = np.zeros_like(L["wo"]); L["wdown"] = np.zeros_like(L["wdown"])
    x = hidden(1, 3)
    kc, vc = _filled_caches(P, 1, D, [2])
    np.testing.assert_array_equal(orc.group_forward(D, nl, d, kc, vc, [2], x), x)


@pytest.mark.parametrize("P", [2, 4])
def test_I3_no_bypass_is_sum_of_independent_layer_updates(P):
    D = tiny_dims()
    _, nl = tiny_layers(P)
    S = [5]
    x = hidden(1, 2)
    kc, vc = _filled_caches(P, 1, D, S)
    expect = x.copy()
    for i in range(P):
        k1, v1 = kc[i:i + 1].copy(), vc[i:i + 1].copy()
        expect += orc.seq_layer(D, nl[i], k1, v1, S, x) - x
    out = orc.group_forward(D, nl, 0, kc, vc, S, x)
    np.testing.assert_allclose(out, expect, rtol=1e-11, atol=1e-12)


def test_I4_bypass_window_saturates_and_counts_transfers():
    for p in range(1, 9):
        for d in range(0, p):
            assert orc.bypass_transfers(p, d) == d * (2 * p - d - 1) // 2   # closed form, Sec.4.3
        assert orc.bypass_transfers(p, p + 3) == orc.bypass_transfers(p, p - 1)
    D = tiny_dims()
    P = 3
    _, nl = tiny_layers(P)
    x = hidden(1, 1)
    outs = []
    for d in (P - 1, P, P + 5):
        kc, vc = _filled_caches(P, 1, D, [4])
        outs.append(orc.group_forward(D, nl, d, kc, vc, [4], x))
    np.testing.assert_array_equal(outs[0], outs[1])
    np.testing.assert_array_equal(outs[0], outs[2])
    kc, vc = _filled_caches(P, 1, D, [4])
    assert np.abs(orc.group_forward(D, nl, 1, kc, vc, [4], x) - outs[0]).max() > 1e-6   # d matters below P-1


def test_I4_window_from_debug_outputs():
    """h_i - x - attn_i must be exactly the sum of the min(d, i) preceding attention outputs."""
    D = tiny_dims()
    P = 4
    _, nl = tiny_layers(P)
    x = hidden(1, 2)
    for d in range(0, P):
        kc, vc = _filled_caches(P, 1, D, [3])
        _, attn, h = orc.group_forward(D, nl, d, kc, vc, [3], x, debug=True)
        for i in range(P):
            expect = x + attn[i]
            for j in range(max(0, i - d), i):
                expect = expect + attn[j]
            np.testing.assert_allclose(h[i], expect, rtol=1e-13, atol=1e-13)


def test_I5_bypass_goes_from_earlier_to_later_layer_only():
    D = tiny_dims()
    _, nl = tiny_layers(2)
    x = hidden(1, 2)
    kc, vc = _filled_caches(2, 1, D, [3])
    _, attn, h = orc.group_forward(D, nl, 1, kc, vc, [3], x, debug=True)
    np.testing.assert_allclose(h[0], x + attn[0], rtol=1e-13)
    np.testing.assert_allclose(h[1] - h[0], attn[1], rtol=1e-9, atol=1e-12)
    nl[1]["wo"] = np.zeros_like(nl[1]["wo"])
    kc, vc = _filled_caches(2, 1, D, [3])
    _, attn, h = orc.group_forward(D, nl, 1, kc, vc, [3], x, debug=True)
    np.testing.assert_array_equal(h[0], h[1])


def test_I6_order_matters_only_with_bypass():
    D = tiny_dims()
    _, nl = tiny_layers(3)
    x = hidden(1, 1)
    perm = [2, 0, 1]

    def run(layers, order, d):
        kc, vc = _filled_caches(3, 1, D, [6])
        kc, vc = np.ascontiguousarray(kc[order]), np.ascontiguousarray(vc[order])
        return orc.group_forward(D, [layers[i] for i in order], d, kc, vc, [6], x)

    np.testing.assert_allclose(run(nl, [0, 1, 2], 0), run(nl, perm, 0), rtol=1e-12, atol=1e-12)
    assert np.abs(run(nl, [0, 1, 2], 1) - run(nl, perm, 1)).max() > 1e-6


@pytest.mark.parametrize("d", [0, 1])
def test_I7_prefill_equals_shorter_prefill_plus_decode(d):
    D = tiny_dims()
    P, T = 2, 7
    _, nl = tiny_layers(P)
    x = hidden(2, T)
    S = [0, 4]
    kcA, vcA = _filled_caches(P, 2, D, S)
    kcB, vcB = kcA.copy(), vcA.copy()
    full = orc.group_forward(D, nl, d, kcA, vcA, S, x)
    head = orc.group_forward(D, nl, d, kcB, vcB, S, x[:, : T - 1])
    tail = orc.group_forward(D, nl, d, kcB, vcB, [s + T - 1 for s in S], x[:, T - 1:])
    np.testing.assert_allclose(full[:, : T - 1], head, rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(full[:, T - 1:], tail, rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(kcA, kcB, rtol=1e-13, atol=0)
    np.testing.assert_allclose(vcA, vcB, rtol=1e-13, atol=0)


def test_batch_of_ragged_sequences_equals_one_call_per_sequence():
    """Batch independence (Eq.2 acts on every sequence alone): a ragged call with B = 3, T = 2 equals three
    B = 1 calls bit for bit, outputs and caches; and against the library composition per sequence, which pins
    the batch term of the cache index and of the input offset to something other than the oracle itself."""
    D = tiny_dims()
    P, T, d = 3, 2, 1
    tl, nl = tiny_layers(P)
    S = [5, 0, 9]
    kc, vc = _filled_caches(P, 3, D, S)
    kc0, vc0 = kc.copy(), vc.copy()
    x = hidden(3, T, seed=41)
    out, attn, _ = orc.group_forward(D, nl, d, kc, vc, S, x, debug=True)
    for b in range(3):
        kb = np.ascontiguousarray(kc0[:, b:b + 1]); vb = np.ascontiguousarray(vc0[:, b:b + 1])
        one, attn1, _ = orc.group_forward(D, nl, d, kb, vb, [S[b]], x[b:b + 1], debug=True)
        np.testing.assert_array_equal(out[b], one[0])
        np.testing.assert_array_equal(attn[:, b], attn1[:, 0])
        np.testing.assert_array_equal(kc[:, b], kb[:, 0])
        np.testing.assert_array_equal(vc[:, b], vb[:, 0])
        # library composition of this sequence alone, from its own past
        xt = torch.from_numpy(x[b])
        for i in range(P):
            a, k_all, _ = torch_attn(tl[i], xt, torch.from_numpy(kc0[i, b, :, :S[b]]), torch.from_numpy(vc0[i, b, :, :S[b]]))
            np.testing.assert_allclose(attn[i, b], a.numpy(), rtol=1e-10, atol=1e-12)
            np.testing.assert_allclose(kc[i, b, :, :S[b] + T], k_all.numpy(), rtol=1e-11, atol=1e-13)
    # sequences are not mixed up: sequence 1's output changes when, and only when, its own input changes
    x2 = x.copy(); x2[1] += 0.5
    out2 = orc.group_forward(D, nl, d, kc0.copy(), vc0.copy(), S, x2)
    np.testing.assert_array_equal(out2[0], out[0]); np.testing.assert_array_equal(out2[2], out[2])
    assert np.abs(out2[1] - out[1]).max() > 1e-3


def test_row_restricted_group_forward_equals_the_rows_of_the_full_call():
    """group_forward_rows (used to sample rows of prefills too long for the oracle to finish): all rows flagged
    is the full call; a subset gives exactly those rows, zeros elsewhere, and the same caches."""
    D = tiny_dims()
    P, T, d = 2, 9, 1
    _, nl = tiny_layers(P)
    S = [3, 0]
    kc, vc = _filled_caches(P, 2, D, S)
    x = hidden(2, T, seed=43)
    kA, vA = kc.copy(), vc.copy()
    full, attn, h = orc.group_forward(D, nl, d, kA, vA, S, x, debug=True)
    kB, vB = kc.copy(), vc.copy()
    allr = orc.group_forward_rows(D, nl, d, kB, vB, S, x, np.ones((2, T), dtype=bool))
    np.testing.assert_array_equal(allr[0], full); np.testing.assert_array_equal(allr[1], attn)
    np.testing.assert_array_equal(allr[2], h)
    rows = np.zeros((2, T), dtype=bool)
    rows[0, 4] = rows[0, 8] = rows[1, 0] = rows[1, 7] = True
    kC, vC = kc.copy(), vc.copy()
    sub, sattn, sh = orc.group_forward_rows(D, nl, d, kC, vC, S, x, rows)
    np.testing.assert_array_equal(sub[rows], full[rows])
    np.testing.assert_array_equal(sattn[:, rows], attn[:, rows])
    np.testing.assert_array_equal(sh[:, rows], h[:, rows])
    assert not sub[~rows].any() and not sattn[:, ~rows].any() and not sh[:, ~rows].any()
    np.testing.assert_array_equal(kC, kA); np.testing.assert_array_equal(vC, vA)


# ----------------------------------------------------------------------------- I9: partition, paper values
def _golden_rows():
    rows = []
    with open(os.path.join(GOLDEN, "partition_examples.txt")) as fh:
        for line in fh:
            line = line.strip()
            if line and not line.startswith("#"):
                rows.append(line.split())
    return rows


def test_I9_partition_matches_the_papers_worked_example_and_tables():
    seen_example = False
    for row in _golden_rows():
        if row[0] == "example":
            L, p, s, e, lead, mid, trail = map(int, row[1:])
            assert orc.partition(L, p, s, e) == [1] * lead + [p] * mid + [1] * trail
            seen_example = True
        else:
            L, p, s, e = map(int, row[1:5])
            printed = float(row[5])
            sizes = orc.partition(L, p, s, e)
            assert sum(sizes) == L and (e - s + 1) % p == 0
            assert sizes == [1] * (s - 1) + [p] * ((e - s + 1) // p) + [1] * (L - e)
            ideal = 100.0 * (1.0 - len(sizes) / L)
            assert printed <= ideal, (row, ideal)
            if row[0] == "table":
                assert ideal < printed + 3.0, (row, ideal)
    assert seen_example


def test_partition_edge_cases():
    assert orc.partition(60, 4, 21, 60) == [1] * 20 + [4] * 10
    assert orc.partition(5, 1, 1, 5) == [1] * 5
    assert orc.partition(7, 3, 2, 6) == [1, 3, 2, 1]          # ragged trailing group
    assert orc.partition(4, 2, 1, 4) == [2, 2]
    with pytest.raises(ValueError):
        orc.partition(4, 2, 0, 4)
    with pytest.raises(ValueError):
        orc.partition(4, 2, 1, 5)


# ----------------------------------------------------------------------------- model level
def test_model_forward_is_the_chain_of_groups_with_embedding_and_head():
    D = tiny_dims()
    Lnum, V = 4, 97
    tl, nl = tiny_layers(Lnum)
    gen = synth.generator(77)
    emb = synth.to_numpy(synth.normal((V, D.d_model), 1.0, torch.float32, gen))
    head = synth.to_numpy(synth.normal((V, D.d_model), 0.05, torch.float32, gen))
    gfin = synth.to_numpy(1.0 + synth.normal((D.d_model,), 0.1, torch.float32, gen))
    tokens = np.array([[5, 96, 0, 31, 5]], dtype=np.int32)
    sizes = orc.partition(Lnum, 2, 1, 4)
    kc, vc = orc.new_cache(Lnum, 1, D), orc.new_cache(Lnum, 1, D)
    res = orc.model_forward(D, nl, sizes, 1, emb, gfin, head, kc, vc, [0], tokens)
    # by hand: embedding rows, two grouped steps, final norm, head, argmax
    x = emb[tokens[0]].astype(np.float64)[None]
    kc2, vc2 = orc.new_cache(Lnum, 1, D), orc.new_cache(Lnum, 1, D)
    x = orc.group_forward(D, nl[0:2], 1, kc2[0:2], vc2[0:2], [0], x)
    x = orc.group_forward(D, nl[2:4], 1, kc2[2:4], vc2[2:4], [0], x)
    np.testing.assert_array_equal(res["hidden"], x)
    logits = head.astype(np.float64) @ orc.rmsnorm(x[0, -1], gfin, D.rms_eps)
    np.testing.assert_allclose(res["logits"][0], logits, rtol=1e-12, atol=1e-13)
    assert res["next"][0] == int(np.argmax(logits))
    np.testing.assert_array_equal(kc, kc2)
    # all-singles partition is the ordinary sequential model
    kc3, vc3 = orc.new_cache(Lnum, 1, D), orc.new_cache(Lnum, 1, D)
    seq = orc.model_forward(D, nl, [1] * Lnum, 1, emb, gfin, head, kc3, vc3, [0], tokens)
    y = emb[tokens[0]].astype(np.float64)[None]
    for i in range(Lnum):
        y = orc.seq_layer(D, nl[i], kc2[i:i + 1] * 0, vc2[i:i + 1] * 0, [0], y)
    np.testing.assert_array_equal(seq["hidden"], y)
    assert np.abs(seq["hidden"] - res["hidden"]).max() > 1e-6    # CQIL is a different function


def test_input_substitution_pins():
    """Sec.3.2: x_{L+1} = x_1 + sum_l F_l(x_l) with the input of one F replaced by an earlier layer's input.
    (i) k = 0 is the plain model bit for bit; (ii) the substituted model written out with the library modules for a
    3-layer model; (iii) when the k layers in between add nothing (zero output projections) the substituted input
    equals the true one and nothing changes; (iv) a real substitution changes the result and the layer's cache."""
    D = tiny_dims()
    Lnum, V = 4, 61
    tl, nl = tiny_layers(Lnum, seed=1301)
    gen = synth.generator(78)
    emb = synth.to_numpy(synth.normal((V, D.d_model), 1.0, torch.float32, gen))
    head = synth.to_numpy(synth.normal((V, D.d_model), 0.05, torch.float32, gen))
    gfin = synth.to_numpy(1.0 + synth.normal((D.d_model,), 0.1, torch.float32, gen))
    tokens = np.array([[7, 3, 60, 0, 12, 7]], dtype=np.int32)
    sizes = [1] * Lnum

    def run(layers, sub_group=-1, sub_k=0, gs=sizes):
        kc, vc = orc.new_cache(Lnum, 1, D), orc.new_cache(Lnum, 1, D)
        return orc.model_forward(D, layers, gs, 0, emb, gfin, head, kc, vc, [0], tokens, sub_group=sub_group, sub_k=sub_k), kc

    plain, kc_plain = run(nl)
    same, kc_same = run(nl, 2, 0)
    np.testing.assert_array_equal(plain["hidden"], same["hidden"]); np.testing.assert_array_equal(kc_plain, kc_same)
    np.testing.assert_array_equal(plain["logits"], same["logits"])
    # (ii) layer 3 (index 2) reads the input of layer 2 (k = 1) / of layer 1 (k = 2), library modules
    x1 = torch.from_numpy(emb[tokens[0]].astype(np.float64))
    empty = torch.zeros(D.n_heads, 0, D.head_dim, dtype=torch.float64)

    def F(i, x):
        a = torch_attn(tl[i], x, empty, empty)[0]
        return a + torch_ffn(tl[i], x + a)

    x2 = x1 + F(0, x1)
    x3 = x2 + F(1, x2)
    for k, src in ((1, x2), (2, x1)):
        x4 = x3 + F(2, src)
        x5 = x4 + F(3, x4)
        got, kc = run(nl, 2, k)
        np.testing.assert_allclose(got["hidden"][0], x5.numpy(), rtol=1e-10, atol=1e-11)
        assert np.abs(got["hidden"] - plain["hidden"]).max() > 1e-4            # (iv)
        assert np.abs(kc[2] - kc_plain[2]).max() > 1e-4 and np.array_equal(kc[:2], kc_plain[:2])
    # (iii) layers 2 and 3 silent: the input of layer 4 equals the inputs of layers 3 and 2
    quiet = [dict(L) for L in nl]
    for i in (1, 2):
        quiet[i]["wo"] = np.zeros_like(quiet[i]["wo"]); quiet[i]["wdown"] = np.zeros_like(quiet[i]["wdown"])
    base, _ = run(quiet)
    for k in (1, 2):
        sub, _ = run(quiet, 3, k)
        np.testing.assert_allclose(sub["hidden"], base["hidden"], rtol=0, atol=1e-12)
    # grouped partitions: a group reads the input of an earlier group
    gsz = [1, 2, 1]
    g_plain, _ = run(nl, gs=gsz)
    g_sub, _ = run(nl, 2, 1, gs=gsz)
    assert np.abs(g_sub["hidden"] - g_plain["hidden"]).max() > 1e-4
    with pytest.raises(RuntimeError):
        run(nl, 1, 2)                      # k reaches before the first layer
    with pytest.raises(RuntimeError):
        run(nl, 4, 1)                      # no such group


def test_argmax_tie_break_is_lowest_index():
    D = tiny_dims()
    _, nl = tiny_layers(1)
    V = 8
    emb = synth.to_numpy(synth.normal((V, D.d_model), 1.0, torch.float32, synth.generator(1)))
    head = np.zeros((V, D.d_model), dtype=np.float32)      # every logit is exactly 0
    gfin = np.ones(D.d_model, dtype=np.float32)
    kc, vc = orc.new_cache(1, 1, D), orc.new_cache(1, 1, D)
    res = orc.model_forward(D, nl, [1], 0, emb, gfin, head, kc, vc, [0], np.array([[3]], dtype=np.int32))
    assert res["next"][0] == 0
