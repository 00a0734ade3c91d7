"""GPU parity at the full sizes of the named workloads, in the launch configurations bench.py times.
Where the oracle cannot finish the whole output in reasonable time it computes sampled outputs one by one
(causality makes a prefix of a prefill independent of the rest), and size-independent properties cover the rest."""
import numpy as np
import pytest
import torch

import oracle as orc
from paper_2404_06709_amd import binding as cq
from paper_2404_06709_amd import runtime as rt
from paper_2404_06709_amd import synth
from parity_util import TOL, Pair, gdims, odims, rel_err, say

pytestmark = pytest.mark.gpu
BF16 = torch.bfloat16


def test_config2_llama7b_group_P4_decode_kv1024():
    """LLaMA-7B-shaped group, bf16, P=4, batch 1, cache of 1024 N(0,1) tokens, one new token per step."""
    pair = Pair(synth.SHAPES["7b"], 4, BF16, max_seq=1040, b_max=1, seed=1002, gen_device="cuda")
    pair.fill_cache([1024], seed=2002, gen_device="cuda")
    for step in range(2):
        pair.step(pair.hidden(1, 1, seed=10 + step), 1, label=f"cfg2 step {step}")
    pair.set_lens([1026])
    pair.step(pair.hidden(1, 1, seed=12), 0, label="cfg2 no bypass")


def test_headline_llama33b_group_P4_decode():
    """The shape the headline metric is quoted on: 33B-shaped group of four, batch 1, cache 576."""
    pair = Pair(synth.SHAPES["33b"], 4, BF16, max_seq=640, b_max=1, seed=1005, gen_device="cuda")
    pair.fill_cache([576], seed=2005, gen_device="cuda")
    pair.step(pair.hidden(1, 1, seed=20), 1, label="33b group")
    pair.step(pair.hidden(1, 1, seed=21), 3, label="33b group d=3")


def test_config3_llama13b_group_P4_batch8_ragged():
    """13B-shaped group, P=4, batch 8, per-sequence cache lengths uniform in [512, 2048]."""
    lens = synth.kv_lengths(8, 512, 2048, seed=1003)
    say(f"  cfg3 cache lengths: {lens.tolist()}")
    pair = Pair(synth.SHAPES["13b"], 4, BF16, max_seq=2056, b_max=8, seed=1003, gen_device="cuda")
    pair.fill_cache(lens.tolist(), seed=2003, gen_device="cuda")
    pair.step(pair.hidden(8, 1, seed=30), 1, label="cfg3")


def test_wide_batch_llama13b_group_P4_batch40():
    """A batch beyond the 32-row tile at full width (the batch sweep's regime): 40 sequences, ragged caches of
    256..700 tokens, one new token each: 128-token tiles, K-split O and down projections, the four-wave attention."""
    B = 40
    lens = synth.kv_lengths(B, 256, 700, seed=1013)
    pair = Pair(synth.SHAPES["13b"], 4, BF16, max_seq=704, b_max=B, seed=1013, gen_device="cuda")
    pair.fill_cache(lens.tolist(), seed=2013, gen_device="cuda")
    pair.step(pair.hidden(B, 1, seed=31), 1, label="13b batch 40")


@pytest.mark.parametrize("B", [128, 256])
def test_batch_sweep_llama13b_group_P4_wide_batches_sampled(B):
    """The wide end of the batch sweep at full 13B width: B = 128 and 256 sequences (several 128-token tiles, the
    four-wave one-query attention), ragged caches of 64..330 tokens, one new token each.  The oracle runs the
    sampled sequences one by one (a sequence's output depends on no other sequence)."""
    shape, P, max_seq = synth.SHAPES["13b"], 4, 336
    lens = synth.kv_lengths(B, 64, 330, seed=1100 + B)
    gd, od = gdims(shape, max_seq, BF16), odims(shape, max_seq, BF16)
    layers = synth.make_layers(P, shape, BF16, seed=1013, device="cuda")
    nl = [synth.layer_to_numpy(L) for L in layers]
    group = rt.Group(gd, layers, b_max=B)
    torch.cuda.synchronize()
    del layers
    gen = synth.generator(2100 + B, "cuda")
    group.k.copy_(synth.normal(tuple(group.k.shape), 1.0, BF16, gen))
    group.v.copy_(synth.normal(tuple(group.v.shape), 1.0, BF16, gen))
    k0, v0 = group.k.clone(), group.v.clone()
    group.set_kv_len(lens.tolist())
    x = synth.normal((B, 1, shape.d_model), 1.0, BF16, gen)
    y = group.forward(x, 1, advance=True)
    torch.cuda.synchronize()
    attn = group.attn_out(B, 1).view(P, B, shape.d_model)
    assert group.kv_len.cpu().tolist() == (lens + 1).tolist()
    sample = sorted({0, 1, 31, 127, B - 129 if B > 129 else 64, B - 1, int(np.argmax(lens)), int(np.argmin(lens))})
    worst = 0.0
    for b in sample:
        S = int(lens[b])
        okc, ovc = orc.new_cache(P, 1, od), orc.new_cache(P, 1, od)
        okc[:, 0, :, :S] = synth.widen(k0[:, b, :, :S]); ovc[:, 0, :, :S] = synth.widen(v0[:, b, :, :S])
        ref, ref_attn, _ = orc.group_forward(od, nl, 1, okc, ovc, [S], synth.widen(x[b:b + 1]), debug=True)
        e = (rel_err(synth.widen(y[b]), ref[0]), rel_err(attn[:, b].cpu().numpy(), ref_attn[:, 0, 0]),
             rel_err(synth.widen(group.k[:, b, :, S]), okc[:, 0, :, S]), rel_err(synth.widen(group.v[:, b, :, S]), ovc[:, 0, :, S]))
        say(f"  B={B} sequence {b} (cache {S}): x_out {e[0]:.2e} attn {e[1]:.2e} k {e[2]:.2e} v {e[3]:.2e}")
        worst = max(worst, *e)
    assert worst <= TOL[BF16]
    # every slot but the appended one of every sequence is untouched
    idx = torch.from_numpy(lens.astype(np.int64)).cuda()
    for cache, before in ((group.k, k0), (group.v, v0)):
        changed = (cache != before).any(dim=-1).any(dim=0).any(dim=1)          # [B, max_seq]
        only = torch.zeros_like(changed)
        only[torch.arange(B, device="cuda"), idx] = True
        assert not (changed & ~only).any()


def test_config4_llama13b_prefill_P2_4x2048_sampled():
    """13B-shaped prefill, P=2, batch 4 x 2048 tokens, causal, empty caches, at full size on the GPU.
    The oracle computes the first 20 positions of two of the sequences (a causal prefix does not depend on
    later tokens); the last position is covered by the any-size property prefill(T) == prefill(T-1) + decode."""
    shape, P, B, T, NPRE = synth.SHAPES["13b"], 2, 4, 2048, 20
    pair = Pair(shape, P, BF16, max_seq=T, b_max=B, seed=1004, gen_device="cuda")
    x = synth.normal((B, T, shape.d_model), 1.0, BF16, synth.generator(3004, "cuda"))
    g = pair.group
    g.set_kv_len([0] * B)
    y = g.forward(x, 1, advance=False)
    torch.cuda.synchronize()
    attn = g.attn_out(B, T).view(P, B, T, shape.d_model)
    say("  cfg4 GPU prefill done")
    for b in (0, 3):
        okc, ovc = orc.new_cache(P, 1, pair.od), orc.new_cache(P, 1, pair.od)
        ref, ref_attn, _ = orc.group_forward(pair.od, pair.np_layers, 1, okc, ovc, [0], synth.widen(x[b:b + 1, :NPRE]),
                                             debug=True)
        e_out = rel_err(synth.widen(y[b, :NPRE]), ref[0])
        e_attn = rel_err(attn[:, b, :NPRE].cpu().numpy(), ref_attn[:, 0])
        e_k = rel_err(synth.widen(g.k[:, b, :, :NPRE]), okc[:, 0, :, :NPRE])
        e_v = rel_err(synth.widen(g.v[:, b, :, :NPRE]), ovc[:, 0, :, :NPRE])
        say(f"  cfg4 sequence {b}, first {NPRE} positions: x_out {e_out:.2e} attn {e_attn:.2e} k {e_k:.2e} v {e_v:.2e}")
        assert max(e_out, e_attn, e_k, e_v) <= TOL[BF16]
    # rows deep inside the chunk (query blocks 1, 7 and the last; later waves of a block; the very last position):
    # the oracle computes the keys and values of the whole sequence and the outputs of the sampled rows only
    b, sample = 1, [130, 131, 1000, 1917, 2047]
    rows = np.zeros((1, T), dtype=bool)
    rows[0, sample] = True
    okc, ovc = orc.new_cache(P, 1, pair.od), orc.new_cache(P, 1, pair.od)
    ref, ref_attn, _ = orc.group_forward_rows(pair.od, pair.np_layers, 1, okc, ovc, [0], synth.widen(x[b:b + 1]), rows)
    e_out = rel_err(synth.widen(y[b, sample]), ref[0, sample])
    e_attn = rel_err(attn[:, b, sample].cpu().numpy(), ref_attn[:, 0, sample])
    e_k = rel_err(synth.widen(g.k[:, b]), okc[:, 0])
    e_v = rel_err(synth.widen(g.v[:, b]), ovc[:, 0])
    say(f"  cfg4 sequence {b}, rows {sample}: x_out {e_out:.2e} attn {e_attn:.2e}; all {T} keys {e_k:.2e} values {e_v:.2e}")
    assert max(e_out, e_attn, e_k, e_v) <= TOL[BF16]
    del okc, ovc
    # any-size property on the GPU: same prefill minus the last token, then one decode step per sequence
    k_full, v_full = g.k.clone(), g.v.clone()
    y_last = y[:, T - 1:].clone()
    g.k.zero_(); g.v.zero_(); g.set_kv_len([0] * B)
    y_head = g.forward(x[:, : T - 1].contiguous(), 1, advance=True)
    y_tail = g.forward(x[:, T - 1:].contiguous(), 1, advance=True)
    torch.cuda.synchronize()
    e1 = rel_err(synth.widen(y_head), synth.widen(y[:, : T - 1]))
    e2 = rel_err(synth.widen(y_tail), synth.widen(y_last))
    e3 = rel_err(synth.widen(g.k[:, :, :, T - 1]), synth.widen(k_full[:, :, :, T - 1]))
    say(f"  cfg4 prefill(T) vs prefill(T-1)+decode: head {e1:.2e} tail {e2:.2e} last key {e3:.2e}")
    assert max(e1, e2, e3) <= TOL[BF16]
    assert g.kv_len.cpu().tolist() == [T] * B


def test_config5_llama33b_shape_reduced_depth_model():
    """33B-shaped model through cqil_model_forward at reduced depth (2 sequential layers + one group of four,
    vocabulary 32000): a 6-token prompt and 3 teacher-forced greedy steps against the oracle.  The full 60-layer
    depth does not fit the oracle's time budget; full-depth self-consistency is the next test."""
    shape, V, max_seq = synth.SHAPES["33b"], 32000, 16
    sizes = cq.cqil_partition(6, 4, 3, 6)
    assert sizes == [1, 1, 4]
    layers = synth.make_layers(6, shape, BF16, seed=1005, device="cuda")
    gen = synth.generator(3005, "cuda")
    emb = synth.normal((V, shape.d_model), 1.0, BF16, gen)
    head = synth.normal((V, shape.d_model), 0.02, BF16, gen)
    gfin = torch.ones(shape.d_model, dtype=BF16, device="cuda")
    gd, od = gdims(shape, max_seq, BF16), odims(shape, max_seq, BF16)
    groups, l0 = [], 0
    for P in sizes:
        groups.append(rt.Group(gd, layers[l0:l0 + P], b_max=1))
        l0 += P
    kv_len = torch.zeros(1, dtype=torch.int32, device="cuda")
    model = cq.Model(gd, sizes, [g.packed for g in groups], [g.k for g in groups], [g.v for g in groups], kv_len, emb,
                     gfin, head)
    nl = [synth.layer_to_numpy(L) for L in layers]
    del layers
    emb_n, head_n, gfin_n = synth.to_numpy(emb), synth.to_numpy(head), synth.to_numpy(gfin)
    okc, ovc = orc.new_cache(6, 1, od), orc.new_cache(6, 1, od)
    tokens = torch.randint(0, V, (1, 6), generator=synth.generator(9)).to(torch.int32)
    olen = 0
    for step in range(4):
        T = tokens.shape[1]
        ws = torch.empty(cq.cqil_model_workspace_bytes(model, 1, T), dtype=torch.uint8, device="cuda")
        logits = torch.empty(1, V, dtype=torch.float32, device="cuda")
        nxt = torch.empty(1, dtype=torch.int32, device="cuda")
        hid = torch.empty(1, T, shape.d_model, dtype=BF16, device="cuda")
        cq.cqil_model_forward(model, tokens.cuda(), 1, T, 1, True, hid, logits, nxt, ws)
        torch.cuda.synchronize()
        ref = orc.model_forward(od, nl, sizes, 1, emb_n, gfin_n, head_n, okc, ovc, [olen], tokens.numpy())
        olen += T
        e_h = rel_err(synth.widen(hid.cpu()), ref["hidden"])
        e_l = rel_err(logits.cpu().numpy(), ref["logits"])
        same = int(nxt.cpu()[0].item() == ref["next"][0])
        say(f"  cfg5 reduced depth, step {step} (T={T}): hidden {e_h:.2e} logits {e_l:.2e} argmax agrees: {same}")
        assert e_h <= TOL[BF16] and e_l <= TOL[BF16]
        tokens = torch.from_numpy(ref["next"].reshape(1, 1).astype(np.int32))


def test_model_forward_full_depth_33b_equals_chain_of_group_calls():
    """Full LLaMA-33B depth on the GPU (60 layers: 20 sequential + 10 groups of four, ~65 GB of weights):
    cqil_model_forward must equal, bit for bit, the chain of cqil_group_forward calls whose parity with the
    oracle the other tests establish.  Prefill of 16 tokens, then 2 decode steps."""
    shape, V, max_seq, L = synth.SHAPES["33b"], 32000, 32, 60
    sizes = cq.cqil_partition(L, 4, 21, 60)
    assert sizes == [1] * 20 + [4] * 10
    gd = gdims(shape, max_seq, BF16)
    gen = synth.generator(1005, "cuda")
    groups = []
    for gi, P in enumerate(sizes):
        layers = [synth.make_layer(shape, BF16, gen) for _ in range(P)]
        groups.append(rt.Group(gd, layers, b_max=1))
        torch.cuda.synchronize()
        del layers
        if gi % 10 == 9:
            say(f"  packed {gi + 1}/{len(sizes)} groups")
    emb = synth.normal((V, shape.d_model), 1.0, BF16, gen)
    head = synth.normal((V, shape.d_model), 0.02, BF16, gen)
    gfin = torch.ones(shape.d_model, dtype=BF16, device="cuda")
    kv_len = torch.zeros(1, dtype=torch.int32, device="cuda")
    model = cq.Model(gd, sizes, [g.packed for g in groups], [g.k for g in groups], [g.v for g in groups], kv_len, emb,
                     gfin, head)
    tokens = torch.randint(0, V, (1, 16), generator=synth.generator(5)).to(torch.int32).cuda()
    n = 0
    for step in range(3):
        T = tokens.shape[1]
        ws = torch.empty(cq.cqil_model_workspace_bytes(model, 1, T), dtype=torch.uint8, device="cuda")
        hid = torch.empty(1, T, shape.d_model, dtype=BF16, device="cuda")
        nxt = torch.empty(1, dtype=torch.int32, device="cuda")
        logits = torch.empty(1, V, dtype=torch.float32, device="cuda")
        k_before = [g.k[:, :, :, n:n + T].clone() for g in groups]
        cq.cqil_model_forward(model, tokens, 1, T, 1, False, hid, logits, nxt, ws)
        k_model = [g.k[:, :, :, n:n + T].clone() for g in groups]
        x = emb[tokens[0].long()].reshape(1, T, -1).contiguous()
        for g, kb in zip(groups, k_before):
            g.k[:, :, :, n:n + T] = kb
            g.set_kv_len([n])
            x = g.forward(x, 1, advance=False)
        torch.cuda.synchronize()
        assert torch.equal(x, hid), f"step {step}: hidden state differs"
        for g, km in zip(groups, k_model):
            assert torch.equal(g.k[:, :, :, n:n + T], km)
        assert torch.isfinite(logits).all() and 0 <= nxt.item() < V
        assert nxt.item() == int(torch.argmax(logits[0]).item())
        n += T
        kv_len.fill_(n)
        model.c.max_kv_len = n
        say(f"  full depth step {step} (T={T}): model loop == chain of group calls; next token {nxt.item()}")
        tokens = nxt.reshape(1, 1).clone()
