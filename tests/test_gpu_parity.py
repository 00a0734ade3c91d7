"""GPU parity: the HIP path (through the C ABI) against the CPU oracle on the same seeded inputs."""
import numpy as np
import pytest
import torch

import oracle as orc
from paper_2404_06709_amd import binding as cq
from paper_2404_06709_amd import runtime as rt
from paper_2404_06709_amd import synth
from parity_util import TOL, Guarded, Pair, gdims, odims, rel_err, say

pytestmark = pytest.mark.gpu

TINY = synth.SHAPES["tiny"]
MID = synth.Shape(512, 4, 128, 1024)        # head_dim 128 like the LLaMA shapes, still small
ODD = synth.Shape(384, 6, 64, 1040)         # d_model not a multiple of 512, d_ffn = 16 * 65
WIDE = synth.Shape(256, 4, 64, 2752)        # P=4 gives a down-projection K of 11008: two K slices


# ------------------------------------------------------------------------------------------ packing
def _pattern_layers(shape, P, dtype):
    """Weights whose bit patterns identify (layer, matrix, row, column)."""
    layers = []
    for l in range(P):
        L = {}
        for m, (name, rows, cols) in enumerate((("wq", shape.d_model, shape.d_model), ("wk", shape.d_model, shape.d_model),
                                                ("wv", shape.d_model, shape.d_model), ("wo", shape.d_model, shape.d_model),
                                                ("wgate", shape.d_ffn, shape.d_model), ("wup", shape.d_ffn, shape.d_model),
                                                ("wdown", shape.d_model, shape.d_ffn), ("g_attn", 1, shape.d_model),
                                                ("g_ffn", 1, shape.d_model))):
            r = torch.arange(rows, dtype=torch.int64)[:, None]
            c = torch.arange(cols, dtype=torch.int64)[None, :]
            if dtype == torch.float32:
                bits = (((l * 9 + m) << 26) + r * cols + c).to(torch.int32)
                t = bits.view(torch.float32)
            else:
                bits = ((r * 131 + c * 7 + m * 9973 + l * 31337) & 0xFFFF).to(torch.int32)
                bits = torch.where(bits >= 32768, bits - 65536, bits).to(torch.int16)
                t = bits.view(torch.bfloat16)
            L[name] = t.reshape(-1) if rows == 1 else t.contiguous()
        layers.append(L)
    return layers


def _bits(t):
    t = t.detach().cpu().contiguous()
    return t.view(torch.int32).numpy() if t.dtype == torch.float32 else t.view(torch.int16).numpy()


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("shape,P", [(TINY, 2), (TINY, 1), (ODD, 3), (MID, 1)])
def test_pack_group_is_a_bit_exact_index_map(shape, P, dtype):
    max_seq = 96
    d = gdims(shape, max_seq, dtype)
    layers = _pattern_layers(shape, P, dtype)
    dev = rt.to_device(layers)
    lay = cq.cqil_packed_layout_of(d, P)
    packed = torch.full((lay.total,), 0xAB, dtype=torch.uint8, device="cuda")
    cq.cqil_pack_group(d, dev, packed)
    torch.cuda.synchronize()
    raw = packed.cpu()
    es = 4 if dtype == torch.float32 else 2
    npdt = np.int32 if dtype == torch.float32 else np.int16
    dm, f = shape.d_model, shape.d_ffn

    def region(off, n):
        return raw[off: off + n * es].numpy().view(npdt)

    src = [{k: _bits(v) for k, v in L.items()} for L in layers]
    V = 16 // es                      # elements per 16-byte piece
    KB = 4 * V                        # columns per tile

    def tiled(mat):
        """[R][K] -> the tiled order: strips of 16 rows, tiles of KB columns, inside a tile [k group][row][element];
        K is padded with zeros to whole tiles."""
        R, K = mat.shape
        Kp = (K + KB - 1) // KB * KB
        pad = np.zeros((R, Kp), dtype=mat.dtype)
        pad[:, :K] = mat
        return pad.reshape(R // 16, 16, Kp // KB, 4, V).transpose(0, 2, 3, 1, 4).reshape(-1)

    exp_qkv = np.concatenate([np.concatenate([s["wq"], s["wk"], s["wv"]], axis=0) for s in src], axis=0)   # N-concat
    np.testing.assert_array_equal(region(lay.wqkv, P * 3 * dm * dm), tiled(exp_qkv))
    exp_wo = np.concatenate([s["wo"] for s in src], axis=1)                                               # K-concat
    np.testing.assert_array_equal(region(lay.wo, P * dm * dm), tiled(exp_wo))
    exp_gu = np.concatenate([np.stack([s["wgate"].reshape(f // 16, 16, dm), s["wup"].reshape(f // 16, 16, dm)],
                                      axis=1).reshape(2 * f, dm) for s in src], axis=0)   # 16 gate rows, 16 up rows, ...
    np.testing.assert_array_equal(region(lay.wgu, P * 2 * f * dm), tiled(exp_gu))
    exp_down = tiled(np.concatenate([s["wdown"] for s in src], axis=1))                                   # K-concat
    down_elems = exp_down.size
    np.testing.assert_array_equal(region(lay.wdown, down_elems), exp_down)
    np.testing.assert_array_equal(region(lay.g_attn, P * dm).reshape(P, dm), np.stack([s["g_attn"] for s in src]))
    np.testing.assert_array_equal(region(lay.g_ffn, P * dm).reshape(P, dm), np.stack([s["g_ffn"] for s in src]))
    # rotary table: (cos, sin)(pos * base^(-2i/d)), fp32 roundings of the double values
    half = shape.head_dim // 2
    table = raw[lay.rope: lay.rope + max_seq * half * 8].numpy().view(np.float32).reshape(max_seq, half, 2)
    phi = np.arange(max_seq)[:, None] * 10000.0 ** (-2.0 * np.arange(half)[None, :] / shape.head_dim)
    np.testing.assert_allclose(table[..., 0], np.cos(phi), atol=1.2e-7, rtol=0)
    np.testing.assert_allclose(table[..., 1], np.sin(phi), atol=1.2e-7, rtol=0)
    # alignment gaps between the parts are not written
    ends = [(lay.wqkv + P * 3 * dm * dm * es, lay.wo), (lay.wo + P * dm * dm * es, lay.wgu),
            (lay.wgu + P * 2 * f * dm * es, lay.wdown), (lay.wdown + down_elems * es, lay.g_attn),
            (lay.g_attn + P * dm * es, lay.g_ffn), (lay.g_ffn + P * dm * es, lay.rope),
            (lay.rope + max_seq * half * 8, lay.total)]
    for a, b in ends:
        assert (raw[a:b] == 0xAB).all()


def test_stream_read_probe_reads_every_chunk_exactly_once():
    """The measurement aid's checksum equals the xor of all 32-bit words of the buffer (each 16-byte chunk read once,
    none beyond the end), for sizes around the kernel's stride and unroll."""
    gen = synth.generator(77)
    for n_chunks in (1, 255, 2047, 2049, 4096 * 2048 - 1, 4096 * 2048 + 13):
        words = torch.randint(-2 ** 31, 2 ** 31 - 1, (n_chunks * 4 + 8,), generator=gen, dtype=torch.int64).to(torch.int32)
        buf = words.cuda()
        sink = torch.zeros(4096, dtype=torch.int32, device="cuda")
        cq.cqil_stream_read_probe(buf[: n_chunks * 4], sink)
        torch.cuda.synchronize()
        got = np.bitwise_xor.reduce(sink.cpu().numpy().view(np.uint32))
        exp = np.bitwise_xor.reduce(words.numpy()[: n_chunks * 4].view(np.uint32))
        assert got == exp, f"{n_chunks} chunks"


# ------------------------------------------------------------------------------------------ Sec.3.1 tooling
@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_input_similarity_of_captured_layer_inputs(dtype):
    """Layer inputs captured from a chain of single-layer steps on the GPU (the inputs x_1..x_L and the final
    state), compared with the oracle's similarity matrix of the same captured tensors; deterministic."""
    L, T = 5, 37
    pairs = [Pair(TINY, 1, dtype, max_seq=64, b_max=1, seed=600 + i, w_std=0.05, gain_jitter=0.1) for i in range(L)]
    x = pairs[0].hidden(1, T, seed=5).cuda()
    states = [x]
    for p in pairs:
        p.group.set_kv_len([0])
        x = p.group.forward(x, 0, advance=False)
        states.append(x)
    X = torch.stack([s_[0] for s_ in states]).contiguous()          # [L+1, T, d_model]
    sim = cq.cqil_input_similarity(X)
    again = cq.cqil_input_similarity(X)
    torch.cuda.synchronize()
    assert torch.equal(sim, again)
    ref = orc.input_similarity(synth.widen(X.cpu()))
    got = sim.cpu().numpy()
    say(f"  similarity {dtype}: adjacent layers {np.diag(ref, 1).round(4).tolist()}")
    assert np.abs(got - ref).max() <= 1e-5                            # cosines are O(1); fp32 sums of the stored values
    np.testing.assert_array_equal(got, got.T)
    assert np.all(np.diag(ref, 1) < 0.99999), "the captured states are too alike to test anything"
    # many tokens and a width that is not a multiple of a wave's stride: several chunks, ragged tail
    Y = synth.normal((3, 1001, 200), 1.0, dtype, synth.generator(6)).cuda()
    assert np.abs(cq.cqil_input_similarity(Y).cpu().numpy() - orc.input_similarity(synth.widen(Y.cpu()))).max() <= 1e-5


# ------------------------------------------------------------------------------------------ LoRA merge
@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_merge_lora_matches_oracle_and_feeds_the_group(dtype):
    """W + Bm A at rank 1, 8 and 64 on a non-square matrix (one rounding to the storage type: at most one unit in
    the last place from the oracle's rounded double sum), then a group step on merged weights against the oracle
    run on its own merged weights."""
    gen = synth.generator(71)
    for r in (1, 8, 64):
        W = synth.normal((48, 104), 0.05, dtype, gen)
        A = synth.normal((r, 104), 0.2, dtype, gen)
        Bm = synth.normal((48, r), 0.2, dtype, gen)
        ref = orc.merge_lora(synth.to_numpy(W), synth.to_numpy(A), synth.to_numpy(Bm), 1.0)
        Wg = W.cuda().clone()
        cq.cqil_merge_lora(Wg, A.cuda(), Bm.cuda(), 1.0)
        got = synth.widen(Wg.cpu())
        # rounding bound: one storage rounding of the result plus fp32 roundings of the terms (which may cancel)
        ulp = 2.0 ** -8 if dtype == torch.bfloat16 else 2.0 ** -23
        terms = np.abs(synth.widen(W)) + np.abs(synth.widen(Bm)) @ np.abs(synth.widen(A))
        assert np.all(np.abs(got - ref) <= ulp * np.abs(ref) + 2.0 ** -22 * terms), f"rank {r}"
        assert np.abs(got - synth.widen(W)).max() > 1e-3                 # the adapter did change the matrix
    # a whole group: adapters on all seven matrices of two layers
    P, shape = 2, TINY
    layers = synth.make_layers(P, shape, dtype, 7100, w_std=0.05, gain_jitter=0.1)
    merged_gpu, merged_np = [], []
    for L in layers:
        Lg = {k: v.cuda().clone() for k, v in L.items()}
        Ln = dict(synth.layer_to_numpy(L))
        for name in ("wq", "wk", "wv", "wo", "wgate", "wup", "wdown"):
            n_out, n_in = L[name].shape
            A = synth.normal((8, n_in), 0.1, dtype, gen)
            Bm = synth.normal((n_out, 8), 0.1, dtype, gen)
            cq.cqil_merge_lora(Lg[name], A.cuda(), Bm.cuda(), 1.0)
            m64 = orc.merge_lora(Ln[name], synth.to_numpy(A), synth.to_numpy(Bm), 1.0)
            Ln[name] = synth.to_numpy(torch.from_numpy(m64).to(dtype))       # the oracle's own rounding
        merged_gpu.append(Lg); merged_np.append(Ln)
    gd, od = gdims(shape, 64, dtype), odims(shape, 64, dtype)
    group = rt.Group(gd, merged_gpu, b_max=1)
    x = synth.normal((1, 6, shape.d_model), 1.0, dtype, synth.generator(72))
    group.set_kv_len([0])
    y = group.forward(x.cuda(), 1)
    okc, ovc = orc.new_cache(P, 1, od), orc.new_cache(P, 1, od)
    ref = orc.group_forward(od, merged_np, 1, okc, ovc, [0], synth.widen(x))
    # the two sides round a few merged weights differently (ties); that is inside the step tolerance
    assert rel_err(synth.widen(y.cpu()), ref) <= TOL[dtype]


# ------------------------------------------------------------------------------------------ decode, one token
@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("shape", [TINY, MID, ODD, WIDE])
def test_decode_step_matches_oracle(shape, dtype):
    """Single-token decode (the bandwidth-bound path) over cache lengths that straddle the split-KV chunk
    boundaries, group sizes 1..4 and every bypass distance."""
    for P, ds in ((1, (0, 2)), (2, (0, 1)), (4, (0, 1, 2, 3, 7))):
        pair = Pair(shape, P, dtype, max_seq=400, b_max=1, seed=1001 + P, w_std=0.05, gain_jitter=0.1)
        for S in (0, 1, 127, 128, 129, 390):
            pair.okc[:] = 0; pair.ovc[:] = 0
            pair.group.k.zero_(); pair.group.v.zero_()
            pair.fill_cache([S], seed=50 + S)
            for i, d in enumerate(ds):
                pair.set_lens([S])
                pair.step(pair.hidden(1, 1, seed=7 + i), d, label=f"decode {dtype} P={P} S={S}")


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("P", [3, 8])
def test_every_bypass_distance_decode_and_prefill(P, dtype):
    """Sec.4.3 / Eq.4 for d = 0 .. P-1 (and one value beyond, which acts as P-1), group sizes 3 and 8, on both
    the single-token kernels and the token-parallel ones."""
    pair = Pair(TINY, P, dtype, max_seq=160, b_max=2, seed=2000 + P, w_std=0.05, gain_jitter=0.1)
    pair.fill_cache([40, 3], seed=12)
    for d in list(range(P)) + [P + 2]:
        pair.step(pair.hidden(1, 1, seed=10 + d), d, label=f"P={P} d={d} decode {dtype}")
        pair.step(pair.hidden(2, 3, seed=30 + d), d, label=f"P={P} d={d} prefill {dtype}")
    # a distance beyond the group equals the largest one: same state, same input
    x = pair.hidden(1, 1, seed=99).cuda()
    lens = pair.lens[:1].tolist()
    pair.group.set_kv_len(lens); a = pair.group.forward(x, P - 1, advance=False).clone()
    pair.group.set_kv_len(lens); b = pair.group.forward(x, P + 5, advance=False).clone()
    assert torch.equal(a, b)


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("head_dim", [32, 256])
def test_smallest_and_largest_head_sizes(head_dim, dtype):
    """Head sizes at both ends of what the attention kernels take (4 and 32 lanes per cache slot for bf16 heads of
    32 and 256; 8 and 64 lanes for fp32 heads of 32 and 256): single-token decode, a batch of decode rows and a short
    prefill."""
    shape = synth.Shape(4 * head_dim, 4, head_dim, 16 * 24)
    pair = Pair(shape, 2, dtype, max_seq=200, b_max=3, seed=2200 + head_dim, w_std=0.05, gain_jitter=0.1)
    pair.fill_cache([150, 0, 37], seed=14)
    pair.step(pair.hidden(1, 1, seed=1), 1, label=f"d_k={head_dim} decode {dtype}")
    pair.step(pair.hidden(3, 1, seed=2), 1, label=f"d_k={head_dim} batch of 3 {dtype}")
    pair.step(pair.hidden(2, 5, seed=3), 0, label=f"d_k={head_dim} prefill {dtype}")


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_group_wider_than_eight_layers(dtype):
    """Ten layers in one group: beyond the eight whose attention outputs the bypass kernel keeps in registers, so
    the general kernel of the token-parallel path (and the decode kernels at P = 10) are the ones checked."""
    P = 10
    pair = Pair(TINY, P, dtype, max_seq=96, b_max=2, seed=2100, w_std=0.05, gain_jitter=0.1)
    pair.fill_cache([20, 5], seed=13)
    for d in (0, 3, P - 1):
        pair.step(pair.hidden(1, 1, seed=50 + d), d, label=f"P={P} d={d} decode {dtype}")
        pair.step(pair.hidden(2, 3, seed=60 + d), d, label=f"P={P} d={d} prefill {dtype}")


def test_decode_is_deterministic_and_in_place():
    pair = Pair(TINY, 4, torch.float32, max_seq=300, b_max=1, seed=5, w_std=0.05, gain_jitter=0.1)
    pair.fill_cache([260], seed=9)
    x = pair.hidden(1, 1, seed=3).cuda()
    outs = []
    for _ in range(3):
        pair.set_lens([260])
        outs.append(pair.group.forward(x, 1, advance=False).clone())
    buf = x.clone()
    pair.group.forward(buf, 1, advance=False, out=buf)          # x_out aliases x_in
    torch.cuda.synchronize()
    assert torch.equal(outs[0], outs[1]) and torch.equal(outs[0], outs[2]) and torch.equal(outs[0], buf)
    assert pair.group.kv_len.cpu()[0].item() == 260             # advance=False leaves the length alone


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_group_steps_replay_from_a_hip_graph(dtype):
    """The library only launches kernels on the caller's stream (no allocation, no synchronisation, no memset):
    a prefill chunk and four decode steps captured into one graph replay bit for bit, three times, with eager
    work and synchronisation between the replays."""
    P, S0 = 2, 20
    pair = Pair(MID, P, dtype, max_seq=64, b_max=1, seed=31, w_std=0.05, gain_jitter=0.1)
    pair.fill_cache([S0], seed=4)
    g = pair.group
    k0, v0 = g.k.clone(), g.v.clone()
    xp = pair.hidden(1, 3, seed=1).cuda()
    xs = [pair.hidden(1, 1, seed=2 + i).cuda() for i in range(4)]

    def run(outs):
        g.forward(xp, 1, advance=True, out=outs[0])
        for i in range(4):
            g.forward(xs[i], 1, advance=True, out=outs[1 + i])

    def reset():
        g.k.copy_(k0); g.v.copy_(v0)
        g.set_kv_len([S0]); g.kv.max_kv_len = S0

    eager = [torch.empty_like(xp)] + [torch.empty_like(x) for x in xs]
    reset(); run(eager)                                   # also sizes the workspaces before the capture
    torch.cuda.synchronize()
    k_e = g.k.clone()
    outs = [torch.empty_like(t) for t in eager]
    reset()
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        run(outs)
    for rep in range(3):
        for t in outs:
            t.fill_(float("nan"))
        reset()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for a, b in zip(outs, eager):
            assert torch.equal(a, b), f"replay {rep}"
        assert torch.equal(g.k, k_e) and g.kv_len.cpu()[0].item() == S0 + 7


# ------------------------------------------------------------------------------------------ launch-shape knobs
KNOBS = [("ksplit_qkv", 1), ("ksplit_qkv", 2), ("ksplit_qkv", 8), ("ksplit_o", 1), ("ksplit_o", 2), ("ksplit_o", 4),
         ("ksplit_o", 8), ("ksplit_gu", 1), ("ksplit_gu", 2), ("ksplit_gu", 4), ("ksplit_gu", 8), ("ksplit_d", 1),
         ("ksplit_d", 2), ("ksplit_d", 4), ("ksplit_d", 8), ("down_slice_max", 512), ("down_slice_max", 2048),
         ("down_slice_max", 12288)]


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_every_decode_launch_shape_knob_matches_oracle(dtype):
    """cqil_set_tuning selects other k splits of the four single-token projections and other K-slice lengths of the
    down projection: every value that changes a launch is run against the oracle (WIDE at P = 4 has a
    concatenated K of 11008: 22, 6 and 1 slices), with the knobs put back afterwards."""
    try:
        for shape, P in ((WIDE, 4), (MID, 1)):
            pair = Pair(shape, P, dtype, max_seq=160, b_max=1, seed=3100 + P, w_std=0.05, gain_jitter=0.1)
            pair.fill_cache([130], seed=21)
            for i, (key, val) in enumerate(KNOBS):
                cq.reset_tuning()
                cq.cqil_set_tuning(key, val)
                pair.set_lens([130])
                pair.step(pair.hidden(1, 1, seed=40 + i), 1, label=f"{key}={val} P={P} {dtype}")
    finally:
        cq.reset_tuning()


@pytest.mark.parametrize("tile", [1, 2])
def test_gemm_tile_knob_matches_oracle(tile):
    """gemm_tile 1 = the 8-wave 256 x 256 instantiation of the matrix-core GEMM (M > 32 rows), 2 = the tiled
    kernel also for up to 8 rows (where the default is the barrier-free streaming kernel)."""
    try:
        cq.cqil_set_tuning("gemm_tile", tile)
        pair = Pair(MID, 2, torch.bfloat16, max_seq=400, b_max=8, seed=3200 + tile, w_std=0.05, gain_jitter=0.1)
        pair.fill_cache([0, 70, 3, 128, 9, 31, 200, 64], seed=22)
        pair.step(pair.hidden(2, 150, seed=1), 1, label=f"gemm_tile={tile} 300 rows")     # ragged second tile
        pair.step(pair.hidden(8, 1, seed=2), 1, label=f"gemm_tile={tile} 8 rows")
        pair.step(pair.hidden(3, 1, seed=3), 0, label=f"gemm_tile={tile} 3 rows")
        pair.step(pair.hidden(1, 40, seed=4), 1, label=f"gemm_tile={tile} 40 rows")
    finally:
        cq.reset_tuning()


# ------------------------------------------------------------------------------------------ branch-dominated inputs
@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("shape,P", [(TINY, 2), (MID, 4)])
def test_small_hidden_states_let_the_branches_dominate(shape, P, dtype):
    """Hidden states N(0, 0.05): RMSNorm makes the attention and feed-forward branches independent of the
    input's scale, so they are 10-20 times larger than x here and an error of either branch shows in x_out at
    full size (with x ~ N(0,1) it would hide behind x)."""
    pair = Pair(shape, P, dtype, max_seq=200, b_max=12, seed=3300 + P, w_std=0.05, gain_jitter=0.1)
    pair.fill_cache([9, 0, 130, 4, 77, 1, 33, 64, 12, 100, 2, 50], seed=23)
    for (B, T, d, seed) in ((1, 1, 1, 1), (3, 5, 1, 2), (12, 1, 0, 3), (1, 1, P - 1, 4), (2, 40, 1, 5)):
        x = pair.hidden(B, T, seed=seed, std=0.05)
        y, ref = pair.step(x, d, label=f"small x {dtype} P={P}")
        assert np.abs(ref - synth.widen(x)).max() > 5 * np.abs(synth.widen(x)).max()


# ------------------------------------------------------------------------------------------ prefill / batch
@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("shape", [MID, ODD, TINY])
def test_prefill_over_several_query_blocks_and_ragged_caches(shape, dtype):
    """Chunks of 300 tokens onto caches of 0 and 70 tokens: three 128-query blocks per head (the last ragged),
    waves whose first query lies beyond several unmasked key tiles, the longest-first block order, and a
    non-empty cache under several query blocks; head sizes 128 (MID) and 64 (ODD, TINY).  600 token rows: for bf16
    MID and TINY (widths that are multiples of 256) the rotary embedding and the KV append run in the epilogue of the
    QKV product, with both row-to-wave maps (head sizes 128 and 64); ODD keeps the separate pass.  Every position
    is compared."""
    pair = Pair(shape, 2, dtype, max_seq=400, b_max=2, seed=3400, w_std=0.05, gain_jitter=0.1)
    try:
        for form in ((0, 1) if dtype == torch.bfloat16 else (0,)):     # both matrix-core attention kernels
            cq.cqil_set_tuning("attn_prefill", form)
            pair.okc[:] = 0; pair.ovc[:] = 0
            pair.group.k.zero_(); pair.group.v.zero_()
            pair.fill_cache([0, 70], seed=24)
            pair.step(pair.hidden(2, 300, seed=1), 1, label=f"prefill 2 x 300 {dtype} form {form}")
            pair.set_lens([0, 70])
            pair.step(pair.hidden(1, 257, seed=2), 0, label=f"prefill 1 x 257 {dtype} form {form}")   # one query past two blocks
            pair.set_lens([0, 70])
            pair.step(pair.hidden(2, 64, seed=3), 1, label=f"prefill 2 x 64 {dtype} form {form}")     # half a query block
    finally:
        cq.reset_tuning()


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("shape", [TINY, ODD])
def test_token_parallel_path_matches_oracle(shape, dtype):
    pair = Pair(shape, 3, dtype, max_seq=200, b_max=4, seed=77, w_std=0.05, gain_jitter=0.1)
    pair.fill_cache([0, 7, 130], seed=5)
    pair.step(pair.hidden(3, 5, seed=1), 1, label=f"prefill {dtype}")      # ragged lengths, T > 1
    pair.step(pair.hidden(3, 1, seed=2), 2, label=f"batched decode {dtype}")
    pair.step(pair.hidden(1, 67, seed=3), 0, label=f"long chunk {dtype}")  # more than one 64-row tile, ragged


@pytest.mark.parametrize("shape,P", [(MID, 1), (MID, 4), (synth.Shape(256, 4, 64, 2752), 2), (synth.Shape(1024, 8, 128, 2816), 3)])
def test_small_batch_decode_matches_oracle(shape, P):
    """bf16, 2..8 token rows per call (token-parallel kernels with few rows; K-split projections)."""
    pair = Pair(shape, P, torch.bfloat16, max_seq=300, b_max=8, seed=900 + P, w_std=0.05, gain_jitter=0.1)
    pair.fill_cache([0, 3, 127, 128, 200, 64, 1, 250], seed=6)
    pair.step(pair.hidden(8, 1, seed=1), 1, label="batch 8")
    pair.step(pair.hidden(2, 1, seed=2), 0, label="batch 2")
    pair.step(pair.hidden(3, 1, seed=3), P - 1, label="batch 3")
    pair.step(pair.hidden(2, 3, seed=4), 1, label="2 sequences x 3 new tokens")
    pair.step(pair.hidden(1, 8, seed=5), 2, label="8-token chunk")
    pair.step(pair.hidden(5, 1, seed=6), 1, label="batch 5")


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("shape,P", [(MID, 2), (synth.Shape(1024, 8, 128, 2816), 3)])
def test_wide_batch_decode_matches_oracle(shape, P, dtype):
    """More than 8 sequences, one new token each: token-parallel projections (split along K when the tile grid is
    small) with the streaming attention kernel reading its queries from the QKV rows."""
    B = 12
    pair = Pair(shape, P, dtype, max_seq=300, b_max=B, seed=1200 + P, w_std=0.05, gain_jitter=0.1)
    pair.fill_cache([0, 3, 127, 128, 200, 64, 1, 250, 17, 90, 255, 31], seed=8)
    pair.step(pair.hidden(B, 1, seed=1), 1, label=f"batch {B} {dtype}")
    pair.step(pair.hidden(B, 1, seed=2), 0, label=f"batch {B} second step {dtype}")
    pair.step(pair.hidden(9, 1, seed=3), P - 1, label=f"batch 9 {dtype}")


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("shape,P", [(TINY, 1), (MID, 3)])
def test_attention_ffn_parallel_form_matches_oracle(shape, P, dtype):
    """App. A, Eq.5 (bypass_d = -1): every feed-forward module reads the shared input itself.  Decode steps,
    a prefill chunk and a batch of decode rows; and the result must be told apart from Eq.3's."""
    d = cq.CQIL_ATTN_FFN_PARALLEL
    pair = Pair(shape, P, dtype, max_seq=200, b_max=10, seed=500 + P, w_std=0.05, gain_jitter=0.1)
    pair.fill_cache([9, 0, 130, 4, 77, 1, 33, 64, 12, 100], seed=9)
    pair.step(pair.hidden(1, 1, seed=1), d, label=f"Eq.5 decode {dtype}")
    pair.step(pair.hidden(3, 5, seed=2), d, label=f"Eq.5 prefill {dtype}")
    pair.step(pair.hidden(10, 1, seed=3), d, label=f"Eq.5 batch of rows {dtype}")
    # discrimination: on the same state, Eq.3 (d = 0) gives a visibly different answer
    x = pair.hidden(1, 1, seed=4)
    lens = pair.lens[:1].copy()
    okc, ovc = pair.okc.copy(), pair.ovc.copy()
    eq5 = orc.group_forward(pair.od, pair.np_layers, d, okc, ovc, lens, synth.widen(x))
    eq3 = orc.group_forward(pair.od, pair.np_layers, 0, pair.okc.copy(), pair.ovc.copy(), lens, synth.widen(x))
    y, _ = pair.step(x, d, label=f"Eq.5 decode again {dtype}")
    assert rel_err(eq3, eq5) > 4 * TOL[dtype], "the test inputs do not separate Eq.5 from Eq.3"
    assert rel_err(synth.widen(y), eq5) <= TOL[dtype] < rel_err(synth.widen(y), eq3)


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("shape,P", [(TINY, 1), (MID, 3), (WIDE, 4)])
def test_eq5_fused_schedule_matches_oracle_and_the_six_kernel_schedule(shape, P, dtype):
    """App. A, Eq.5 on the single-token path: the default schedule runs QKV + gate/up as one shared-input launch and
    O + down as one K-concatenated launch (WIDE at P = 4: four layer segments of Wo and two slices of Wdown).  Against
    the oracle, and bit for bit against the six-kernel schedule; also with k splits that give the two parts of a
    fused launch different numbers of workgroups."""
    d = cq.CQIL_ATTN_FFN_PARALLEL
    pair = Pair(shape, P, dtype, max_seq=200, b_max=1, seed=5400 + P, w_std=0.05, gain_jitter=0.1)
    pair.fill_cache([131], seed=19)
    try:
        for knobs in ({}, {"ksplit_o": 1, "ksplit_d": 8, "ksplit_qkv": 8, "ksplit_gu": 1},
                      {"ksplit_o": 8, "ksplit_d": 1, "ksplit_qkv": 1, "ksplit_gu": 8, "down_slice_max": 512}):
            outs = []
            for fused in (1, 0):
                cq.reset_tuning()
                for kk, vv in knobs.items():
                    cq.cqil_set_tuning(kk, vv)
                cq.cqil_set_tuning("eq5_fused", fused)
                pair.set_lens([131])
                y, _ = pair.step(pair.hidden(1, 1, seed=5), d, label=f"Eq.5 fused={fused} {knobs} P={P} {dtype}")
                outs.append((y, pair.group.k[:, 0, :, 131].clone(), pair.group.v[:, 0, :, 131].clone()))
            assert torch.equal(outs[0][0].view(torch.uint8), outs[1][0].view(torch.uint8))
            assert torch.equal(outs[0][1], outs[1][1]) and torch.equal(outs[0][2], outs[1][2])
    finally:
        cq.reset_tuning()


def test_prefill_then_decode_equals_one_prefill():
    """Property that holds at any size: prefilling T tokens equals prefilling T-1 and decoding one."""
    pair = Pair(TINY, 2, torch.float32, max_seq=64, b_max=1, seed=11, w_std=0.05, gain_jitter=0.1)
    x = pair.hidden(1, 9, seed=4)
    g = pair.group
    g.set_kv_len([0])
    full = g.forward(x.cuda(), 1).cpu()
    k_full = g.k.clone()
    g.k.zero_(); g.v.zero_(); g.set_kv_len([0])
    head = g.forward(x[:, :8].cuda(), 1).cpu()
    tail = g.forward(x[:, 8:].cuda(), 1).cpu()
    assert rel_err(head.numpy(), full[:, :8].numpy()) < 1e-5
    assert rel_err(tail.numpy(), full[:, 8:].numpy()) < 1e-5
    assert rel_err(g.k.cpu().numpy(), k_full.cpu().numpy()) < 1e-5


# ------------------------------------------------------------------------------------------ configuration 1
@pytest.mark.parametrize("d", [0, 1])
def test_config1_tiny_two_groups_prefill_32_then_16_decode_steps(d):
    """Tiny fp32 decoder, 4 layers as 2 groups of P=2, weights N(0,0.02), gains 1: a 32-token prefill of
    N(0,1) hidden states, then 16 decode steps; each side chains its own two groups."""
    dtype = torch.float32
    pairs = [Pair(TINY, 2, dtype, max_seq=64, b_max=1, seed=1001 + g) for g in range(2)]
    gen = synth.generator(4242)
    worst = 0.0
    for step in range(17):
        T = 32 if step == 0 else 1
        x = synth.normal((1, T, TINY.d_model), 1.0, dtype, gen)
        y_gpu, y_ref = x, synth.widen(x)
        # teacher forcing between the groups: the second group of both sides reads the oracle's state
        # rounded to the storage type, so that an error of group 1 is not judged twice
        y_gpu, y_ref = pairs[0].step(x, d, label=f"cfg1 step {step} group 0")
        x2 = torch.from_numpy(y_ref).to(dtype)
        y_gpu2, y_ref2 = pairs[1].step(x2, d, label=f"cfg1 step {step} group 1")
        worst = max(worst, rel_err(synth.widen(y_gpu2), y_ref2))
    assert worst <= TOL[dtype]


def _tiny_model(dtype, group_sizes, vocab, max_seq, seed, w_std=0.05):
    L = sum(group_sizes)
    layers = synth.make_layers(L, TINY, dtype, seed, w_std=w_std, gain_jitter=0.1)
    gen = synth.generator(seed + 1)
    emb = synth.normal((vocab, TINY.d_model), 1.0, dtype, gen)
    head = synth.normal((vocab, TINY.d_model), 0.05, dtype, gen)
    gfin = (1.0 + synth.normal((TINY.d_model,), 0.1, torch.float32, gen)).to(dtype)
    gd = gdims(TINY, max_seq, dtype)
    groups, l0 = [], 0
    for P in group_sizes:
        groups.append(rt.Group(gd, rt.to_device(layers[l0:l0 + P]), b_max=1))
        l0 += P
    kv_len = torch.zeros(1, dtype=torch.int32, device="cuda")
    model = cq.Model(gd, group_sizes, [g.packed for g in groups], [g.k for g in groups], [g.v for g in groups], kv_len,
                     emb.cuda(), gfin.cuda(), head.cuda())
    np_layers = [synth.layer_to_numpy(x) for x in layers]
    return model, groups, kv_len, np_layers, synth.to_numpy(emb), synth.to_numpy(gfin), synth.to_numpy(head)


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_model_forward_teacher_forced(dtype):
    """cqil_model_forward on a tiny 6-layer model, partition (p=2, s=2, e=5): prefill 12 tokens, then
    8 greedy steps fed with the ORACLE's tokens; logits compared at every step."""
    vocab, max_seq = 1003, 48
    sizes = cq.cqil_partition(6, 2, 2, 5)
    assert sizes == [1, 2, 2, 1]
    model, groups, kv_len, nl, emb, gfin, head = _tiny_model(dtype, sizes, vocab, max_seq, seed=300)
    od = odims(TINY, max_seq, dtype)
    okc, ovc = orc.new_cache(6, 1, od), orc.new_cache(6, 1, od)
    tokens = torch.randint(0, vocab, (1, 12), generator=synth.generator(8)).to(torch.int32)
    olen = 0
    agree = 0
    for step in range(9):
        T = tokens.shape[1]
        # every output and the workspace between sentinel bands
        gws = Guarded(cq.cqil_model_workspace_bytes(model, 1, T))
        glog, gnxt = Guarded(vocab * 4), Guarded(16)
        ghid = Guarded(T * TINY.d_model * (4 if dtype == torch.float32 else 2))
        ws = gws.body
        logits = glog.view(torch.float32, (1, vocab))
        nxt = gnxt.body[:4].view(torch.int32)
        hid = ghid.view(dtype, (1, T, TINY.d_model))
        cq.cqil_model_forward(model, tokens.cuda(), 1, T, 1, True, hid, logits, nxt, ws)
        torch.cuda.synchronize()
        ref = orc.model_forward(od, nl, sizes, 1, emb, gfin, head, okc, ovc, [olen], tokens.numpy())
        olen += T
        e_h = rel_err(synth.widen(hid.cpu()), ref["hidden"])
        e_l = rel_err(logits.cpu().numpy(), ref["logits"])
        say(f"  model {dtype} step {step}: hidden {e_h:.2e} logits {e_l:.2e}")
        assert e_h <= TOL[dtype] and e_l <= TOL[dtype]
        glog.check(f"model {dtype} step {step}: logits"); gnxt.check(f"model {dtype} step {step}: next token")
        ghid.check(f"model {dtype} step {step}: hidden state"); gws.check(f"model {dtype} step {step}: workspace")
        top2 = np.sort(ref["logits"][0])[-2:]
        if top2[1] - top2[0] > 8 * TOL[dtype] * np.abs(ref["logits"]).max():
            assert nxt.cpu()[0].item() == ref["next"][0]
        agree += int(nxt.cpu()[0].item() == ref["next"][0])
        assert kv_len.cpu()[0].item() == olen and model.c.max_kv_len == olen
        tokens = torch.from_numpy(ref["next"].reshape(1, 1).astype(np.int32))
    say(f"  greedy tokens agreeing with the oracle: {agree}/9")


@pytest.mark.parametrize("L,p,s,e", [(7, 3, 2, 6), (9, 4, 1, 9), (5, 8, 2, 4)])
def test_model_forward_general_partitions(L, p, s, e):
    """Sec.4.2 partitions with a ragged trailing group, a group at the very bottom and top, and p larger than
    the grouped range: prefill and two decode steps against the oracle, fp32."""
    dtype, vocab, max_seq = torch.float32, 211, 24
    sizes = cq.cqil_partition(L, p, s, e)
    assert sizes == orc.partition(L, p, s, e) and sum(sizes) == L
    model, groups, kv_len, nl, emb, gfin, head = _tiny_model(dtype, sizes, vocab, max_seq, seed=4000 + L)
    od = odims(TINY, max_seq, dtype)
    okc, ovc = orc.new_cache(L, 1, od), orc.new_cache(L, 1, od)
    tokens = torch.randint(0, vocab, (1, 7), generator=synth.generator(3)).to(torch.int32)
    olen = 0
    for step in range(3):
        T = tokens.shape[1]
        ws = torch.empty(cq.cqil_model_workspace_bytes(model, 1, T), dtype=torch.uint8, device="cuda")
        logits = torch.empty(1, vocab, dtype=torch.float32, device="cuda")
        hid = torch.empty(1, T, TINY.d_model, dtype=dtype, device="cuda")
        cq.cqil_model_forward(model, tokens.cuda(), 1, T, 2, True, hid, logits, None, ws)
        torch.cuda.synchronize()
        ref = orc.model_forward(od, nl, sizes, 2, emb, gfin, head, okc, ovc, [olen], tokens.numpy())
        olen += T
        e_h = rel_err(synth.widen(hid.cpu()), ref["hidden"])
        e_l = rel_err(logits.cpu().numpy(), ref["logits"])
        say(f"  partition {sizes} step {step}: hidden {e_h:.2e} logits {e_l:.2e}")
        assert e_h <= TOL[dtype] and e_l <= TOL[dtype]
        tokens = torch.from_numpy(ref["next"].reshape(1, 1).astype(np.int32))


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_model_forward_with_input_substitution(dtype):
    """Sec.3.2 through cqil_model_forward_substituted: a 5-layer model of single layers (the paper's experiment) with
    layer 4 reading the input of layers 3 / 2 / 1, and a grouped partition with a group reading an earlier group's
    input; an 11-token prompt (token-parallel kernels) and two single-token steps (decode kernels), hidden state,
    logits and the substituted layer's KV cache against the oracle; k = 0 equals cqil_model_forward bit for bit."""
    vocab, max_seq = 509, 32
    for sizes, grp, ks in (([1, 1, 1, 1, 1], 3, (1, 2, 3)), ([1, 2, 2], 2, (1, 2))):
        L = sum(sizes)
        for k in ks:
            model, groups, kv_len, nl, emb, gfin, head = _tiny_model(dtype, sizes, vocab, max_seq, seed=5200 + L)
            od = odims(TINY, max_seq, dtype)
            okc, ovc = orc.new_cache(L, 1, od), orc.new_cache(L, 1, od)
            tokens = torch.randint(0, vocab, (1, 11), generator=synth.generator(4)).to(torch.int32)
            olen = 0
            for step in range(3):
                T = tokens.shape[1]
                gws = Guarded(cq.cqil_model_substituted_workspace_bytes(model, 1, T))
                logits = torch.empty(1, vocab, dtype=torch.float32, device="cuda")
                hid = torch.empty(1, T, TINY.d_model, dtype=dtype, device="cuda")
                cq.cqil_model_forward_substituted(model, tokens.cuda(), 1, T, 1, True, grp, k, hid, logits, None, gws.body)
                torch.cuda.synchronize()
                gws.check(f"substituted model {sizes} k={k}")
                ref = orc.model_forward(od, nl, sizes, 1, emb, gfin, head, okc, ovc, [olen], tokens.numpy(),
                                        sub_group=grp, sub_k=k)
                plain = orc.model_forward(od, nl, sizes, 1, emb, gfin, head, okc.copy(), ovc.copy(), [olen], tokens.numpy())
                e_h = rel_err(synth.widen(hid.cpu()), ref["hidden"])
                e_l = rel_err(logits.cpu().numpy(), ref["logits"])
                l0 = sum(sizes[:grp])
                e_k = rel_err(synth.widen(groups[grp].k[:, 0, :, olen:olen + T].cpu()), okc[l0:l0 + sizes[grp], 0, :, olen:olen + T])
                sep = rel_err(plain["hidden"], ref["hidden"])
                say(f"  substitution {sizes} group {grp} k={k} {dtype} step {step}: hidden {e_h:.2e} logits {e_l:.2e} "
                    f"cache {e_k:.2e} (plain model differs by {sep:.2e})")
                assert max(e_h, e_l, e_k) <= TOL[dtype]
                assert sep > 4 * TOL[dtype], "the substitution is not visible in this test"
                olen += T
                tokens = torch.from_numpy(ref["next"].reshape(1, 1).astype(np.int32))
    # k = 0 is the plain model loop, bit for bit
    model, groups, kv_len, *_ = _tiny_model(dtype, [1, 2, 1], vocab, max_seq, seed=5300)
    tokens = torch.randint(0, vocab, (1, 5), generator=synth.generator(6)).to(torch.int32).cuda()
    ws = torch.empty(cq.cqil_model_substituted_workspace_bytes(model, 1, 5), dtype=torch.uint8, device="cuda")
    a = torch.empty(1, 5, TINY.d_model, dtype=dtype, device="cuda")
    b = torch.empty_like(a)
    cq.cqil_model_forward(model, tokens, 1, 5, 1, False, a, None, None, ws)
    cq.cqil_model_forward_substituted(model, tokens, 1, 5, 1, False, 2, 0, b, None, None, ws)
    torch.cuda.synchronize()
    assert torch.equal(a, b)


@pytest.mark.parametrize("vocab", [1003, 1024])
def test_greedy_token_is_the_lowest_index_among_equal_maxima(vocab):
    """Ties in the logits (duplicated and all-zero rows of the lm head): the greedy token is the first maximum."""
    dtype, max_seq = torch.float32, 16
    model, groups, kv_len, nl, emb, gfin, head = _tiny_model(dtype, [1, 2], vocab, max_seq, seed=910)
    lm = model._keep[6]
    lm.zero_()
    v = synth.normal((TINY.d_model,), 1.0, dtype, synth.generator(3)).cuda()
    for row in (977, 41, 500, 42):
        lm[row] = v
    tokens = torch.randint(0, vocab, (1, 4), generator=synth.generator(2)).to(torch.int32).cuda()
    ws = torch.empty(cq.cqil_model_workspace_bytes(model, 1, 4), dtype=torch.uint8, device="cuda")
    logits = torch.empty(1, vocab, dtype=torch.float32, device="cuda")
    nxt = torch.empty(1, dtype=torch.int32, device="cuda")
    for sign in (1.0, -1.0):
        for row in (977, 41, 500, 42):
            lm[row] = sign * v
        kv_len.zero_(); model.c.max_kv_len = 0
        cq.cqil_model_forward(model, tokens, 1, 4, 1, False, None, logits, nxt, ws)
        torch.cuda.synchronize()
        lg = logits.cpu().numpy()[0]
        assert (lg[[41, 42, 500, 977]] == lg[41]).all() and lg[0] == 0.0
        assert nxt.item() == int(np.argmax(lg))              # numpy returns the first maximum: 41 or 0
        assert nxt.item() in (0, 41)


def test_model_forward_equals_chain_of_group_calls():
    """Bit-for-bit: the model loop is the embedding followed by cqil_group_forward per group."""
    dtype, vocab, max_seq = torch.bfloat16, 257, 32
    sizes = [1, 3, 2]
    model, groups, kv_len, *_ = _tiny_model(dtype, sizes, vocab, max_seq, seed=17)
    tokens = torch.randint(0, vocab, (1, 6), generator=synth.generator(1)).to(torch.int32).cuda()
    ws = torch.empty(cq.cqil_model_workspace_bytes(model, 1, 6), dtype=torch.uint8, device="cuda")
    hid = torch.empty(1, 6, TINY.d_model, dtype=dtype, device="cuda")
    cq.cqil_model_forward(model, tokens, 1, 6, 1, False, hid, None, None, ws)
    k_model = [g.k.clone() for g in groups]
    emb = model._keep[4]
    x = emb[tokens[0].long()].reshape(1, 6, -1).contiguous()
    for g in groups:
        g.k.zero_(); g.v.zero_(); g.set_kv_len([0])
        x = g.forward(x, 1, advance=False)
    torch.cuda.synchronize()
    assert torch.equal(x, hid)
    for g, k in zip(groups, k_model):
        assert torch.equal(g.k, k)
