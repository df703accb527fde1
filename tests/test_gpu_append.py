"""The cache policy behind the C ABI (dq_cache_append; Section 3.2: rows are buffered in fp16 and a
tail is compressed when it holds a block's worth): device-side decisions, a generic step under graph
capture replayed across block boundaries, ragged counts, a full cache, and the 13B-shaped
configuration's flow at full size (mixed-length cache, 128 rows appended per sequence, 320 blocks
compressed, decode) against the oracle reading the GPU's own arrays."""
import dataclasses

import numpy as np
import pytest
import torch

from oracle import decoquant_oracle as O
import paper_2405_12591_amd as dq
import workloads
from gpu_util import DEV, formats, tolerance

pytestmark = pytest.mark.gpu


def _say(msg):
    print(msg, flush=True)


def _oracle_decode(layer, ofmt, q, pairs=None):
    arrs = {n: t.cpu().numpy() for n, t in layer.cache.t.items()}
    lens = layer.seq_lens.cpu().numpy()
    return O.attention_decode(arrs, ofmt, q, lens, pairs=pairs, k_tail=layer.k_tail.cpu().numpy(),
                              v_tail=layer.v_tail.cpu().numpy(), tail_lens=layer.tail_lens.cpu().numpy())


@pytest.mark.parametrize("bits,group,d,i3", [(4, 128, 128, 1), (2, 64, 128, 8), (4, 64, 64, 1)])
def test_generic_step_under_graph_capture_across_block_boundaries(bits, group, d, i3):
    """One captured step (append one row per sequence, decode) replayed 14 times: two of the three
    sequences cross a block boundary on different replays, so the very same graph sometimes compresses
    a tail and sometimes does not.  Every replay must match an eagerly driven twin bit for bit, and
    the oracle's reading of the GPU's arrays."""
    w = dataclasses.replace(workloads.get_workload("llama7b_4bit"), batch=3, q_heads=4, kv_heads=2, max_seq=400,
                            min_seq=400, bits=bits, group=group, head_dim=d, j1=d // 8, j2=8, i3=i3,
                            n_outlier=2 if d == 64 else 4, seed=8100 + bits)
    fmt, ofmt = formats(w)
    _say("captured serving step: bits=%d G=%d d=%d i3=%d" % (bits, group, d, i3))
    k, v = workloads.kv_tensor(w)
    kd, vd = torch.from_numpy(k).to(DEV), torch.from_numpy(v).to(DEV)
    start = [120, 250, 5]
    counts = torch.tensor(start, dtype=torch.int32, device=DEV)
    layers = [dq.KVCacheLayer(fmt, 3, 4, 2, 512, DEV) for _ in range(2)]
    for layer in layers:
        layer.prefill(kd[:, :, :256].contiguous(), vd[:, :, :256].contiguous(), counts=counts)
    assert layers[0].n_blocks == [0, 1, 0] and layers[0].n_tail == [120, 122, 5]
    graphed, eager = layers
    q = workloads.query(w)
    qd = torch.from_numpy(q).to(DEV)
    row_k = torch.empty((3, 2, 1, d), dtype=torch.float16, device=DEV)
    row_v = torch.empty_like(row_k)
    out = torch.empty_like(qd)

    def feed(step):
        for b in range(3):
            row_k[b] = kd[b, :, start[b] + step:start[b] + step + 1]
            row_v[b] = vd[b, :, start[b] + step:start[b] + step + 1]

    def step_fn(layer, o):
        dq.cache_append(layer.cache, layer.k_tail, layer.v_tail, layer.tail_lens, layer.seq_lens, row_k, row_v, None,
                        layer.ws_append)
        layer.decode(qd, out=o, max_seq_len=512)

    # capture (the captured launches do not run; the warm-up step ahead of it does, as step 0)
    stream = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    feed(0)
    torch.cuda.synchronize()
    with torch.cuda.stream(stream):
        step_fn(graphed, out)
        stream.synchronize()
        with torch.cuda.graph(graph, stream=stream):
            step_fn(graphed, out)
    torch.cuda.synchronize()
    out_e = torch.empty_like(qd)
    step_fn(eager, out_e)
    torch.cuda.synchronize()
    assert torch.equal(out, out_e)
    for step in range(1, 15):
        feed(step)
        scratch = torch.randn(1 << 18, device=DEV).sum()     # eager work between replays
        out.fill_(float("nan"))
        graph.replay()
        step_fn(eager, out_e)
        torch.cuda.synchronize()
        assert torch.equal(graphed.seq_lens, eager.seq_lens) and torch.equal(graphed.tail_lens, eager.tail_lens), step
        assert torch.equal(out, out_e), step
        for n in graphed.cache.t:
            assert torch.equal(graphed.cache.t[n], eager.cache.t[n]), (step, n)
        if step in (1, 5, 6, 7, 8, 14):
            want = _oracle_decode(graphed, ofmt, q)
            got = out.cpu().numpy().astype(np.float64)
            assert (np.abs(got - want) <= tolerance(want)).all(), (step, np.abs(got - want).max())
        del scratch
    # sequence 1 crossed at step 5 (250 + 6 rows = 256), sequence 0 at step 7 (120 + 8 = 128)
    assert graphed.n_blocks == [1, 2, 0] and graphed.n_tail == [7, 9, 20]
    assert graphed.status == 0
    # the compressed blocks hold the rows that were appended
    arrs = {n: t.cpu().numpy() for n, t in graphed.cache.t.items()}
    for b, n_tok in ((0, 128), (1, 256)):
        for h in range(2):
            k_hat, v_hat = O.reconstruct_sequence(arrs, ofmt, b, h, n_tok)
            for x_hat, x in ((k_hat, k[b, h, :n_tok]), (v_hat, v[b, h, :n_tok])):
                assert np.linalg.norm(x_hat - x.astype(np.float64)) < (0.6 if bits == 2 else 0.2) * np.linalg.norm(x.astype(np.float64))
        nt = graphed.n_tail[b]
        assert np.array_equal(graphed.k_tail[b, :, :nt].cpu().numpy(), k[b, :, n_tok:n_tok + nt])


def test_append_ragged_counts_several_rows_and_a_full_cache():
    """Many rows per call with a count per sequence: rows fill the tail, the tail is compressed, the
    rest restarts it; a sequence whose cache has no free slot keeps its full tail and raises the
    status bit; a zero count leaves a sequence alone."""
    w = dataclasses.replace(workloads.get_workload("llama7b_4bit"), batch=4, q_heads=2, kv_heads=2, max_seq=512, min_seq=512,
                            seed=8200)
    fmt, ofmt = formats(w)
    k, v = workloads.kv_tensor(w)
    kd, vd = torch.from_numpy(k).to(DEV), torch.from_numpy(v).to(DEV)
    layer = dq.KVCacheLayer(fmt, 4, 2, 2, 256, DEV)            # two block slots per sequence
    pos = [0, 0, 0, 0]
    plan = [(100, [100, 37, 0, 100]), (128, [128, 91, 0, 128]), (128, [50, 128, 128, 128]), (60, [60, 0, 60, 60])]
    for n, counts in plan:
        rows_k = torch.stack([kd[b, :, pos[b]:pos[b] + n] for b in range(4)]).contiguous()
        rows_v = torch.stack([vd[b, :, pos[b]:pos[b] + n] for b in range(4)]).contiguous()
        layer.append(rows_k, rows_v, counts=torch.tensor(counts, dtype=torch.int32, device=DEV))
        pos = [p + c for p, c in zip(pos, counts)]
    torch.cuda.synchronize()
    # sequence 3: 356 rows fill both slots and 100 rows of the tail; 28 of the last 60 fill it, and it cannot be compressed
    assert layer.n_blocks == [2, 2, 1, 2] and layer.n_tail == [82, 0, 60, 128]
    assert layer.status == 1
    arrs = {n: t.cpu().numpy() for n, t in layer.cache.t.items()}
    for b in range(3):
        nb, nt = layer.n_blocks[b], layer.n_tail[b]
        assert nb * 128 + nt == pos[b]
        for h in range(2):
            k_hat, _ = O.reconstruct_sequence(arrs, ofmt, b, h, nb * 128)
            x = k[b, h, :nb * 128].astype(np.float64)
            assert np.linalg.norm(k_hat - x) < 0.2 * np.linalg.norm(x)
            assert np.array_equal(layer.k_tail[b, h, :nt].cpu().numpy(), k[b, h, nb * 128:pos[b]])
            assert np.array_equal(layer.v_tail[b, h, :nt].cpu().numpy(), v[b, h, nb * 128:pos[b]])
    assert np.array_equal(layer.k_tail[3, 0].cpu().numpy(), k[3, 0, 256:384])       # the rows that found room
    q = workloads.query(w)
    want = _oracle_decode(layer, ofmt, q)
    got = layer.decode(torch.from_numpy(q).to(DEV), max_seq_len=256).cpu().numpy().astype(np.float64)
    assert (np.abs(got - want) <= tolerance(want)).all()


def test_no_compress_flag_leaves_the_launch_out_and_reports_a_broken_promise():
    fmt = dq.Format(4, 128, 128, 16, 8, 128)
    layer = dq.KVCacheLayer(fmt, 2, 2, 2, 256, DEV)
    rows = torch.randn((2, 2, 100, 128), device=DEV).to(torch.float16)
    dq.cache_append(layer.cache, layer.k_tail, layer.v_tail, layer.tail_lens, layer.seq_lens, rows, rows, None,
                    layer.ws_append, flags=dq.APPEND_NO_COMPRESS)
    torch.cuda.synchronize()
    assert layer.n_tail == [100, 100] and layer.n_blocks == [0, 0] and layer.status == 0
    assert torch.equal(layer.k_tail[:, :, :100], rows)
    dq.cache_append(layer.cache, layer.k_tail, layer.v_tail, layer.tail_lens, layer.seq_lens, rows, rows,
                    torch.tensor([27, 28], dtype=torch.int32, device=DEV), layer.ws_append, flags=dq.APPEND_NO_COMPRESS)
    torch.cuda.synchronize()
    assert layer.n_tail == [127, 128] and layer.n_blocks == [0, 0] and layer.status == 2


def test_13b_configuration_flow_at_full_size():
    """The 13B-shaped configuration as stated: a cache of mixed lengths (4 sequences x 40 heads, 8192 to
    16384 tokens), 128 new rows per sequence appended through the tail path, every tail fills and is
    compressed (320 blocks in one call), then decode over S_b + 128 tokens.  Sampled (sequence, head)
    pairs carry the workload's values and are compared with the oracle reading the GPU's own arrays;
    the other pairs hold random rows."""
    w = workloads.get_workload("llama13b_mixed")
    fmt, ofmt = formats(w)
    lens = workloads.seq_lens(w)
    tb = w.block_tokens
    order = np.argsort(lens)
    pairs = [(int(order[0]), 0), (int(order[-1]), 39), (1, 7), (2, 20), (int(order[0]), 38), (3, 13), (0, 1), (2, 39)]
    _say("13B flow at full size: lens=%s pairs=%s" % (lens.tolist(), pairs))
    n_max = int(lens.max())
    gen = torch.Generator(device=DEV).manual_seed(5)
    layer = dq.KVCacheLayer(fmt, w.batch, w.q_heads, w.kv_heads, w.max_seq + w.append_tokens, DEV)
    kd = torch.randn((w.batch, w.kv_heads, n_max, w.head_dim), device=DEV, generator=gen).to(torch.float16)
    vd = torch.randn((w.batch, w.kv_heads, n_max, w.head_dim), device=DEV, generator=gen).to(torch.float16)
    ka = torch.randn((w.batch, w.kv_heads, w.append_tokens, w.head_dim), device=DEV, generator=gen).to(torch.float16)
    va = torch.randn((w.batch, w.kv_heads, w.append_tokens, w.head_dim), device=DEV, generator=gen).to(torch.float16)
    host = {}
    for b, h in pairs:
        kk, vv = workloads.kv_pair(w, b, h, int(lens[b]))
        ak, av = workloads.appended_pair(w, b, h)
        host[b, h] = (np.concatenate([kk, ak]), np.concatenate([vv, av]))
        kd[b, h, :lens[b]] = torch.from_numpy(kk).to(DEV)
        vd[b, h, :lens[b]] = torch.from_numpy(vv).to(DEV)
        ka[b, h] = torch.from_numpy(ak).to(DEV)
        va[b, h] = torch.from_numpy(av).to(DEV)
    layer.prefill(kd, vd, counts=torch.from_numpy(lens).to(DEV))
    torch.cuda.synchronize()
    assert layer.n_blocks == (lens // tb).tolist() and layer.n_tail == (lens % tb).tolist()
    before = layer.n_blocks
    layer.append(ka, va)                                        # 128 rows each: every tail fills -> 320 blocks compressed
    q = workloads.query(w)
    out = layer.decode(torch.from_numpy(q).to(DEV))
    torch.cuda.synchronize()
    assert layer.n_blocks == [nb + 1 for nb in before] and layer.n_tail == (lens % tb).tolist() and layer.status == 0
    want = _oracle_decode(layer, ofmt, q, pairs=pairs)
    got = out.cpu().numpy().astype(np.float64)
    arrs = {n: t.cpu().numpy() for n, t in layer.cache.t.items()}
    worst = 0.0
    for b, h in pairs:
        err = np.abs(got[b, h] - want[b, h])
        assert (err <= tolerance(want[b, h])).all(), (b, h, err.max())
        worst = max(worst, err.max())
        # the block the append compressed holds rows [S_b - S_b % 128, ... + 128) of the sequence
        nb = before[b]
        kk, vv = host[b, h]
        for which, x in (("k", kk), ("v", vv)):
            small, steps, codes = O.load_block(arrs, ofmt, b, h, nb, which)
            x_blk = x[nb * tb:(nb + 1) * tb].astype(np.float64)
            x_hat = O.reconstruct_block(small, steps, codes, ofmt)
            bound = O.reconstruction_bound(small, steps, ofmt)
            # Eq. 1's half step per code through |T_S|, plus the fp16 rounding of T_S and fp32 of T_L
            slack = 2.0 ** -9 * np.abs(x_blk) + 2e-3 * np.abs(x_blk).max()
            assert (np.abs(x_hat - x_blk) <= bound + slack).all(), (b, h, which)
        nt = int(lens[b] % tb)
        assert np.array_equal(layer.k_tail[b, h, :nt].cpu().numpy(), kk[(nb + 1) * tb:(nb + 1) * tb + nt])
    _say("  worst fp16 abs err on %d pairs %.3g" % (len(pairs), worst))
