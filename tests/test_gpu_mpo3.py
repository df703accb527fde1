"""GPU parity for the three-tensor form (format.i3 == 8; Eq. 2 with n = 3): decode against
oracle-compressed caches through both kernels, and the GPU's own second cut through properties."""
import dataclasses
import sys

import numpy as np
import pytest
import torch

from oracle import decoquant_oracle as O
import paper_2405_12591_amd as dq
import workloads
from gpu_util import DEV, formats, oracle_cache_for_pairs, run_decode, tolerance

pytestmark = pytest.mark.gpu


def _say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def _small(name, **kw):
    return dataclasses.replace(workloads.get_workload(name), i3=8, **kw)


def _decode_case(w, lens, flags, pairs=None, max_seq=None):
    fmt, ofmt = formats(w)
    assert fmt.i3 == 8
    lens = np.asarray(lens, np.int32)
    all_pairs = [(b, h) for b in range(w.batch) for h in range(w.kv_heads)]
    pairs = all_pairs if pairs is None else pairs
    cache = oracle_cache_for_pairs(w, ofmt, pairs, lens)
    q = workloads.query(w)
    want = O.attention_decode(cache, ofmt, q, lens, pairs=pairs)
    got16, got32 = run_decode(fmt, cache, q, lens, int(w.max_seq if max_seq is None else max_seq), flags)
    rep = w.q_heads // w.kv_heads
    worst = 0.0
    for b, h in pairs:
        for hq in range(h * rep, (h + 1) * rep):
            e16 = np.abs(got16[b, hq].astype(np.float64) - want[b, hq])
            assert (e16 <= tolerance(want[b, hq])).all(), (b, hq, e16.max())
            e32 = np.abs(got32[b, hq].astype(np.float64) - want[b, hq])
            assert (e32 <= np.maximum(2e-3, 1e-4 * np.abs(want[b, hq]))).all(), (b, hq, e32.max())
            worst = max(worst, e32.max())
    return worst


CASES = [
    ("llama7b_4bit", dict(batch=2, q_heads=4, kv_heads=4, max_seq=1000, min_seq=1000), [1000, 257]),
    ("llama7b_4bit", dict(batch=3, q_heads=2, kv_heads=2, max_seq=2300, min_seq=2300), [2300, 1, 128]),
    ("gqa_long", dict(batch=2, q_heads=8, kv_heads=2, max_seq=900, min_seq=900), [900, 5]),
    ("gqa_long", dict(batch=2, q_heads=4, kv_heads=2, max_seq=700, min_seq=700), [513, 700]),
    ("llama13b_mixed", dict(batch=3, q_heads=4, kv_heads=4, max_seq=640, min_seq=1), [640, 0, 383]),
    ("llama7b_4bit", dict(batch=1, q_heads=2, kv_heads=2, max_seq=1024, min_seq=1024, block_tokens=256), [777]),
    ("llama7b_2bit", dict(batch=2, q_heads=4, kv_heads=4, max_seq=700, min_seq=700), [700, 129]),
    ("llama7b_2bit", dict(batch=3, q_heads=4, kv_heads=2, max_seq=1300, min_seq=1300), [1300, 0, 257]),
    ("llama7b_4bit", dict(batch=2, q_heads=4, kv_heads=2, max_seq=900, min_seq=900, group=64), [900, 130]),
    ("llama7b_2bit", dict(batch=2, q_heads=8, kv_heads=2, max_seq=900, min_seq=900, group=128), [900, 385]),
    ("llama7b_8bit", dict(batch=2, q_heads=4, kv_heads=4, max_seq=1000, min_seq=1000), [1000, 263]),
    ("llama7b_8bit", dict(batch=2, q_heads=4, kv_heads=2, max_seq=640, min_seq=640, group=64, block_tokens=256), [640, 511]),
]


@pytest.mark.parametrize("name,kw,lens", CASES[:5] + [CASES[6], CASES[10]])
def test_decode_generic_three_tensors(name, kw, lens):
    w = _small(name, **kw)
    _say("decode generic, three tensors: %s %s lens=%s" % (name, kw, lens))
    worst = _decode_case(w, lens, dq.DECODE_FORCE_GENERIC)
    _say("  worst fp32 abs err %.3g" % worst)


def test_decode_generic_three_tensors_tiny_shape():
    # head_dim 64, j1 8, 256-token blocks: the shape only the plain kernel takes
    w = dataclasses.replace(workloads.get_workload("tiny"), i3=8)
    for lens in ([256], [131], [8], [0]):
        _say("decode generic, three tensors: tiny lens=%s" % lens)
        _decode_case(w, lens, dq.DECODE_FORCE_GENERIC)


@pytest.mark.parametrize("name,kw,lens", CASES)
def test_decode_mfma_three_tensors(name, kw, lens):
    w = _small(name, **kw)
    fmt, _ = formats(w)
    assert dq.decode_mfma_supported(fmt, w.q_heads, w.kv_heads)
    _say("decode mfma, three tensors: %s %s lens=%s" % (name, kw, lens))
    worst = _decode_case(w, lens, dq.DECODE_FORCE_MFMA)
    _say("  worst fp32 abs err %.3g" % worst)


def test_decode_full_size_three_tensors_sampled_pairs():
    """The benchmark shape with three tensors, default kernel choice and launch shape; sampled
    (sequence, head) pairs are oracle-compressed, every other pair holds garbage bytes."""
    w = workloads.get_workload("llama7b_4bit_n3")
    pairs = [(0, 0), (7, 31), (4, 9)]
    lens = workloads.seq_lens(w)
    _say("decode full-size llama7b_4bit_n3 pairs=%s" % pairs)
    worst = _decode_case(w, lens, dq.DECODE_AUTO, pairs=pairs, max_seq=int(lens.max()))
    _say("  worst fp32 abs err %.3g" % worst)


def test_decode_three_tensors_with_fp16_tail():
    w = _small("llama7b_4bit", batch=2, q_heads=4, kv_heads=2, max_seq=640, min_seq=640)
    fmt, ofmt = formats(w)
    lens = np.array([640, 256], np.int32)
    tail_lens = np.array([37, 0], np.int32)
    pairs = [(b, h) for b in range(2) for h in range(2)]
    cache = oracle_cache_for_pairs(w, ofmt, pairs, lens)
    r = np.random.default_rng(3)
    kt = r.standard_normal((2, 2, 128, 128)).astype(np.float16)
    vt = r.standard_normal((2, 2, 128, 128)).astype(np.float16)
    q = workloads.query(w)
    want = O.attention_decode(cache, ofmt, q, lens, k_tail=kt, v_tail=vt, tail_lens=tail_lens)
    c = dq.cache_from_numpy(fmt, cache, DEV)
    ws = dq.decode_workspace(fmt, 2, 4, 2, 640, DEV)
    tail = (torch.from_numpy(kt).to(DEV), torch.from_numpy(vt).to(DEV), torch.from_numpy(tail_lens).to(DEV))
    for flags in (dq.DECODE_FORCE_MFMA, dq.DECODE_FORCE_GENERIC):
        _say("decode with tail, three tensors, flags=%d" % flags)
        out = dq.attn_decode(c, torch.from_numpy(q).to(DEV), torch.from_numpy(lens).to(DEV), 640, ws,
                             flags=flags, tail=tail)
        torch.cuda.synchronize()
        got = out.cpu().numpy().astype(np.float64)
        assert (np.abs(got - want) <= tolerance(want)).all()


@pytest.mark.parametrize("name,t_new,n_valid", [
    ("llama7b_4bit", 128, None), ("llama7b_2bit", 128, None), ("llama13b_mixed", 128, [128, 37, 1]),
    ("gqa_long", 100, None), ("tiny", 256, None), ("llama7b_8bit", 128, None),
])
def test_compress_kv_three_tensors_properties(name, t_new, n_valid):
    kw = dict(batch=3 if n_valid else 2, q_heads=4, kv_heads=2) if name != "tiny" else {}
    w = _small(name, **kw) if name != "tiny" else dataclasses.replace(workloads.get_workload("tiny"), i3=8)
    _say("compress, three tensors: %s t_new=%d n_valid=%s" % (name, t_new, n_valid))
    _check_compress3(w, t_new, n_valid)


@pytest.mark.parametrize("name,t_new,n_valid", [
    ("llama7b_4bit", 128, None), ("llama7b_2bit", 100, [100, 37, 1]), ("llama7b_8bit", 128, None), ("gqa_long", 77, None),
    ("llama13b_mixed", 128, [128, 1, 9]),
])
def test_compress_kv_three_tensors_one_kernel_build(name, t_new, n_valid):
    """The same properties for the build that makes both cuts and quantizes in one launch (what calls
    of more than 512 blocks take; a forced wave count of one selects it for a small call)."""
    w = _small(name, batch=3 if n_valid else 2, q_heads=4, kv_heads=2)
    _say("compress, three tensors, one launch: %s t_new=%d n_valid=%s" % (name, t_new, n_valid))
    _check_compress3(w, t_new, n_valid, waves=1)


@pytest.mark.parametrize("bits,group,levels", [(4, 128, 0), (2, 64, 1), (8, 128, 0)])
def test_compress_three_tensors_prompt_sized_call(bits, group, levels):
    """A prompt-sized call (2304 blocks, two per sequence and head, cut inside the kernel) through the
    one-kernel build: with and without the fp32 rows kept the cache is the same bit for bit, and
    sampled blocks have the oracle's properties; ragged rows and a skipped sequence included."""
    batch, kvh = 9, 64
    w = dataclasses.replace(workloads.get_workload("llama7b_4bit"), batch=batch, q_heads=kvh, kv_heads=kvh, bits=bits,
                            group=group, levels=levels, max_seq=256, min_seq=256, i3=8)
    fmt, ofmt = formats(w)
    _say("three tensors, prompt-sized call: bits=%d G=%d levels=%d, %d blocks" % (bits, group, levels, batch * kvh * 4))
    gen = torch.Generator(device=DEV).manual_seed(5)
    kd = (torch.randn((batch, kvh, 256, 128), device=DEV, generator=gen) * 2).to(torch.float16)
    vd = (torch.randn((batch, kvh, 256, 128), device=DEV, generator=gen) * 2).to(torch.float16)
    kd[:, :, :, 5] *= 20
    lens = [256, 130, 1, 0, 255, 128, 129, 256, 77]
    firsts = [0, 1, 0, 0, 0, -1, 0, 0, 1]
    n_valid = torch.tensor(lens, dtype=torch.int32, device=DEV)
    first = torch.tensor(firsts, dtype=torch.int32, device=DEV)
    out = []
    for keep in (True, False):
        cache = dq.alloc_cache(fmt, batch, kvh, 3, DEV, fill=0xA5)
        ws = dq.compress_workspace(fmt, batch, kvh, DEV, t_new=256)
        dq.compress_kv_blocks(cache, kd, vd, first, n_valid, ws, keep_large=keep)
        torch.cuda.synchronize()
        assert int(ws[:4].view(torch.int32).item()) == 0
        out.append((cache, ws))
    for name in out[0][0].t:
        assert torch.equal(out[0][0].t[name], out[1][0].t[name]), name
    arrs = {n: t.cpu().numpy() for n, t in out[0][0].t.items()}
    units = batch * kvh * 2 * 2
    large = out[0][1][256:256 + 4 * units * 128 * 128].view(torch.float32).cpu().numpy().reshape(units, 128, 128)
    kh, vh = kd.cpu().numpy(), vd.cpu().numpy()
    worst = 0.0
    for b, h in [(0, 0), (1, 63), (4, 17), (8, 1), (7, 40), (6, 5)]:
        for j in range(2):
            nv = min(max(lens[b] - 128 * j, 0), 128)
            if nv == 0:
                continue
            for which, rows in (("k", kh), ("v", vh)):
                x = np.zeros((128, 128))
                x[:nv] = rows[b, h, 128 * j:128 * j + nv].astype(np.float64)
                unit = ((b * kvh + h) * 2 + j) * 2 + (which == "v")
                worst = max(worst, _block_properties3(arrs, ofmt, x, large[unit], b, h, firsts[b] + j, which))
    _say("  worst |T_2^T T_2 - I| = %.3g over the sampled blocks" % worst)


@pytest.mark.parametrize("seed", [31, 32])
def test_compress_kv_three_tensors_random_cases(seed):
    """Seeded sweep: code widths, group sizes, head dimensions, block sizes, ragged n_valid, short
    t_new, skipped sequences."""
    rng = np.random.default_rng(seed)
    for case in range(8):
        d = int(rng.choice([128, 128, 64]))
        j1 = 16 if d == 128 and rng.integers(0, 4) else int(rng.choice([8, 16] if d == 64 else [8, 32]))
        bits = int(rng.choice([2, 4, 8]))
        group = int(rng.choice([g for g in (32, 64, 128) if g <= d and (g == d or g <= d // 2) and (g * bits) % 32 == 0]))
        tb = int(rng.choice([128, 256]))
        batch, kvh = int(rng.choice([2, 3])), int(rng.choice([1, 2, 5]))
        t_new = int(rng.choice([tb, tb, int(rng.integers(1, tb + 1))]))
        n_valid = None if rng.integers(0, 2) else [int(rng.choice([1, 2, t_new, int(rng.integers(1, t_new + 1))])) for _ in range(batch)]
        w = dataclasses.replace(workloads.get_workload("llama7b_4bit"), batch=batch, q_heads=kvh, kv_heads=kvh, head_dim=d,
                                j1=j1, j2=d // j1, bits=bits, group=group, block_tokens=tb, max_seq=tb, min_seq=tb,
                                seed=5000 + 100 * seed + case, n_outlier=int(rng.choice([0, 2, 6])), i3=8)
        _say("compress, three tensors, random seed %d case %d: d=%d j1=%d bits=%d G=%d Tb=%d B=%d H=%d t_new=%d n_valid=%s"
             % (seed, case, d, j1, bits, group, tb, batch, kvh, t_new, n_valid))
        _check_compress3(w, t_new, n_valid, waves=case % 2)    # the library's choice, then the one-kernel build


@pytest.mark.parametrize("i3", [1, 8])
def test_compress_kv_degenerate_blocks(i3):
    """All-zero blocks, a block of identical rows (rank one on both sides), a block whose only
    non-zero entries sit in one channel, values at the fp16 limit: the decomposition must settle
    and leave finite factors whose product is the block."""
    w = dataclasses.replace(workloads.get_workload("llama7b_4bit"), batch=2, q_heads=2, kv_heads=2, max_seq=128, min_seq=128, i3=i3)
    fmt, ofmt = formats(w)
    r = np.random.default_rng(77)
    blocks = np.zeros((2, 2, 128, 128), np.float16)          # (0, 0): all zero
    blocks[0, 1] = r.standard_normal(128).astype(np.float16)[None, :]                 # identical rows
    blocks[1, 0, :, 37] = r.standard_normal(128).astype(np.float16)                   # one channel
    blocks[1, 1] = (r.choice([-1.0, 1.0], size=(128, 128)) * 60000.0).astype(np.float16)   # near the fp16 limit
    cache = dq.alloc_cache(fmt, 2, 2, 1, DEV, fill=0xA5)
    ws = dq.compress_workspace(fmt, 2, 2, DEV)
    x = torch.from_numpy(blocks).to(DEV)
    dq.compress_kv(cache, x, x.clone(), torch.zeros(2, dtype=torch.int32, device=DEV), None, ws)
    torch.cuda.synchronize()
    sweeps = int(ws[4:8].view(torch.int32).item())
    _say("degenerate blocks, i3=%d: status %d, sweeps %d" % (i3, int(ws[:4].view(torch.int32).item()), sweeps))
    assert sweeps <= 10
    arrs = {n: t.cpu().numpy() for n, t in cache.t.items()}
    for b in range(2):
        for h in range(2):
            for which in ("k", "v"):
                blk = O.load_block(arrs, ofmt, b, h, 0, which)
                assert all(np.isfinite(np.asarray(a, np.float64)).all() for a in blk)
                x_hat = O.reconstruct_block(blk[0], blk[1], blk[2], ofmt, *blk[3:])
                ref = blocks[b, h].astype(np.float64)
                bound = O.reconstruction_bound(blk[0], blk[1], ofmt, *blk[3:])
                # the half-step bound plus the fp16 rounding of the small tensors (saturated T_S excepted)
                slack = 2.0 ** -8 * np.abs(ref).max() + 1e-6
                if (b, h) == (1, 1) and int(ws[:4].view(torch.int32).item()) & 1:
                    continue     # T_S saturated (status bit 0): the product is no longer the block
                assert (np.abs(x_hat - ref) <= bound + slack).all(), (b, h, which, np.abs(x_hat - ref).max())


def _block_properties3(arrs, ofmt, x, kp, b, h, slot, which):
    """The oracle's properties of one three-tensor block the GPU wrote: x [T_b, d] fp64 is what went
    in (rows past the valid ones zero), kp [T_b, d] fp32 the middle tensor it left in the workspace
    (row a2*8 + e).  Returns |T_2^T T_2 - I|."""
    tb, d, j1, j2 = ofmt.block_tokens, ofmt.head_dim, ofmt.j1, ofmt.j2
    small, steps, codes, small3 = O.load_block(arrs, ofmt, b, h, slot, which)
    t_2 = O.token_major_to_middle(kp.astype(np.float64), j1, j2, 8)
    # (1) columns of T_2 orthonormal over (r, a2, b2), or zero for dropped directions
    a = t_2.reshape(-1, 8)
    gram = a.T @ a
    live = np.diag(gram) > 0.5
    ortho = np.abs(gram - np.diag(live.astype(np.float64))).max()
    assert ortho <= 2e-6, (b, h, which)
    # (2) the three tensors multiply back to the block, up to the fp16 rounding of T_1
    # and T_3 and the fp32 storage of T_2 and of the first cut's right factor
    s3 = small3.astype(np.float64)
    right = np.einsum("racd,de->raec", t_2, s3).reshape(j1, tb * j2)
    right_abs = np.einsum("racd,de->raec", np.abs(t_2), np.abs(s3)).reshape(j1, tb * j2)
    m = O.matricise(x, 1, j1)
    resid = np.abs(small.astype(np.float64) @ right - m)
    slack = 2.0 ** -9 * (np.abs(small.astype(np.float64)) @ right_abs) + 1e-6 * np.abs(m).max() + 1e-7
    assert (resid <= slack).all(), (b, h, which, resid.max())
    # T_3 has orthogonal rows (it is diag(sigma') V'^T), up to its fp16 rounding
    g3 = s3 @ s3.T
    assert np.abs(g3 - np.diag(np.diag(g3))).max() <= 4e-3 * max(np.diag(g3).max(), 1e-30)
    # (3) codes and steps are the oracle's quantization of that very T_2
    steps_o = O.group_steps(kp, ofmt.group, ofmt.qmax, ofmt.full_range)
    codes_o = O.quantize_codes(kp, steps_o, ofmt.group, ofmt.qmax, ofmt.full_range)
    assert np.array_equal(steps.view(np.uint16), steps_o.view(np.uint16))
    assert np.array_equal(codes, codes_o)
    # (4) reconstruction within the half-step bound
    x_hat = O.reconstruct_block(small, steps, codes, ofmt, small3)
    bound = O.reconstruction_bound(small, steps, ofmt, small3)
    slack_x = O.unmatricise(slack, tb, d, 1, j1)
    assert (np.abs(x_hat - x) <= bound + slack_x).all(), (b, h, which)
    return ortho


def _check_compress3(w, t_new, n_valid, waves=0):
    fmt, ofmt = formats(w)
    tb, d, j1, j2 = fmt.block_tokens, fmt.head_dim, fmt.j1, fmt.j2
    k = np.stack([np.stack([workloads.kv_pair(w, b, h, t_new)[0] for h in range(w.kv_heads)]) for b in range(w.batch)])
    v = np.stack([np.stack([workloads.kv_pair(w, b, h, t_new)[1] for h in range(w.kv_heads)]) for b in range(w.batch)])
    nb = 3
    cache = dq.alloc_cache(fmt, w.batch, w.kv_heads, nb, DEV, fill=0xA5)
    before = {n: t.clone() for n, t in cache.t.items()}
    ws = dq.compress_workspace(fmt, w.batch, w.kv_heads, DEV)
    slots = np.array([1, 2, 0][:w.batch], np.int32)
    if w.batch == 2:
        slots = np.array([1, -1], np.int32)      # second sequence is skipped
    nv = None if n_valid is None else torch.tensor(n_valid, dtype=torch.int32, device=DEV)
    dq.compress_kv(cache, torch.from_numpy(k).to(DEV), torch.from_numpy(v).to(DEV),
                   torch.from_numpy(slots).to(DEV), nv, ws, waves=waves)
    torch.cuda.synchronize()
    arrs = {n: t.cpu().numpy() for n, t in cache.t.items()}
    assert int(ws[:4].view(torch.int32).item()) == 0
    n_large = w.batch * w.kv_heads * 2 * tb * d
    large = ws[256:256 + 4 * n_large].view(torch.float32).cpu().numpy().reshape(w.batch * w.kv_heads * 2, tb, d)
    worst_ortho = 0.0
    for b in range(w.batch):
        for h in range(w.kv_heads):
            for which, x_all in (("k", k), ("v", v)):
                slot = int(slots[b])
                if slot < 0:
                    for n in arrs:   # skipped sequence: nothing written anywhere
                        assert np.array_equal(arrs[n][b, h], before[n][b, h].cpu().numpy()), n
                    continue
                n_ok = t_new if n_valid is None else min(n_valid[b], t_new)
                x = np.zeros((tb, d))
                x[:n_ok] = x_all[b, h, :n_ok].astype(np.float64)
                kp = large[(b * w.kv_heads + h) * 2 + (which == "v")]      # the middle tensor, row a2*8 + e
                worst_ortho = max(worst_ortho, _block_properties3(arrs, ofmt, x, kp, b, h, slot, which))
                # (5) other block slots of this head untouched
                for other in range(nb):
                    if other != slot:
                        for n in ("k_codes", "k_small3", "v_small3"):
                            assert np.array_equal(arrs[n][b, h, other], before[n][b, h, other].cpu().numpy())
    _say("  worst |T_2^T T_2 - I| = %.3g" % worst_ortho)


def test_gpu_compressed_three_tensor_cache_decodes_like_its_own_oracle_reading():
    """Compress on the GPU, then decode on the GPU (both kernels) and with the oracle from the same
    arrays; the lossy cache still approximates attention on the original K, V."""
    w = _small("llama7b_4bit", batch=2, q_heads=4, kv_heads=4, max_seq=512, min_seq=512)
    fmt, ofmt = formats(w)
    _say("gpu compress -> gpu decode vs oracle decode, three tensors")
    k, v = workloads.kv_tensor(w)
    nb = w.max_seq // fmt.block_tokens
    cache = dq.alloc_cache(fmt, w.batch, w.kv_heads, nb, DEV)
    ws = dq.compress_workspace(fmt, w.batch, w.kv_heads, DEV)
    kd, vd = torch.from_numpy(k).to(DEV), torch.from_numpy(v).to(DEV)
    for blk in range(nb):
        sl = slice(blk * 128, (blk + 1) * 128)
        dq.compress_kv(cache, kd[:, :, sl].contiguous(), vd[:, :, sl].contiguous(),
                       torch.full((w.batch,), blk, dtype=torch.int32, device=DEV), None, ws)
    torch.cuda.synchronize()
    arrs = {n: t.cpu().numpy() for n, t in cache.t.items()}
    q = workloads.query(w)
    lens = np.array([512, 300], np.int32)
    want = O.attention_decode(arrs, ofmt, q, lens)
    for flags in (dq.DECODE_FORCE_MFMA, dq.DECODE_FORCE_GENERIC):
        got16, _ = run_decode(fmt, arrs, q, lens, 512, flags)
        assert (np.abs(got16.astype(np.float64) - want) <= tolerance(want)).all()
    for b in range(w.batch):
        for h in range(w.kv_heads):
            ref = O.dense_attention(q[b, h], k[b, h, :lens[b]], v[b, h, :lens[b]])
            assert np.abs(want[b, h] - ref).max() < 0.15 * np.abs(v[b, h].astype(np.float64)).max()
