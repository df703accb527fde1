"""GPU parity: the HIP library against the CPU oracle, through the C ABI."""
import numpy as np
import pytest
import torch

from oracle import decoquant_oracle as O
import paper_2405_12591_amd as dq
import workloads
from gpu_util import DEV, formats, oracle_cache_for_pairs, tolerance, run_decode

pytestmark = pytest.mark.gpu


def _say(msg):
    print(msg, flush=True)


# ------------------------------------------------------------------------------------------
# quantize + pack: bit-exact codes and steps from the same large tensor
# ------------------------------------------------------------------------------------------
@pytest.mark.parametrize("bits,group,d,j1", [(4, 128, 128, 16), (4, 64, 128, 16), (2, 64, 128, 16),
                                             (8, 128, 128, 16), (4, 64, 64, 8), (2, 32, 64, 8),
                                             (4, 32, 128, 32)])
def test_quantize_pack_bit_exact(bits, group, d, j1):
    _say("quantize_pack bits=%d G=%d d=%d j1=%d" % (bits, group, d, j1))
    j2 = d // j1
    fmt, ofmt = dq.Format(bits, group, d, j1, j2, 128), O.Format(bits, group, d, j1, j2, 128)
    r = np.random.default_rng(bits * 1000 + group)
    rows = []
    for i in range(3):                          # three real decomposed blocks (ragged: 3 tiles)
        x = r.standard_normal((128, d))
        x[:, r.choice(d, 3, replace=False)] *= 20
        rows.append(O.compress_block(x.astype(np.float16), ofmt).large32)
    kp = np.concatenate(rows)
    qmax = ofmt.qmax
    kp[5, :] = 0.0                                             # zero row -> step 0, codes 0
    kp[6, :group] = np.float32(0.125) * (r.integers(-2 * qmax, 2 * qmax + 1, group) / 2.0)  # exact ties
    kp[6, 0] = np.float32(0.125 * qmax)
    kp[7, :group] = 1e-7 * r.standard_normal(group)            # subnormal steps
    kp = kp.astype(np.float32)
    # a step that is not a power of two, with elements on, just above and just below every tie
    s16 = np.float32(np.float16(0.01234))
    ties = np.array([(k + 0.5) * float(s16) for k in range(-qmax, qmax)], np.float32)
    near = np.concatenate([ties, np.nextafter(ties, np.float32(np.inf)), np.nextafter(ties, np.float32(-np.inf))])
    near = np.resize(near, group).astype(np.float32)
    near[0] = np.float32(float(s16) * qmax)                     # fixes the group's step at s16
    kp[8, :group] = near
    # group maxima whose quotient by qmax sits on, or one and two fp32 steps beside, an fp16 midpoint
    h = np.float16(0.0371)
    for i in range(12):
        lo = np.float16(h) if i < 8 else np.float16(3e-6)       # normal and subnormal fp16 steps
        mid = (float(lo) + float(np.nextafter(lo, np.float16(np.inf)))) / 2.0
        a = np.float32(mid * qmax)
        for _ in range(abs(i % 5 - 2)):
            a = np.nextafter(a, np.float32(np.inf) if i % 5 > 2 else np.float32(0))
        row = (0.3 * float(a) * r.standard_normal(group)).astype(np.float32)
        row = np.clip(row, -float(a), float(a))
        row[i % group] = a
        kp[9 + i, :group] = row
        h = np.nextafter(np.nextafter(h, np.float16(np.inf)), np.float16(np.inf))
    steps = O.group_steps(kp, group, qmax)
    codes = O.quantize_codes(kp, steps, group, qmax)
    want_k = O.pack_rows(codes, bits)
    want_v = O.pack_rows(np.concatenate([O.value_codes_to_tiles(codes[i * 128:(i + 1) * 128], j1, j2)
                                         for i in range(3)]), bits)
    t = torch.from_numpy(kp).to(DEV)
    for layout, want in ((False, want_k), (True, want_v)):
        got_c, got_s = dq.quantize_pack(fmt, t, layout)
        torch.cuda.synchronize()
        assert np.array_equal(got_s.cpu().numpy().view(np.uint16), steps.view(np.uint16))
        assert np.array_equal(got_c.cpu().numpy().reshape(want.shape), want)


# ------------------------------------------------------------------------------------------
# decode attention on an oracle-compressed cache
# ------------------------------------------------------------------------------------------
def _decode_case(w, lens, flags, pairs=None):
    fmt, ofmt = formats(w)
    lens = np.asarray(lens, np.int32)
    all_pairs = [(b, h) for b in range(w.batch) for h in range(w.kv_heads)]
    pairs = all_pairs if pairs is None else pairs
    cache = oracle_cache_for_pairs(w, ofmt, pairs, lens)
    q = workloads.query(w)
    want = O.attention_decode(cache, ofmt, q, lens, pairs=pairs)
    got16, got32 = run_decode(fmt, cache, q, lens, int(w.max_seq), flags)
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


def test_decode_generic_tiny_full():
    w = workloads.get_workload("tiny")
    _say("decode generic tiny")
    worst = _decode_case(w, workloads.seq_lens(w), dq.DECODE_FORCE_GENERIC)
    _say("  worst fp32 abs err %.3g" % worst)


@pytest.mark.parametrize("flags", [dq.DECODE_FORCE_GENERIC, dq.DECODE_FORCE_MFMA])
def test_tiny_worst_error_where_the_plain_bound_applies(flags):
    """The Tiny configuration's outputs reach |20| (x20 outlier channels), where half an fp16 ulp alone
    is 8e-3; this reports, and holds to the plain 2e-3, the error of the elements with |exact| < 2."""
    w = workloads.get_workload("tiny")
    fmt, ofmt = formats(w)
    lens = workloads.seq_lens(w)
    pairs = [(0, h) for h in range(w.kv_heads)]
    cache = oracle_cache_for_pairs(w, ofmt, pairs, lens)
    q = workloads.query(w)
    want = O.attention_decode(cache, ofmt, q, lens)
    got16, got32 = run_decode(fmt, cache, q, lens, int(w.max_seq), flags)
    plain = np.abs(want) < 2.0
    e16 = np.abs(got16.astype(np.float64) - want)[plain].max()
    e32 = np.abs(got32.astype(np.float64) - want)[plain].max()
    _say("tiny, flags=%d, %d of %d elements with |exact| < 2: worst fp16-output err %.3g, fp32-output err %.3g; max |exact| %.3g"
         % (flags, int(plain.sum()), want.size, e16, e32, np.abs(want).max()))
    assert e16 <= 2e-3 and e32 <= 2e-3


@pytest.mark.parametrize("lens", [[256], [1], [0], [129], [255]])
def test_decode_generic_tiny_ragged(lens):
    w = workloads.get_workload("tiny")
    _say("decode generic tiny lens=%s" % lens)
    _decode_case(w, lens, dq.DECODE_FORCE_GENERIC)


def _small(name, **kw):
    import dataclasses
    return dataclasses.replace(workloads.get_workload(name), **kw)


@pytest.mark.parametrize("name,kw,lens", [
    ("llama7b_4bit", dict(batch=2, q_heads=4, kv_heads=4, max_seq=1000, min_seq=1000), [1000, 257]),
    ("llama7b_2bit", dict(batch=2, q_heads=4, kv_heads=4, max_seq=700, min_seq=700), [700, 128]),
    ("gqa_long", dict(batch=2, q_heads=8, kv_heads=2, max_seq=900, min_seq=900), [900, 5]),
    ("llama13b_mixed", dict(batch=3, q_heads=4, kv_heads=4, max_seq=640, min_seq=1), [640, 0, 383]),
])
def test_decode_generic_multi_block(name, kw, lens):
    w = _small(name, **kw)
    _say("decode generic %s %s lens=%s" % (name, kw, lens))
    worst = _decode_case(w, lens, dq.DECODE_FORCE_GENERIC)
    _say("  worst fp32 abs err %.3g" % worst)


# ------------------------------------------------------------------------------------------
# compress_kv: the GPU's own decomposition, checked through properties
# ------------------------------------------------------------------------------------------
@pytest.mark.parametrize("name,t_new,n_valid", [
    ("tiny", 256, None), ("llama7b_4bit", 128, None), ("llama7b_2bit", 128, None),
    ("llama13b_mixed", 128, [128, 37, 1]), ("gqa_long", 100, None),
])
def test_compress_kv_properties(name, t_new, n_valid):
    w = _small(name, batch=3 if n_valid else 2, q_heads=4, kv_heads=2 if name == "gqa_long" else 4)
    w = _small(name, batch=w.batch, q_heads=w.q_heads, kv_heads=w.kv_heads,
               n_outlier=min(w.n_outlier, 8))
    _say("compress_kv %s t_new=%d n_valid=%s" % (name, t_new, n_valid))
    _check_compress(w, t_new, n_valid)


@pytest.mark.parametrize("seed", [21, 22])
def test_compress_kv_random_cases(seed):
    """Seeded sweep: code widths, group sizes, head dimensions, ragged n_valid (1, a few, full),
    short t_new, skipped sequences, and forced waves-per-block of the decomposition kernel."""
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
        waves = str(rng.choice(["", "1", "2", "4"]))
        w = _small("llama7b_4bit", batch=batch, q_heads=kvh, kv_heads=kvh, head_dim=d, j1=j1, j2=d // j1, bits=bits,
                   group=group, block_tokens=tb, max_seq=tb, min_seq=tb, seed=4000 + 100 * seed + case,
                   n_outlier=int(rng.choice([0, 2, 6])))
        _say("compress_kv random seed %d case %d: d=%d j1=%d bits=%d G=%d Tb=%d B=%d H=%d t_new=%d n_valid=%s waves=%r"
             % (seed, case, d, j1, bits, group, tb, batch, kvh, t_new, n_valid, waves))
        _check_compress(w, t_new, n_valid, waves=int(waves or 0))


def block_properties(arrs, ofmt, x, kp, b, h, slot, which):
    """What the paper fixes about one GPU-compressed block (the factors themselves are not unique):
    x: the block's rows as given (fp64, missing rows zero); kp: the GPU's fp32 large tensor in
    token-major form.  Returns the largest |T_L T_L^T - I| entry."""
    tb, d, j1, j2 = ofmt.block_tokens, ofmt.head_dim, ofmt.j1, ofmt.j2
    small, steps, codes = O.load_block(arrs, ofmt, b, h, slot, which)
    t_l = O.token_major_to_large(kp.astype(np.float64), j1, j2, ofmt.i1)
    # (1) rows of T_L orthonormal (or zero for dropped directions)
    gram = t_l @ t_l.T
    live = np.diag(gram) > 0.5
    ortho = np.abs(gram - np.diag(live.astype(np.float64))).max()
    assert ortho <= 2e-6, (b, h, which, ortho)       # fp32 storage of T_L allows about 1e-6
    # (2) exact factorisation up to the fp16 rounding of T_S and fp32 of T_L (Eq. 3)
    m = O.matricise(x, ofmt.i1, j1)
    resid = np.abs(small.astype(np.float64) @ t_l - m)
    slack = 2.0 ** -10 * (np.abs(small.astype(np.float64)) @ np.abs(t_l)) + 1e-6 * np.abs(m).max() + 1e-7
    assert (resid <= slack).all(), (b, h, which, resid.max())
    # (3) codes and steps are the oracle's quantization of that very T_L (Eq. 1)
    steps_o = O.group_steps(kp, ofmt.group, ofmt.qmax, ofmt.full_range)
    codes_o = O.quantize_codes(kp, steps_o, ofmt.group, ofmt.qmax, ofmt.full_range)
    assert np.array_equal(steps.view(np.uint16), steps_o.view(np.uint16)), (b, h, which)
    assert np.array_equal(codes, codes_o), (b, h, which)
    # (4) reconstruction within the half-step bound
    x_hat = O.reconstruct_block(small, steps, codes, ofmt)
    bound = O.reconstruction_bound(small, steps, ofmt)
    slack_x = O.unmatricise(slack, tb, d, ofmt.i1, j1)
    assert (np.abs(x_hat - x) <= bound + slack_x).all(), (b, h, which)
    return ortho


def _check_compress(w, t_new, n_valid, waves=0):
    assert w.batch <= 3 and w.i3 == 1          # three block slots below; two local tensors
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
    status = int(ws[:4].view(torch.int32).item())
    assert status == 0
    n_large = w.batch * w.kv_heads * 2 * tb * d                     # fp32 large tensors follow the 256-byte header
    large = ws[256:256 + 4 * n_large].view(torch.float32).cpu().numpy().reshape(w.batch * w.kv_heads * 2, tb, d)
    worst_ortho = 0.0
    for b in range(w.batch):
        for h in range(w.kv_heads):
            for which, x_all in (("k", k), ("v", v)):
                slot = int(slots[b])
                if slot < 0:
                    for n in arrs:   # skipped sequence: nothing written anywhere
                        assert np.array_equal(arrs[n][b, h], before[n][b, h].cpu().numpy())
                    continue
                n_ok = t_new if n_valid is None else min(n_valid[b], t_new)
                x = np.zeros((tb, d))
                x[:n_ok] = x_all[b, h, :n_ok].astype(np.float64)
                kp = large[(b * w.kv_heads + h) * 2 + (which == "v")]
                worst_ortho = max(worst_ortho, block_properties(arrs, ofmt, x, kp, b, h, slot, which))
                # (5) other block slots of this head untouched
                for other in range(nb):
                    if other != slot:
                        assert np.array_equal(arrs["k_codes"][b, h, other], before["k_codes"][b, h, other].cpu().numpy())
    _say("  worst |T_L T_L^T - I| = %.3g, sweeps %d" % (worst_ortho, int(ws[4:8].view(torch.int32).item())))


def test_gpu_compressed_cache_decodes_like_its_own_oracle_reading():
    """Compress on the GPU, then decode on the GPU and with the oracle from the same arrays."""
    w = _small("llama7b_4bit", batch=2, q_heads=4, kv_heads=4, max_seq=512, min_seq=512)
    fmt, ofmt = formats(w)
    _say("gpu compress -> gpu decode vs oracle decode")
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
    got16, got32 = run_decode(fmt, arrs, q, lens, 512, dq.DECODE_FORCE_GENERIC)
    assert (np.abs(got16.astype(np.float64) - want) <= tolerance(want)).all()
    # and the lossy cache still approximates attention on the original K, V
    for b in range(w.batch):
        for h in range(w.kv_heads):
            ref = O.dense_attention(q[b, h], k[b, h, :lens[b]], v[b, h, :lens[b]])
            assert np.abs(want[b, h] - ref).max() < 0.15 * np.abs(v[b, h].astype(np.float64)).max()


def test_stream_read_runs():
    src = torch.arange(1 << 20, dtype=torch.int32, device=DEV)
    sink = torch.zeros(4, dtype=torch.int32, device=DEV)
    dq.stream_read(src, sink)
    torch.cuda.synchronize()


# ------------------------------------------------------------------------------------------
# matrix-core decode kernel (4-bit, d = 128, G = 128)
# ------------------------------------------------------------------------------------------
@pytest.mark.parametrize("name,kw,lens", [
    ("llama7b_4bit", dict(batch=2, q_heads=4, kv_heads=4, max_seq=1000, min_seq=1000), [1000, 257]),
    ("llama7b_4bit", dict(batch=3, q_heads=2, kv_heads=2, max_seq=2300, min_seq=2300), [2300, 1, 128]),
    ("gqa_long", dict(batch=2, q_heads=8, kv_heads=2, max_seq=900, min_seq=900), [900, 5]),
    ("gqa_long", dict(batch=2, q_heads=4, kv_heads=2, max_seq=700, min_seq=700), [513, 700]),
    ("llama13b_mixed", dict(batch=3, q_heads=4, kv_heads=4, max_seq=640, min_seq=1), [640, 0, 383]),
    ("llama7b_4bit", dict(batch=1, q_heads=2, kv_heads=2, max_seq=1024, min_seq=1024, block_tokens=256), [777]),
    ("llama7b_2bit", dict(batch=2, q_heads=4, kv_heads=4, max_seq=700, min_seq=700), [700, 128]),
    ("llama7b_2bit", dict(batch=3, q_heads=4, kv_heads=2, max_seq=1300, min_seq=1300), [1300, 0, 257]),
    ("llama7b_2bit", dict(batch=1, q_heads=2, kv_heads=2, max_seq=1024, min_seq=1024, block_tokens=256), [1000]),
    # the other two pairings of code width and group size
    ("llama7b_4bit", dict(batch=2, q_heads=4, kv_heads=2, max_seq=900, min_seq=900, group=64), [900, 130]),
    ("llama7b_2bit", dict(batch=2, q_heads=8, kv_heads=2, max_seq=900, min_seq=900, group=128), [900, 385]),
    # more query heads per kv head than one workgroup takes: head groups
    ("gqa_long", dict(batch=2, q_heads=16, kv_heads=2, max_seq=900, min_seq=900), [900, 130]),       # 2 groups of 4
    ("gqa_long", dict(batch=2, q_heads=6, kv_heads=2, max_seq=700, min_seq=700), [700, 1]),          # 3 heads in a group of 4
    ("gqa_long", dict(batch=1, q_heads=14, kv_heads=2, max_seq=2300, min_seq=2300), [2300]),         # 7 = 4 + 3
    ("llama7b_2bit", dict(batch=2, q_heads=6, kv_heads=2, max_seq=640, min_seq=640), [640, 200]),    # G64: 3 = 2 + 1
    ("llama7b_2bit", dict(batch=2, q_heads=8, kv_heads=2, max_seq=900, min_seq=900), [900, 385]),    # G64: 2 groups of 2
    # 8-bit codes
    ("llama7b_8bit", dict(batch=2, q_heads=4, kv_heads=4, max_seq=1000, min_seq=1000), [1000, 257]),
    ("llama7b_8bit", dict(batch=3, q_heads=8, kv_heads=2, max_seq=1300, min_seq=1300), [1300, 0, 129]),
    ("llama7b_8bit", dict(batch=2, q_heads=4, kv_heads=2, max_seq=640, min_seq=640, group=64, block_tokens=256), [640, 511]),
])
def test_decode_mfma_multi_block(name, kw, lens):
    w = _small(name, **kw)
    fmt, _ = formats(w)
    assert dq.decode_mfma_supported(fmt, w.q_heads, w.kv_heads)
    _say("decode mfma %s %s lens=%s" % (name, kw, lens))
    worst = _decode_case(w, lens, dq.DECODE_FORCE_MFMA)
    _say("  worst fp32 abs err %.3g" % worst)


def test_mfma_path_is_the_default_where_supported_and_rejected_elsewhere():
    fmt4 = dq.Format(4, 128, 128, 16, 8, 128)
    assert dq.decode_mfma_supported(fmt4, 32, 32) and dq.decode_mfma_supported(fmt4, 32, 8)
    assert dq.decode_mfma_supported(dq.Format(2, 64, 128, 16, 8, 128), 32, 32)
    assert dq.decode_mfma_supported(dq.Format(2, 64, 128, 16, 8, 128), 32, 8)      # two head groups of two
    assert dq.decode_mfma_supported(dq.Format(2, 128, 128, 16, 8, 128), 32, 8)
    assert dq.decode_mfma_supported(dq.Format(4, 64, 128, 16, 8, 128), 32, 16)
    assert dq.decode_mfma_supported(dq.Format(4, 128, 128, 16, 8, 128), 64, 8)     # two head groups of four
    assert dq.decode_mfma_supported(dq.Format(4, 128, 128, 16, 8, 128), 24, 8)     # three heads in a workgroup built for four
    assert dq.decode_mfma_supported(dq.Format(4, 128, 128, 16, 8, 128), 34, 2)     # 17 = 4 + 4 + 4 + 4 + 1
    assert not dq.decode_mfma_supported(dq.Format(4, 128, 128, 16, 8, 128), 130, 2)  # seventeen groups
    assert not dq.decode_mfma_supported(dq.Format(4, 32, 128, 16, 8, 128), 32, 32)
    assert dq.decode_mfma_supported(dq.Format(8, 128, 128, 16, 8, 128), 32, 32)
    assert not dq.decode_mfma_supported(dq.Format(8, 32, 128, 16, 8, 128), 32, 32)
    assert dq.decode_mfma_supported(dq.Format(4, 64, 64, 8, 8, 256), 4, 4)          # 64-channel heads ride in pairs
    assert not dq.decode_mfma_supported(dq.Format(4, 64, 64, 8, 8, 256), 3, 3)      # an odd head is left over
    fmt = dq.Format(4, 64, 64, 8, 8, 256)
    cache = dq.alloc_cache(fmt, 1, 3, 1, DEV)
    ws = dq.decode_workspace(fmt, 1, 3, 3, 256, DEV)
    q = torch.zeros((1, 3, 64), dtype=torch.float16, device=DEV)
    with pytest.raises(dq.DQError):
        dq.attn_decode(cache, q, torch.zeros(1, dtype=torch.int32, device=DEV), 256, ws, flags=dq.DECODE_FORCE_MFMA)


def test_decode_full_size_llama7b_sampled_pairs():
    """The benchmark's configuration (batch 8, 32 heads, 4096 tokens, default kernel choice and
    split count): sampled (sequence, head) pairs are oracle-compressed and checked element by
    element; every other pair holds garbage bytes."""
    w = workloads.get_workload("llama7b_4bit")
    fmt, ofmt = formats(w)
    pairs = [(0, 0), (7, 31), (3, 17), (5, 2)]
    _say("decode full-size llama7b_4bit pairs=%s" % pairs)
    lens = workloads.seq_lens(w)
    cache = oracle_cache_for_pairs(w, ofmt, pairs, lens)
    q = workloads.query(w)
    want = O.attention_decode(cache, ofmt, q, lens, pairs=pairs)
    got16, got32 = run_decode(fmt, cache, q, lens, int(w.max_seq), dq.DECODE_AUTO)
    for b, h in pairs:
        e16 = np.abs(got16[b, h].astype(np.float64) - want[b, h])
        assert (e16 <= tolerance(want[b, h])).all(), (b, h, e16.max())
        e32 = np.abs(got32[b, h].astype(np.float64) - want[b, h])
        assert (e32 <= np.maximum(2e-3, 1e-4 * np.abs(want[b, h]))).all(), (b, h, e32.max())
        _say("  pair %s max fp32 err %.3g, max |out| %.3g" % ((b, h), e32.max(), np.abs(want[b, h]).max()))


def _full_size_case(name, pairs, flags=0):
    """Sampled (sequence, kv head) pairs of a full-size workload, default launch configuration.
    Also reports the worst error over the elements with |exact| < 2, where the tolerance is the plain
    2e-3 (the relative branch of the fp16 bound only starts at |exact| = 2.048)."""
    w = workloads.get_workload(name)
    fmt, ofmt = formats(w)
    lens = workloads.seq_lens(w)
    _say("decode full-size %s pairs=%s lens=%s" % (name, pairs, sorted(set(int(x) for x in lens))[:4]))
    cache = oracle_cache_for_pairs(w, ofmt, pairs, lens)
    q = workloads.query(w)
    want = O.attention_decode(cache, ofmt, q, lens, pairs=pairs)
    got16, got32 = run_decode(fmt, cache, q, lens, int(lens.max()), flags)
    rep = w.q_heads // w.kv_heads
    small16, small32, n_small = 0.0, 0.0, 0
    for b, h in pairs:
        for hq in range(h * rep, (h + 1) * rep):
            e16 = np.abs(got16[b, hq].astype(np.float64) - want[b, hq])
            assert (e16 <= tolerance(want[b, hq])).all(), (b, hq, e16.max())
            e32 = np.abs(got32[b, hq].astype(np.float64) - want[b, hq])
            assert (e32 <= np.maximum(2e-3, 1e-4 * np.abs(want[b, hq]))).all(), (b, hq, e32.max())
            plain = np.abs(want[b, hq]) < 2.0
            if plain.any():
                small16, small32, n_small = max(small16, e16[plain].max()), max(small32, e32[plain].max()), n_small + int(plain.sum())
        _say("  pair %s max fp32 err %.3g" % ((b, h), e32.max()))
    assert small16 <= 2e-3 and small32 <= 2e-3
    _say("  where |exact| < 2 (%d elements, plain 2e-3 bound): worst fp16-output err %.3g, worst fp32-output err %.3g"
         % (n_small, small16, small32))


def test_decode_full_size_llama13b_mixed_lengths():
    w = workloads.get_workload("llama13b_mixed")
    lens = workloads.seq_lens(w)
    b_short, b_long = int(np.argmin(lens)), int(np.argmax(lens))
    _full_size_case("llama13b_mixed", [(b_short, 0), (b_long, 39), (1, 20)])


def test_decode_full_size_gqa_long():
    _full_size_case("gqa_long", [(0, 0), (15, 7)])


def test_decode_full_size_llama7b_2bit():
    _full_size_case("llama7b_2bit", [(0, 0), (15, 31)])


def test_decode_full_size_gqa8_long():
    """Eight query heads per kv head at the bench shape: two head groups per (sequence, kv head)."""
    _full_size_case("gqa8_long", [(0, 0), (15, 7)])


# ------------------------------------------------------------------------------------------
# widening: 8-bit codes, identity small tensor (plain group round-to-nearest), graph replay
# ------------------------------------------------------------------------------------------
@pytest.mark.parametrize("bits,group", [(8, 128), (8, 64)])
def test_decode_8bit_generic(bits, group):
    """Section 3.2 names 2/4/8-bit variants of the fused kernel; here 8-bit on the plain fp32 kernel."""
    w = _small("llama7b_4bit", batch=2, q_heads=4, kv_heads=2, max_seq=600, min_seq=600, bits=bits, group=group)
    _say("decode 8-bit G=%d" % group)
    worst = _decode_case(w, [600, 130], dq.DECODE_FORCE_GENERIC)
    _say("  worst fp32 abs err %.3g" % worst)


@pytest.mark.parametrize("name,flags", [("llama7b_4bit", 2), ("llama7b_2bit", 2), ("llama7b_8bit", 2), ("llama7b_4bit", 1)])
def test_identity_small_tensor_is_plain_rtn_attention(name, flags):
    """With T_S = I the cache is plain group round-to-nearest of K and V (the paper's RTN
    baseline, Section 4.1); the same kernels must decode it.  Steps are then as large as the
    data (|x| up to 512), which exercises the kernels' range normalisation."""
    w = _small(name, batch=2, q_heads=4, kv_heads=2, max_seq=520, min_seq=520)
    fmt, ofmt = formats(w)
    lens = np.array([520, 300], np.int32)
    _say("identity small tensor %s flags=%d" % (name, flags))
    cache = O.empty_cache(ofmt, w.batch, w.kv_heads, -(-w.max_seq // w.block_tokens))
    for b in range(w.batch):
        for h in range(w.kv_heads):
            k, v = workloads.kv_pair(w, b, h, int(lens[b]))
            O.compress_sequence(cache, ofmt, b, h, k, v, identity_small=True)
    q = workloads.query(w)
    want = O.attention_decode(cache, ofmt, q, lens)
    got16, got32 = run_decode(fmt, cache, q, lens, 520, flags)
    assert (np.abs(got16.astype(np.float64) - want) <= tolerance(want)).all()
    assert (np.abs(got32.astype(np.float64) - want) <= np.maximum(2e-3, 1e-4 * np.abs(want))).all()


def test_decode_under_graph_capture_replays_identically():
    """The decode call records no memset and allocates nothing, so it can be captured; every
    replay, with eager work and synchronisations in between, must equal the eager result."""
    w = _small("llama7b_4bit", batch=4, q_heads=8, kv_heads=8, max_seq=3000, min_seq=3000)
    fmt, ofmt = formats(w)
    lens = np.array([3000, 1, 1500, 2999], np.int32)
    pairs = [(b, h) for b in range(w.batch) for h in range(w.kv_heads)]
    cache_np = oracle_cache_for_pairs(w, ofmt, pairs[:6], lens)       # six real pairs, rest garbage
    cache = dq.cache_from_numpy(fmt, cache_np, DEV)
    q = torch.from_numpy(workloads.query(w)).to(DEV)
    ld = torch.from_numpy(lens).to(DEV)
    ws = dq.decode_workspace(fmt, w.batch, w.q_heads, w.kv_heads, 3000, DEV)
    eager = dq.attn_decode(cache, q, ld, 3000, ws).clone()
    torch.cuda.synchronize()
    out = torch.empty_like(q)
    stream = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(stream):
        dq.attn_decode(cache, q, ld, 3000, ws, out=out)      # warm-up on the capture stream
        stream.synchronize()
        with torch.cuda.graph(graph, stream=stream):
            dq.attn_decode(cache, q, ld, 3000, ws, out=out)
    torch.cuda.synchronize()
    for rep in range(4):
        out.fill_(float("nan"))
        scratch = torch.randn(1 << 20, device=DEV).sum()     # eager work between replays
        graph.replay()
        torch.cuda.synchronize()
        real = [(b, h) for b, h in pairs[:6]]
        for b, h in real:
            assert torch.equal(out[b, h], eager[b, h]), (rep, b, h)
        del scratch


@pytest.mark.parametrize("i3,q_heads", [(1, 8), (8, 8), (1, 32)])
def test_serving_step_under_graph_capture_replays_identically(i3, q_heads):
    """One serving step as a graph: compress a full block of appended rows into the next slot, then
    decode over blocks + fp16 tail.  Neither call allocates, records a memset or reads a host value
    that changes, so every replay must give the bits of the eager run.  Also with three local
    tensors, and with eight query heads per kv head (two head groups)."""
    w = _small("llama7b_4bit", batch=2, q_heads=q_heads, kv_heads=4, max_seq=768, min_seq=768, i3=i3)
    fmt, ofmt = formats(w)
    nb = 8
    k, v = workloads.kv_tensor(w, 768)
    kd, vd = torch.from_numpy(k).to(DEV), torch.from_numpy(v).to(DEV)
    cache = dq.alloc_cache(fmt, w.batch, w.kv_heads, nb, DEV)
    cws = dq.compress_workspace(fmt, w.batch, w.kv_heads, DEV)
    for blk in range(5):                                   # five blocks already compressed
        sl = slice(blk * 128, (blk + 1) * 128)
        dq.compress_kv(cache, kd[:, :, sl].contiguous(), vd[:, :, sl].contiguous(),
                       torch.full((w.batch,), blk, dtype=torch.int32, device=DEV), None, cws)
    new_k, new_v = kd[:, :, 640:768].contiguous(), vd[:, :, 640:768].contiguous()   # the block being compressed
    slot = torch.full((w.batch,), 5, dtype=torch.int32, device=DEV)
    r = np.random.default_rng(9)
    kt = torch.from_numpy((r.standard_normal((w.batch, w.kv_heads, 128, 128)) * 2).astype(np.float16)).to(DEV)
    vt = torch.from_numpy((r.standard_normal((w.batch, w.kv_heads, 128, 128)) * 2).astype(np.float16)).to(DEV)
    tl = torch.tensor([3, 100], dtype=torch.int32, device=DEV)
    lens = torch.tensor([768, 700], dtype=torch.int32, device=DEV)
    q = torch.from_numpy(workloads.query(w)).to(DEV)
    ws = dq.decode_workspace(fmt, w.batch, w.q_heads, w.kv_heads, 768, DEV)

    def step(out):
        dq.compress_kv(cache, new_k, new_v, slot, None, cws)
        dq.attn_decode(cache, q, lens, 768, ws, out=out, tail=(kt, vt, tl))

    eager = torch.empty_like(q)
    step(eager)
    torch.cuda.synchronize()
    eager_cache = {n: t.clone() for n, t in cache.t.items()}
    out = torch.empty_like(q)
    stream = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(stream):
        step(out)                                            # warm-up on the capture stream
        stream.synchronize()
        with torch.cuda.graph(graph, stream=stream):
            step(out)
    torch.cuda.synchronize()
    for rep in range(3):
        out.fill_(float("nan"))
        for t in cache.t.values():                           # the replay must rewrite slot 5 itself
            t[:, :, 5].zero_()
        scratch = torch.randn(1 << 20, device=DEV).sum()     # eager work between replays
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(out, eager), rep
        for n, t in cache.t.items():
            assert torch.equal(t, eager_cache[n]), (rep, n)
        del scratch


# ------------------------------------------------------------------------------------------
# fp16 residual tail: tokens generated since the last compression (Section 3.2)
# ------------------------------------------------------------------------------------------
@pytest.mark.parametrize("name,kw,lens,tail_lens,flags", [
    ("llama7b_4bit", dict(batch=4, q_heads=4, kv_heads=4, max_seq=1024, min_seq=1024), [1024, 0, 384, 128], [5, 128, 0, 77], 0),
    ("llama7b_4bit", dict(batch=4, q_heads=4, kv_heads=4, max_seq=1024, min_seq=1024), [1024, 0, 384, 128], [5, 128, 0, 77], 1),
    ("gqa_long", dict(batch=2, q_heads=8, kv_heads=2, max_seq=8192, min_seq=8192), [8192, 4096], [100, 1], 0),
    ("llama7b_2bit", dict(batch=2, q_heads=4, kv_heads=4, max_seq=640, min_seq=640), [640, 256], [64, 127], 0),
    ("tiny", dict(), [256], [200], 0),
    # blocks of 512 and 1024 tokens: tails of up to that many rows (one workgroup per pair, and splits)
    ("llama7b_4bit", dict(batch=3, q_heads=4, kv_heads=2, max_seq=1024, min_seq=1024, block_tokens=512), [1024, 512, 0], [511, 300, 512], 0),
    ("llama7b_4bit", dict(batch=3, q_heads=4, kv_heads=2, max_seq=1024, min_seq=1024, block_tokens=512), [1024, 512, 0], [511, 300, 512], 1),
    ("gqa_long", dict(batch=2, q_heads=8, kv_heads=2, max_seq=8192, min_seq=8192, block_tokens=1024), [8192, 1024], [1023, 700], 0),
    ("llama7b_2bit", dict(batch=2, q_heads=2, kv_heads=2, max_seq=2048, min_seq=2048, block_tokens=1024), [2048, 1024], [1024, 1], 0),
    ("llama7b_4bit", dict(batch=2, q_heads=4, kv_heads=4, max_seq=1024, min_seq=1024, block_tokens=512,
                          head_dim=64, j1=8, j2=8, group=64), [1024, 512], [400, 512], 0),
])
def test_decode_with_fp16_tail(name, kw, lens, tail_lens, flags):
    w = _small(name, **kw)
    fmt, ofmt = formats(w)
    lens = np.asarray(lens, np.int32)
    tl = np.asarray(tail_lens, np.int32)
    cap = int(w.block_tokens)
    _say("decode with tail %s lens=%s tail=%s flags=%d" % (name, list(lens), list(tl), flags))
    pairs = [(b, h) for b in range(w.batch) for h in range(w.kv_heads)]
    cache = oracle_cache_for_pairs(w, ofmt, pairs, lens)
    r = np.random.default_rng(5)
    kt = (r.standard_normal((w.batch, w.kv_heads, cap, w.head_dim)) * 2).astype(np.float16)
    vt = (r.standard_normal((w.batch, w.kv_heads, cap, w.head_dim)) * 2).astype(np.float16)
    for b in range(w.batch):            # rows beyond the tail length may hold anything
        kt[b, :, tl[b]:] = np.float16(np.nan)
        vt[b, :, tl[b]:] = np.float16(np.inf)
    q = workloads.query(w)
    want = O.attention_decode(cache, ofmt, q, lens, k_tail=kt, v_tail=vt, tail_lens=tl)
    dcache = dq.cache_from_numpy(fmt, cache, DEV)
    ws = dq.decode_workspace(fmt, w.batch, w.q_heads, w.kv_heads, int(w.max_seq), DEV)
    qd, ld = torch.from_numpy(q).to(DEV), torch.from_numpy(lens).to(DEV)
    tail = (torch.from_numpy(kt).to(DEV), torch.from_numpy(vt).to(DEV), torch.from_numpy(tl).to(DEV))
    o32 = torch.empty((w.batch, w.q_heads, w.head_dim), dtype=torch.float32, device=DEV)
    out = dq.attn_decode(dcache, qd, ld, int(w.max_seq), ws, out_f32=o32, flags=flags, tail=tail)
    # the same workspace then serves a call without tail
    out_plain = dq.attn_decode(dcache, qd, ld, int(w.max_seq), ws, flags=flags)
    torch.cuda.synchronize()
    got16, got32 = out.cpu().numpy().astype(np.float64), o32.cpu().numpy().astype(np.float64)
    assert (np.abs(got16 - want) <= tolerance(want)).all(), np.abs(got16 - want).max()
    assert (np.abs(got32 - want) <= np.maximum(2e-3, 1e-4 * np.abs(want))).all(), np.abs(got32 - want).max()
    want_plain = O.attention_decode(cache, ofmt, q, lens)
    assert (np.abs(out_plain.cpu().numpy().astype(np.float64) - want_plain) <= tolerance(want_plain)).all()


@pytest.mark.parametrize("i3,d", [(1, 128), (8, 128), (1, 64)])
def test_kv_cache_layer_policy_prefill_then_decode_steps(i3, d):
    """Section 3.2 end to end: a ragged prefill goes through the tail, whole blocks are compressed
    as they fill, then single tokens are appended step by step and every decode attends to blocks +
    tail.  Checked against the oracle reading the GPU's own compressed arrays.  i3 = 8: the same
    with three local tensors per block.  d = 64: heads of 64 channels (worked in pairs by the
    matrix-core kernel, tail included)."""
    if d == 128:
        w = _small("llama7b_4bit", batch=2, q_heads=4, kv_heads=2, max_seq=400, min_seq=400, i3=i3)
    else:
        w = _small("llama7b_4bit", batch=2, q_heads=2, kv_heads=2, max_seq=400, min_seq=400, i3=i3,
                   head_dim=64, j1=8, j2=8, group=64)
    fmt, ofmt = formats(w)
    assert dq.decode_mfma_supported(fmt, w.q_heads, w.kv_heads)
    _say("KVCacheLayer policy, i3=%d d=%d" % (i3, d))
    layer = dq.KVCacheLayer(fmt, w.batch, w.q_heads, w.kv_heads, 512, DEV)
    k, v = workloads.kv_tensor(w)                      # [2, 2, 400, d]
    kd, vd = torch.from_numpy(k).to(DEV), torch.from_numpy(v).to(DEV)
    prefill = [300, 130]
    layer.append(kd[:, :, :300].contiguous(), vd[:, :, :300].contiguous(), counts=prefill)
    assert layer.n_blocks == [2, 1] and layer.n_tail == [44, 2]
    q = workloads.query(w)
    qd = torch.from_numpy(q).to(DEV)
    pos = list(prefill)
    for step in range(90):                             # sequence 0 crosses a block boundary at 384
        rows_k = torch.stack([kd[b, :, pos[b]:pos[b] + 1] for b in range(w.batch)])
        rows_v = torch.stack([vd[b, :, pos[b]:pos[b] + 1] for b in range(w.batch)])
        layer.append(rows_k.contiguous(), rows_v.contiguous())
        pos = [p + 1 for p in pos]
        if step in (0, 83, 84, 89):
            out = layer.decode(qd)
            torch.cuda.synchronize()
            arrs = {n: t.cpu().numpy() for n, t in layer.cache.t.items()}
            lens = np.array([nb * 128 for nb in layer.n_blocks], np.int32)
            want = O.attention_decode(arrs, ofmt, q, lens, k_tail=layer.k_tail.cpu().numpy(),
                                      v_tail=layer.v_tail.cpu().numpy(), tail_lens=np.array(layer.n_tail, np.int32))
            got = out.cpu().numpy().astype(np.float64)
            assert (np.abs(got - want) <= tolerance(want)).all(), (step, np.abs(got - want).max())
            # and the blocks hold the right rows: they reconstruct the original K, V to 4-bit accuracy
            for b in range(w.batch):
                for h in range(w.kv_heads):
                    k_hat, v_hat = O.reconstruct_sequence(arrs, ofmt, b, h, int(lens[b]))
                    for x_hat, x in ((k_hat, k[b, h, :lens[b]]), (v_hat, v[b, h, :lens[b]])):
                        x = x.astype(np.float64)
                        assert np.linalg.norm(x_hat - x) < 0.2 * np.linalg.norm(x)
                    nt = layer.n_tail[b]
                    assert np.array_equal(layer.k_tail[b, h, :nt].cpu().numpy(), k[b, h, lens[b]:lens[b] + nt])
    assert layer.n_blocks == [3, 1] and layer.n_tail == [6, 92]


@pytest.mark.parametrize("i3,bits,tb,d", [(1, 4, 128, 128), (8, 4, 128, 128), (1, 2, 256, 128), (8, 8, 128, 128),
                                          (1, 4, 128, 64), (8, 2, 256, 64)])
def test_compress_kv_blocks_writes_what_block_by_block_calls_write(i3, bits, tb, d):
    """A prompt's worth of rows in one call (dq_compress_kv_blocks): every block must come out with
    the very bits that compressing it alone gives, ragged lengths and all; blocks past a sequence's
    rows or past the cache's capacity stay untouched."""
    group = 64 if (bits == 2 or d == 64) else 128
    w = _small("llama7b_4bit", batch=3, q_heads=2, kv_heads=2, bits=bits, group=group, block_tokens=tb,
               head_dim=d, j1=d // 8, j2=8,
               max_seq=4 * tb, min_seq=4 * tb, i3=i3)
    fmt, ofmt = formats(w)
    t_new = 3 * tb + 37                                   # three whole blocks and a short one
    k, v = workloads.kv_tensor(w, t_new)
    kd, vd = torch.from_numpy(k).to(DEV), torch.from_numpy(v).to(DEV)
    n_valid = [t_new, tb + 5, 0]                          # full, ragged, nothing
    first = [0, 1, 2]
    nb = 4                                                # sequence 1: blocks 1, 2 fit; its others have no rows
    _say("compress_kv_blocks i3=%d bits=%d Tb=%d t_new=%d n_valid=%s" % (i3, bits, tb, t_new, n_valid))
    bulk = dq.alloc_cache(fmt, w.batch, w.kv_heads, nb, DEV, fill=0xA5)
    ws = dq.compress_workspace(fmt, w.batch, w.kv_heads, DEV, t_new=t_new)
    dq.compress_kv_blocks(bulk, kd, vd, torch.tensor(first, dtype=torch.int32, device=DEV),
                          torch.tensor(n_valid, dtype=torch.int32, device=DEV), ws)
    torch.cuda.synchronize()
    assert int(ws[:4].view(torch.int32).item()) == 0
    single = dq.alloc_cache(fmt, w.batch, w.kv_heads, nb, DEV, fill=0xA5)
    ws1 = dq.compress_workspace(fmt, w.batch, w.kv_heads, DEV)
    for j in range(4):
        rows = min(tb, t_new - j * tb)
        slots = [first[b] + j if (n_valid[b] - j * tb > 0 and first[b] + j < nb) else -1 for b in range(w.batch)]
        nv = [max(0, min(n_valid[b] - j * tb, rows)) for b in range(w.batch)]
        dq.compress_kv(single, kd[:, :, j * tb:j * tb + rows].contiguous(), vd[:, :, j * tb:j * tb + rows].contiguous(),
                       torch.tensor(slots, dtype=torch.int32, device=DEV), torch.tensor(nv, dtype=torch.int32, device=DEV), ws1)
    torch.cuda.synchronize()
    for name in bulk.t:
        assert torch.equal(bulk.t[name], single.t[name]), name
    # sequence 2 (no valid rows) and the slots nothing was sent to still hold the fill pattern
    assert (bulk.t["k_codes"][2] == 0xA5).all() and (bulk.t["k_codes"][1, :, 0] == 0xA5).all()
    assert (bulk.t["k_codes"][1, :, 3] == 0xA5).all()
    # and the blocks decode like the oracle's reading of them
    arrs = {n: t.cpu().numpy() for n, t in bulk.t.items()}
    q = workloads.query(w)
    lens = np.array([t_new, 0, 0], np.int32)
    want = O.attention_decode(arrs, ofmt, q, lens, pairs=[(0, 0), (0, 1)])
    got16, _ = run_decode(fmt, arrs, q, lens, 4 * tb, dq.DECODE_AUTO)
    assert (np.abs(got16[0].astype(np.float64) - want[0]) <= tolerance(want[0])).all()


def test_kv_cache_layer_prefill_in_one_call_equals_appending():
    w = _small("llama7b_4bit", batch=3, q_heads=4, kv_heads=2, max_seq=700, min_seq=700)
    fmt, _ = formats(w)
    k, v = workloads.kv_tensor(w)
    kd, vd = torch.from_numpy(k).to(DEV), torch.from_numpy(v).to(DEV)
    counts = [700, 130, 90]
    a = dq.KVCacheLayer(fmt, w.batch, w.q_heads, w.kv_heads, 768, DEV)
    b = dq.KVCacheLayer(fmt, w.batch, w.q_heads, w.kv_heads, 768, DEV)
    a.append(kd, vd, counts=counts)
    b.prefill(kd, vd, counts=counts)
    torch.cuda.synchronize()
    assert a.n_blocks == b.n_blocks == [5, 1, 0] and a.n_tail == b.n_tail == [60, 2, 90]
    for name in a.cache.t:
        assert torch.equal(a.cache.t[name], b.cache.t[name]), name
    for bb in range(3):
        assert torch.equal(a.k_tail[bb, :, :a.n_tail[bb]], b.k_tail[bb, :, :b.n_tail[bb]])
    q = torch.from_numpy(workloads.query(w)).to(DEV)
    assert torch.equal(a.decode(q), b.decode(q))


@pytest.mark.parametrize("kw,lens", [
    (dict(bits=4, group=128, q_heads=14, kv_heads=2, batch=2, block_tokens=128, max_seq=1152, min_seq=1152, seed=2027), [128, 128]),
    (dict(bits=8, group=64, q_heads=12, kv_heads=3, batch=3, block_tokens=256, max_seq=256, min_seq=256, seed=2001), [128, 128, 128]),
])
def test_decode_peaked_softmax_keeps_a_margin(kw, lens):
    """Short sequences with outlier channels: two tokens share the weight and their values differ by
    tens, so an error in a score goes to the output at full size.  With three limbs for the folded
    query these two cases sat 5 % over the fp32-output tolerance; with four they must stay under
    half of it."""
    w = _small("llama7b_4bit", **kw)
    fmt, ofmt = formats(w)
    lens = np.asarray(lens, np.int32)
    pairs = [(b, h) for b in range(w.batch) for h in range(w.kv_heads)]
    cache = oracle_cache_for_pairs(w, ofmt, pairs, lens)
    q = workloads.query(w)
    want = O.attention_decode(cache, ofmt, q, lens)
    _, got32 = run_decode(fmt, cache, q, lens, int(w.max_seq), dq.DECODE_FORCE_MFMA)
    ratio = np.abs(got32.astype(np.float64) - want) / np.maximum(2e-3, 1e-4 * np.abs(want))
    _say("peaked softmax %s: worst fp32 error / tolerance %.3f, max |out| %.1f" % (kw, ratio.max(), np.abs(want).max()))
    assert ratio.max() <= 0.5


def test_kv_cache_layer_with_blocks_of_512_tokens():
    """The same policy with blocks of 512 tokens: the fp16 tail grows to 511 rows before it is
    compressed; decode attends to blocks + tail throughout."""
    w = _small("llama7b_4bit", batch=2, q_heads=4, kv_heads=2, max_seq=1024, min_seq=1024, block_tokens=512)
    fmt, ofmt = formats(w)
    _say("KVCacheLayer policy, blocks of 512 tokens")
    layer = dq.KVCacheLayer(fmt, w.batch, w.q_heads, w.kv_heads, 1024, DEV)
    k, v = workloads.kv_tensor(w)                      # [2, 2, 1024, 128]
    kd, vd = torch.from_numpy(k).to(DEV), torch.from_numpy(v).to(DEV)
    prefill = [700, 505]
    layer.append(kd[:, :, :700].contiguous(), vd[:, :, :700].contiguous(), counts=prefill)
    assert layer.n_blocks == [1, 0] and layer.n_tail == [188, 505]
    q = workloads.query(w)
    qd = torch.from_numpy(q).to(DEV)
    pos = list(prefill)
    for step in range(10):                             # sequence 1 fills its first block at 512
        rows_k = torch.stack([kd[b, :, pos[b]:pos[b] + 1] for b in range(w.batch)])
        rows_v = torch.stack([vd[b, :, pos[b]:pos[b] + 1] for b in range(w.batch)])
        layer.append(rows_k.contiguous(), rows_v.contiguous())
        pos = [p + 1 for p in pos]
        if step in (0, 5, 6, 9):
            out = layer.decode(qd)
            torch.cuda.synchronize()
            arrs = {n: t.cpu().numpy() for n, t in layer.cache.t.items()}
            lens = np.array([nb * 512 for nb in layer.n_blocks], np.int32)
            want = O.attention_decode(arrs, ofmt, q, lens, k_tail=layer.k_tail.cpu().numpy(),
                                      v_tail=layer.v_tail.cpu().numpy(), tail_lens=np.array(layer.n_tail, np.int32))
            got = out.cpu().numpy().astype(np.float64)
            assert (np.abs(got - want) <= tolerance(want)).all(), (step, np.abs(got - want).max())
    assert layer.n_blocks == [1, 1] and layer.n_tail == [198, 3]


def test_binding_rejects_tensors_of_the_wrong_size():
    """The library sees pointers only; the binding checks the sizes that go with them."""
    w = _small("llama7b_4bit", batch=3, q_heads=4, kv_heads=2, max_seq=128, min_seq=128)
    fmt, _ = formats(w)
    cache = dq.alloc_cache(fmt, 3, 2, 1, DEV)
    ws = dq.compress_workspace(fmt, 3, 2, DEV)
    k = torch.zeros((3, 2, 128, 128), dtype=torch.float16, device=DEV)
    idx3, idx2 = torch.zeros(3, dtype=torch.int32, device=DEV), torch.zeros(2, dtype=torch.int32, device=DEV)
    with pytest.raises(dq.DQError):
        dq.compress_kv(cache, k, k, idx2, None, ws)                      # one block index short
    with pytest.raises(dq.DQError):
        dq.compress_kv(cache, k, k, idx3, idx2, ws)                      # one row count short
    with pytest.raises(dq.DQError):
        dq.compress_kv(cache, k[:2].contiguous(), k[:2].contiguous(), idx3, None, ws)   # a sequence short
    with pytest.raises(dq.DQError):
        dq.compress_kv(cache, k[:, :, :, :64].contiguous(), k[:, :, :, :64].contiguous(), idx3, None, ws)
    dws = dq.decode_workspace(fmt, 3, 4, 2, 128, DEV)
    q = torch.zeros((3, 4, 128), dtype=torch.float16, device=DEV)
    with pytest.raises(dq.DQError):
        dq.attn_decode(cache, q, idx2, 128, dws)                         # one length short
    with pytest.raises(dq.DQError):
        dq.attn_decode(cache, q[:2].contiguous(), idx3, 128, dws)
    with pytest.raises(dq.DQError):
        dq.attn_decode(cache, q, idx3, 128, dws, tail=(k[:, :, :16].contiguous(), k[:, :, :16].contiguous(), idx2))
    dq.attn_decode(cache, q, idx3, 128, dws)                             # and the right sizes go through
    torch.cuda.synchronize()


@pytest.mark.parametrize("flags", [dq.DECODE_FORCE_MFMA, dq.DECODE_FORCE_GENERIC])
def test_more_sequence_head_pairs_than_a_grid_extent(flags):
    """65 600 (sequence, query head) pairs: beyond the 65 535 rows a launch's y index takes, the rows
    ride on the x index.  Sampled pairs hold oracle-compressed blocks and are compared with the oracle;
    the rest of the cache is zero-filled (every code dequantizes to zero there)."""
    import dataclasses
    batch, heads = 16400, 4
    w = dataclasses.replace(workloads.get_workload("llama7b_4bit"), batch=batch, q_heads=heads, kv_heads=heads,
                            max_seq=128, min_seq=128, seed=9100)
    fmt, ofmt = formats(w)
    _say("decode with %d (sequence, head) pairs, flags=%d" % (batch * heads, flags))
    cache = dq.alloc_cache(fmt, batch, heads, 1, DEV, fill=0)
    sample = [(0, 0), (batch - 1, heads - 1), (8191, 2), (16383, 1), (12345, 3)]
    q = np.zeros((batch, heads, 128), np.float16)
    lens = np.full(batch, 128, np.int32)
    lens[12345] = 77
    want = {}
    r = np.random.default_rng(4)
    for b, h in sample:
        k, v = workloads.kv_pair(w, b, h, 128)
        one = O.empty_cache(ofmt, 1, 1, 1)
        O.compress_sequence(one, ofmt, 0, 0, k, v)
        for name, arr in one.items():
            cache.t[name][b, h] = torch.from_numpy(arr[0, 0]).to(DEV)
        q[b, h] = r.standard_normal(128).astype(np.float16)
        want[b, h] = O.attention_decode(one, ofmt, q[b:b + 1, h:h + 1], lens[b:b + 1])[0, 0]
    ws = dq.decode_workspace(fmt, batch, heads, heads, 128, DEV)
    out = dq.attn_decode(cache, torch.from_numpy(q).to(DEV), torch.from_numpy(lens).to(DEV), 128, ws, flags=flags)
    torch.cuda.synchronize()
    got = out.cpu().numpy().astype(np.float64)
    for b, h in sample:
        assert (np.abs(got[b, h] - want[b, h]) <= tolerance(want[b, h])).all(), (b, h)
    assert np.isfinite(got).all() and np.abs(got[1]).max() == 0.0     # zero-filled pairs give zeros
