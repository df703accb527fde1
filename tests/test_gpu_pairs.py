"""Matrix-core decode for heads of 64 channels (j1 = j2 = 8, one step per row, one query head per
kv head): two neighbouring kv heads are worked as one head of 128 channels.  Parity against the
oracle, element by element, over code widths, block sizes, ragged lengths, forced splits and wave
counts, fp16 tails; the plain kernel on the same inputs as a cross-check of the test itself."""
import dataclasses

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


def _w64(**kw):
    base = dict(head_dim=64, j1=8, j2=8, group=64, i3=1, append_tokens=0)
    base.update(kw)
    w = dataclasses.replace(workloads.get_workload("llama7b_4bit"), **base)
    return dataclasses.replace(w, min_seq=w.max_seq)


def test_which_shapes_pair_up():
    f = dq.Format(4, 64, 64, 8, 8, 128)
    assert dq.decode_mfma_supported(f, 4, 4)
    assert not dq.decode_mfma_supported(f, 3, 3)          # odd number of heads
    assert not dq.decode_mfma_supported(f, 8, 4)          # two query heads per kv head
    assert not dq.decode_mfma_supported(dq.Format(4, 32, 64, 8, 8, 128), 4, 4)       # two steps per row
    assert not dq.decode_mfma_supported(dq.Format(4, 64, 64, 8, 8, 128, 8), 4, 4)    # three local tensors
    assert not dq.decode_mfma_supported(dq.Format(4, 64, 64, 16, 4, 128), 4, 4)      # other factor shapes


@pytest.mark.parametrize("kw,lens", [
    (dict(batch=1, q_heads=4, kv_heads=4, max_seq=256, block_tokens=256, bits=4), [256]),      # the Tiny shape
    (dict(batch=1, q_heads=4, kv_heads=4, max_seq=256, block_tokens=256, bits=4), [129]),
    (dict(batch=2, q_heads=2, kv_heads=2, max_seq=1024, block_tokens=128, bits=4), [1000, 257]),
    (dict(batch=3, q_heads=6, kv_heads=6, max_seq=768, block_tokens=128, bits=4), [768, 0, 1]),
    (dict(batch=2, q_heads=4, kv_heads=4, max_seq=2304, block_tokens=256, bits=4), [2300, 127]),
    (dict(batch=2, q_heads=4, kv_heads=4, max_seq=1152, block_tokens=128, bits=2), [1152, 385]),
    (dict(batch=2, q_heads=2, kv_heads=2, max_seq=1024, block_tokens=256, bits=2), [513, 1024]),
    (dict(batch=2, q_heads=4, kv_heads=4, max_seq=896, block_tokens=128, bits=8), [896, 130]),
    (dict(batch=1, q_heads=2, kv_heads=2, max_seq=512, block_tokens=256, bits=8), [300]),
])
def test_decode_pairs_against_the_oracle(kw, lens):
    w = _w64(**kw)
    fmt, _ = formats(w)
    assert dq.decode_mfma_supported(fmt, w.q_heads, w.kv_heads)
    _say("decode, pairs of 64-channel heads: %s lens=%s" % (kw, lens))
    worst = 0.0
    from test_gpu_parity import _decode_case
    for flags in (dq.DECODE_FORCE_MFMA, dq.DECODE_FORCE_GENERIC):
        worst = max(worst, _decode_case(w, lens, flags))
    _say("  worst fp32 abs err %.3g" % worst)


@pytest.mark.parametrize("seed", [31, 32, 33])
def test_random_pair_cases(seed):
    """Seeded sweep: code widths, block sizes, head counts, ragged lengths, tails, forced launch shapes."""
    rng = np.random.default_rng(seed)
    for case in range(12):
        bits = int(rng.choice([2, 4, 8]))
        kvh, batch = int(rng.choice([2, 4, 6])), int(rng.choice([1, 2, 3]))
        tb = int(rng.choice([128, 256]))
        max_seq = int(rng.choice([128, 300, 640, 1100, 2100]))
        w = _w64(batch=batch, q_heads=kvh, kv_heads=kvh, max_seq=-(-max_seq // tb) * tb, bits=bits, block_tokens=tb,
                 seed=5000 + 100 * seed + case)
        fmt, ofmt = formats(w)
        lens = np.array([int(rng.choice([0, 1, 127, 128, 129, max_seq, int(rng.integers(0, max_seq + 1))]))
                         for _ in range(batch)], np.int32)
        lens = np.minimum(lens, max_seq)
        use_tail = bool(rng.integers(0, 2))
        cap = int(rng.choice([16, 128, 256]))
        tl = np.array([int(rng.choice([0, 1, cap, int(rng.integers(0, cap + 1))])) for _ in range(batch)], np.int32)
        splits, waves = str(rng.choice(["", "1", "2", "3", "5"])), str(rng.choice(["", "4", "8"]))
        shape = dq.decode_flags(splits=int(splits or 0), waves=int(waves or 0))   # launch-shape overrides in the flags word
        _say("seed %d case %d: bits=%d kvh=%d B=%d Tb=%d max_seq=%d lens=%s tail=%s cap=%d tl=%s splits=%r waves=%r"
             % (seed, case, bits, kvh, batch, tb, max_seq, lens.tolist(), use_tail, cap, tl.tolist(), splits, waves))
        pairs = [(b, h) for b in range(batch) for h in range(kvh)]
        cache = oracle_cache_for_pairs(w, ofmt, pairs, lens, seed=case)
        q = workloads.query(w)
        kt = (rng.standard_normal((batch, kvh, cap, 64)) * 2).astype(np.float16)
        vt = (rng.standard_normal((batch, kvh, cap, 64)) * 2).astype(np.float16)
        for b in range(batch):            # rows beyond the tail length may hold anything
            kt[b, :, tl[b]:] = np.float16(np.nan)
            vt[b, :, tl[b]:] = np.float16(np.inf)
        if use_tail:
            want = O.attention_decode(cache, ofmt, q, lens, k_tail=kt, v_tail=vt, tail_lens=tl)
        else:
            want = O.attention_decode(cache, ofmt, q, lens)
        dcache = dq.cache_from_numpy(fmt, cache, DEV)
        ws = dq.decode_workspace(fmt, batch, kvh, kvh, max_seq, DEV)
        qd, ld = torch.from_numpy(q).to(DEV), torch.from_numpy(lens).to(DEV)
        tail = (torch.from_numpy(kt).to(DEV), torch.from_numpy(vt).to(DEV), torch.from_numpy(tl).to(DEV)) if use_tail else None
        o32 = torch.empty((batch, kvh, 64), dtype=torch.float32, device=DEV)
        out = dq.attn_decode(dcache, qd, ld, max_seq, ws, out_f32=o32, flags=dq.DECODE_FORCE_MFMA | shape, tail=tail)
        again = dq.attn_decode(dcache, qd, ld, max_seq, ws, flags=dq.DECODE_FORCE_MFMA | shape, tail=tail)   # counters left clean
        torch.cuda.synchronize()
        g16, g32 = out.cpu().numpy().astype(np.float64), o32.cpu().numpy().astype(np.float64)
        assert torch.equal(out, again), (seed, case)
        assert (np.abs(g16 - want) <= tolerance(want)).all(), (seed, case, np.nanmax(np.abs(g16 - want)))
        assert (np.abs(g32 - want) <= np.maximum(2e-3, 1e-4 * np.abs(want))).all(), (seed, case)


@pytest.mark.parametrize("bits", [2, 4, 8])
def test_a_head_does_not_depend_on_its_partner(bits):
    """Only one head of each pair holds a cache; its partner's arrays are garbage bytes with NaN and
    Inf among the steps and small tensors.  The valid heads must come out as if they were alone."""
    w = _w64(batch=2, q_heads=4, kv_heads=4, max_seq=640, block_tokens=128, bits=bits)
    from test_gpu_parity import _decode_case
    _say("pairs with a garbage partner, %d-bit" % bits)
    kept = [(0, 0), (0, 3), (1, 1), (1, 2)]
    _decode_case(w, [640, 300], dq.DECODE_FORCE_MFMA, pairs=kept)
    # and bit for bit what they are when the partners hold caches of their own
    fmt, ofmt = formats(w)
    lens = np.array([640, 300], np.int32)
    q = workloads.query(w)
    everyone = [(b, h) for b in range(w.batch) for h in range(w.kv_heads)]
    alone, _ = run_decode(fmt, oracle_cache_for_pairs(w, ofmt, kept, lens), q, lens, int(w.max_seq), dq.DECODE_FORCE_MFMA)
    full, _ = run_decode(fmt, oracle_cache_for_pairs(w, ofmt, everyone, lens), q, lens, int(w.max_seq), dq.DECODE_FORCE_MFMA)
    for b, h in kept:
        assert np.array_equal(alone[b, h].view(np.uint16), full[b, h].view(np.uint16)), (b, h)


def test_decode_full_size_64_channel_heads():
    """The opt_d64_4bit bench configuration (batch 16, 32 heads, 4096 tokens, default launch shape):
    sampled (sequence, head) pairs are oracle-compressed and checked element by element; every other
    head, the partners of three of the sampled ones among them, holds garbage bytes."""
    from test_gpu_parity import _full_size_case
    _full_size_case("opt_d64_4bit", [(0, 0), (15, 31), (7, 12), (7, 13), (3, 17)])


# ------------------------------------------------------------------------------------------
# compression of 64-channel heads: two heads per workgroup of the tuned decomposition kernel
# ------------------------------------------------------------------------------------------
@pytest.mark.parametrize("bits,kvh,tb,waves", [(4, 2, 128, ""), (2, 6, 256, "1"), (8, 4, 128, "2"), (4, 4, 256, "4")])
def test_compress_pairs_properties(bits, kvh, tb, waves):
    """Exact product, orthonormal rows of the large tensor, codes and steps equal to the oracle's
    quantizer on the GPU's large tensor, untouched neighbours: the checks every compression test
    runs, on shapes that go through the paired kernel, full and ragged."""
    from test_gpu_parity import _check_compress
    w = _w64(batch=3, q_heads=kvh, kv_heads=kvh, max_seq=tb, block_tokens=tb, bits=bits, n_outlier=2)
    _say("compress_kv, pairs of 64-channel heads: bits=%d H=%d Tb=%d waves=%r" % (bits, kvh, tb, waves))
    _check_compress(w, tb, [tb, 37, 1], waves=int(waves or 0))
    _check_compress(w, tb - 5, None, waves=int(waves or 0))


def test_compress_pairs_heads_of_very_different_size():
    """A head a hundred thousand times smaller than its partner is decomposed as well as alone: the
    rows of its large tensor are orthonormal and the product gives the block back."""
    fmt, ofmt = dq.Format(4, 64, 64, 8, 8, 128), O.Format(4, 64, 64, 8, 8, 128)
    r = np.random.default_rng(77)
    k = r.standard_normal((1, 2, 128, 64)).astype(np.float32)
    k[0, 1] *= 1e-5 * 3                                        # fp16 values around 3e-5: subnormal steps and all
    k[0, 0, :, 5] *= 20
    k = k.astype(np.float16)
    cache = dq.alloc_cache(fmt, 1, 2, 1, DEV)
    ws = dq.compress_workspace(fmt, 1, 2, DEV)
    kd = torch.from_numpy(k).to(DEV)
    dq.compress_kv(cache, kd, kd, torch.zeros(1, dtype=torch.int32, device=DEV), None, ws)
    torch.cuda.synchronize()
    large = ws[256:256 + 4 * 4 * 128 * 64].view(torch.float32).cpu().numpy().reshape(4, 128, 64)
    small = cache.t["k_small"].cpu().numpy()
    for h in range(2):
        t_l = O.token_major_to_large(large[2 * h].astype(np.float64), 8, 8)        # [8, 128 * 8]
        gram = t_l @ t_l.T
        assert np.abs(gram - np.eye(8)).max() <= 1e-5, (h, np.abs(gram - np.eye(8)).max())
        m = O.matricise(k[0, h].astype(np.float64), 1, 8)
        t_s = small[0, h, 0].astype(np.float64).T                                   # keys are stored transposed
        assert np.linalg.norm(t_s @ t_l - m) <= 2e-3 * np.linalg.norm(m), h         # fp16 small tensor, fp32 large
