"""Helpers shared by the GPU parity tests (input staging only, no method arithmetic)."""
import numpy as np
import torch

from oracle import decoquant_oracle as O
import paper_2405_12591_amd as dq

DEV = "cuda:0"


def formats(w):
    args = (w.bits, w.group, w.head_dim, w.j1, w.j2, w.block_tokens, w.i3, w.levels, w.i1)
    return dq.Format(*args), O.Format(*args)


def oracle_cache_for_pairs(w, ofmt, pairs, lens, poison=True, seed=0):
    """Oracle-compress the listed (b, h) pairs up to lens[b]; everything else is garbage bytes
    (when poison) so that a kernel reading beyond seq_len or into unused blocks is caught."""
    nb = -(-w.max_seq // w.block_tokens)
    cache = O.empty_cache(ofmt, w.batch, w.kv_heads, nb)
    if poison:
        r = np.random.default_rng(seed)
        for name, arr in cache.items():
            raw = arr.view(np.uint8)
            raw[...] = r.integers(0, 256, size=raw.shape, dtype=np.uint8)
            if arr.dtype == np.float16:   # make sure NaN/Inf patterns are present
                arr.reshape(-1)[::7] = np.float16(np.nan)
                arr.reshape(-1)[3::11] = np.float16(np.inf)
    import workloads
    for b, h in pairs:
        n = int(lens[b])
        k, v = workloads.kv_pair(w, b, h, n)
        if n:
            O.compress_sequence(cache, ofmt, b, h, k, v)
            if poison:
                _poison_tail(cache, ofmt, b, h, n, r)
    return cache


def _poison_tail(cache, ofmt, b, h, n, r):
    """Overwrite the rows >= n of the last block (codes and steps) with garbage."""
    tb = ofmt.block_tokens
    blk, row = (n - 1) // tb, (n - 1) % tb + 1
    row = -(-row // ofmt.i3) * ofmt.i3   # three tensors: the rows of a run with a valid token all count
    if ofmt.i1 > 1:
        return                           # a token factor: every row of a block with a valid token counts
    if row >= tb:
        return
    cache["k_codes"][b, h, blk, row:] = r.integers(0, 256, size=cache["k_codes"][b, h, blk, row:].shape, dtype=np.uint8)
    cache["k_scales"][b, h, blk, row:] = np.float16(np.nan)
    cache["v_scales"][b, h, blk, row:] = np.float16(np.inf)
    # value codes are token-contiguous: poison the fields of tokens >= row
    vc = O.unpack_rows(cache["v_codes"][b, h, blk], ofmt.bits)          # [tile, b2, r, 128]
    flat = vc.reshape(vc.shape[0], vc.shape[1], vc.shape[2], O.TILE_TOKENS)
    qmax = ofmt.qmax
    for tile in range(flat.shape[0]):
        lo = max(row - tile * O.TILE_TOKENS, 0)
        if lo < O.TILE_TOKENS:
            flat[tile, :, :, lo:] = r.integers(-qmax, qmax + 1, size=flat[tile, :, :, lo:].shape)
    cache["v_codes"][b, h, blk] = O.pack_rows(flat, ofmt.bits)


def tolerance(want):
    """max(2e-3, |want| * 2^-10): 2e-3 absolute, or just under one fp16 ulp of the exact result
    where that is larger (an fp16 output cannot be closer than half an ulp)."""
    return np.maximum(2e-3, np.abs(want) * 2.0 ** -10)


def run_decode(fmt, cache_arrays, q, lens, max_seq, flags=0, want_f32=True):
    cache = dq.cache_from_numpy(fmt, cache_arrays, DEV)
    bsz, hq, d = q.shape
    ws = dq.decode_workspace(fmt, bsz, hq, cache.kv_heads, max_seq, DEV)
    qd = torch.from_numpy(q).to(DEV)
    ld = torch.from_numpy(lens.astype(np.int32)).to(DEV)
    o32 = torch.full((bsz, hq, d), float("nan"), dtype=torch.float32, device=DEV) if want_f32 else None
    out = dq.attn_decode(cache, qd, ld, max_seq, ws, out_f32=o32, flags=flags)
    # second call on the same workspace must give the same bits (counters are left clean)
    out2 = dq.attn_decode(cache, qd, ld, max_seq, ws, flags=flags)
    torch.cuda.synchronize()
    assert torch.equal(out, out2)
    return out.cpu().numpy(), (o32.cpu().numpy() if want_f32 else None)
