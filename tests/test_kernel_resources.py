"""The compiler's report on the kernels of the in-tree build: no kernel of the streaming paths may
keep data in scratch memory (a stack object or a register spill there costs a large part of the
bandwidth these kernels are bound by)."""
import json
import os

from paper_2405_12591_amd import build as B


def _resources():
    if not os.path.exists(B.RESOURCES_PATH):
        B.build_library()
    with open(B.RESOURCES_PATH) as f:
        return json.load(f)


def test_no_scratch_in_the_streaming_kernels():
    res = _resources()
    decode = {k: v for k, v in res.items() if "decode_mfma_kernel" in k}
    assert len(decode) >= 100            # every (bits, groups, heads, waves, tail mode, tensors, head pairing) instance
    for name, r in res.items():
        if any(s in name for s in ("decode_mfma_kernel", "decompose16_kernel", "quantize_tiles_kernel",
                                   "quantize_pack_kernel", "split3_kernel", "stream_read_kernel")):
            assert r["ScratchSize"] == 0 and r["VGPRs Spill"] == 0, (name, r)


def test_occupancy_the_launch_shapes_count_on():
    import re
    res = _resources()
    seen = 0
    for name, r in res.items():
        m = re.search(r"decode_mfma_kernelILi(\d)ELi(\d)ELi(\d)ELi(\d)ELi(\d)ELb([01])ELb([01])E", name)
        if not m:
            continue
        seen += 1
        bits, _, _, waves, _, _, _ = (int(x) for x in m.groups())
        assert r["LDS Size"] <= 160 * 1024, (name, r)
        if bits < 8 and waves == 4:
            # these workgroups run two to a compute unit: two waves per SIMD share its 512 registers
            assert r["VGPRs"] + r["AGPRs"] <= 256 and r["LDS Size"] <= 80 * 1024, (name, r)
    assert seen >= 100
