"""Build-time checks of the draft kernels' machine code (hipcc only, no GPU).

No instantiation may spill vector registers: the in-flight tile windows live in registers, and
a spilled window turns the weight stream into scratch-memory traffic (measured once: 36.8 us
instead of 29.6 us per call on the phi shape with 12 spilled registers).

The streaming kernel copies scale / zero entries into LDS with loads issued from inline assembly
that set the M0 register themselves; the compiler is not told, so nothing else in those kernels
may depend on M0."""
import os
import re
import subprocess
import tempfile

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _assembly(name):
    from paper_2511_14102_amd import build as B
    src = os.path.join(B.CSRC, name)
    with tempfile.TemporaryDirectory() as tmp:
        out = os.path.join(tmp, name + ".s")
        cmd = [B.HIPCC] + B.FLAGS + ["--cuda-device-only", "-S", src, "-o", out]
        r = subprocess.run(cmd, capture_output=True, text=True)
        assert r.returncode == 0, r.stderr[-2000:]
        return open(out).read()


def _kernel_blocks(text, kernel):
    """Metadata blocks (one per kernel, after '.name:') of the instantiations of `kernel`."""
    return [blk for blk in text.split(".name:")[1:] if kernel in blk.split("\n", 1)[0]]


def test_draft_kernel_instantiations_do_not_spill():
    checked = 0
    for src, kernel, expect in (("draft_int4.hip", "draft_stream_kernel", 18),     # 3 token capacities x 3 group sizes x 2 formats
                                ("draft_slice.hip", "draft_fused_kernel", 6),      # one token: 3 group sizes x 2 formats
                                ("draft_prefill.hip", "prefill_tile_kernel", 4)):  # (gate/up, down) x 2 formats
        text = _assembly(src)
        blocks = _kernel_blocks(text, kernel)
        assert len(blocks) >= expect, (src, len(blocks))
        for blk in blocks:
            m = re.search(r"\.vgpr_spill_count:\s+(\d+)", blk)
            assert m is not None
            assert int(m.group(1)) == 0, blk.split("\n", 1)[0].strip()
            checked += 1
    assert checked >= 28


def test_streaming_kernel_uses_m0_only_for_its_loads_to_lds():
    text = _assembly("draft_int4.hip")
    body = text.split("draft_stream_kernel", 1)[1]
    uses = [l.strip() for l in body.splitlines() if re.search(r"\bm0\b", l) and not l.strip().startswith(";")]
    assert uses, "the loads to LDS are gone?"
    for l in uses:
        assert l.startswith("s_mov_b32 m0,"), l
    assert "global_load_lds_dwordx4" in body
