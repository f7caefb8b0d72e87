"""Host-side check of the generated code of the persistent grouped-GEMM kernel (no GPU needed).

The kernel orders its LDS DMA loads with hand-placed ``s_waitcnt vmcnt(N)`` in inline assembly, which the
compiler does not see.  If the compiler believes that an ordinary global load is still pending when the
main loop starts (an epilogue load that some path leaves unconsumed, say), it adds waits of its own inside
the loop; they wait for the DMA loads too and cost 15-20 % of the kernel, silently.  So: compile the
kernels to assembly and look at every basic block of the main loops.
"""
import os
import re
import shutil
import subprocess

import pytest

from paper_2602_11686_amd import build as B

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
pytestmark = pytest.mark.skipif(shutil.which(HIPCC) is None, reason="hipcc not installed")


@pytest.fixture(scope="module")
def ffn_asm(tmp_path_factory):
    out = tmp_path_factory.mktemp("asm") / "moe_ffn.s"
    cmd = [HIPCC, *B.FLAGS, "-S", "--cuda-device-only", os.path.join(B.CSRC, "moe_ffn.hip"), "-o", str(out)]
    r = subprocess.run(cmd, capture_output=True, text=True)
    assert r.returncode == 0, r.stderr[-2000:]
    return out.read_text()


def kernels(asm):
    """{mangled kernel name: [(block label, [instructions])]} for the gg256 kernels."""
    out, kern, label, cur = {}, None, None, []
    for line in asm.split("\n"):
        m = re.match(r"^(_ZN3moe12gg256_kernel\w+):", line)
        if m:
            kern, label, cur = m.group(1), "entry", []
            out[kern] = [(label, cur)]
            continue
        if kern is None:
            continue
        if re.match(r"^\s*\.(size|end_amdhsa_kernel|section)", line) or re.match(r"^_Z\w+:", line):
            kern = None
            continue
        m = re.match(r"^(\.LBB\d+_\d+):", line)
        if m:
            label, cur = m.group(1), []
            out[kern].append((label, cur))
            continue
        t = line.strip()
        if t and not t.startswith(";") and not t.startswith("."):
            cur.append(t)
    return out


def test_main_loops_hold_only_the_hand_placed_vmcnt_waits(ffn_asm):
    ks = kernels(ffn_asm)
    assert len(ks) >= 6, sorted(ks)
    seen_loops = 0
    for name, blocks in ks.items():
        for label, ins in blocks:
            mfma = sum(i.startswith("v_mfma") for i in ins)
            if mfma < 8 or not any("s_barrier" in i for i in ins):
                continue  # not a main-loop block (a stage = MFMAs around one barrier)
            seen_loops += 1
            waits = [int(re.search(r"vmcnt\((\d+)\)", i).group(1)) for i in ins
                     if i.startswith("s_waitcnt") and "vmcnt" in i]
            # the one wait of a stage lets the two youngest stages (8 DMA loads per wavefront) stay in flight
            assert waits == [8], f"{name} {label}: vmcnt waits {waits} inside a main-loop stage"
    assert seen_loops >= len(ks)


def test_kernels_do_not_spill(ffn_asm):
    for m in re.finditer(r"\.amdhsa_kernel (_ZN3moe12gg256_kernel\w+)(.*?)\.end_amdhsa_kernel", ffn_asm, re.S):
        body = m.group(2)
        scratch = re.search(r"\.amdhsa_private_segment_fixed_size (\d+)", body)
        assert scratch and int(scratch.group(1)) == 0, (m.group(1), scratch and scratch.group(1))
        vgpr = re.search(r"\.amdhsa_next_free_vgpr (\d+)", body)
        assert vgpr and int(vgpr.group(1)) <= 256, (m.group(1), vgpr and vgpr.group(1))
