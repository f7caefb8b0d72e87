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
            waits = [(n, int(re.search(r"vmcnt\((\d+)\)", i).group(1))) for n, i in enumerate(ins)
                     if i.startswith("s_waitcnt") and "vmcnt" in i]
            # the one wait of a stage sits right in front of its barrier: the next stage has landed, and since
            # the stage after it is requested only behind the barrier, nothing else is in flight
            assert [w for _, w in waits] == [0], f"{name} {label}: vmcnt waits {waits} inside a main-loop stage"
            bar = next(n for n, i in enumerate(ins) if "s_barrier" in i)
            between = [i for i in ins[waits[0][0] + 1:bar] if i.startswith(("ds_read", "global_load", "buffer_load"))]
            assert 0 < bar - waits[0][0] and not between, f"{name} {label}: the wait is not the one in front of the barrier"
    assert seen_loops >= len(ks)


def test_look_ahead_draw_is_first_read_behind_a_full_wait(ffn_asm):
    """The queue draw for the next tile is a returning atomic issued from inline assembly; its result arrives
    asynchronously.  The only reader of the destination register must be the LDS store that publishes it, and
    that store must follow an s_waitcnt vmcnt(0) in its own straight-line code."""
    found = 0
    for m in re.finditer(r"^(_ZN3moe12gg256_kernel\w+Lb1EEEvNS_5GArgsE):(.*?)\n\s*s_endpgm", ffn_asm, re.S | re.M):
        lines = [l.strip() for l in m.group(2).split("\n")]
        lines = [l for l in lines if l and not l.startswith(";") and (not l.startswith(".") or l.startswith(".LBB"))]
        for n, l in enumerate(lines):
            a = re.match(r"global_atomic_add (v\d+), v\[\d+:\d+\], v\d+, off sc0", l)
            if not a:
                continue
            found += 1
            reg = a.group(1)
            word = re.compile(r"\b%s\b" % reg)
            readers = []
            for k in range(n + 1, len(lines)):
                x = lines[k]
                if not word.search(x):
                    continue
                if re.match(r"\S+ %s\b" % reg, x) and not x.startswith(("ds_write", "global_store", "buffer_store")):
                    break          # the register gets a new value: the draw's life ends here
                readers.append((k, x))
            assert readers, (m.group(1), "the draw is never read")
            for k, x in readers:
                assert re.match(r"ds_write_b32 v\d+, %s$" % reg, x), (m.group(1), x)
                back = lines[max(0, k - 40):k]
                labels = [i for i, y in enumerate(back) if y.startswith(".LBB")]
                straight = back[labels[-1] + 1:] if labels else back
                # the wait may sit in the block in front of the predicated store: look through one label
                window = straight if any("vmcnt(0)" in y for y in straight) else back
                assert any(y.startswith("s_waitcnt") and "vmcnt(0)" in y for y in window), (m.group(1), x)
    assert found >= 2   # the two weight-gradient kernels draw their tiles


def test_kernels_do_not_spill(ffn_asm):
    for m in re.finditer(r"\.amdhsa_kernel (_ZN3moe12gg256_kernel\w+)(.*?)\.end_amdhsa_kernel", ffn_asm, re.S):
        body = m.group(2)
        scratch = re.search(r"\.amdhsa_private_segment_fixed_size (\d+)", body)
        assert scratch and int(scratch.group(1)) == 0, (m.group(1), scratch and scratch.group(1))
        vgpr = re.search(r"\.amdhsa_next_free_vgpr (\d+)", body)
        assert vgpr and int(vgpr.group(1)) <= 256, (m.group(1), vgpr and vgpr.group(1))
