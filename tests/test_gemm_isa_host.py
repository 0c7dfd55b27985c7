"""Host-side check of the compiled many-row projection loops (no GPU).

The main loop of the kernels with 256-row tiles or taller issues its LDS operand reads and MFMAs as inline assembly
and places the `s_waitcnt` for the reads by hand, because the compiler's own wait insertion would serialise reads and
MFMAs.  The compiler therefore believes that a read's result is in its registers as soon as the instruction has been
issued.  That is harmless as long as nothing but an MFMA after the hand-placed wait touches those registers - and
wrong, silently, if the register allocator ever decides to copy or spill one in between.  This test compiles the source
to gfx950 assembly and requires that the loops contain no register-to-register copy, no accumulation-register traffic
and no spill; it also pins the instruction counts per stage, so a change that unrolls or duplicates the loop body
shows up here first."""
import os
import re
import subprocess
from collections import Counter

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "paper_2605_21603_amd", "csrc", "kernels_gemm.hip")
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
MFMA = "v_mfma_f32_16x16x32_bf16"


@pytest.fixture(scope="module")
def kernels(tmp_path_factory):
    if not os.path.exists(HIPCC):
        pytest.skip("no ROCm toolchain")
    from paper_2605_21603_amd.build import FLAGS
    out = str(tmp_path_factory.mktemp("isa") / "kernels_gemm.s")
    flags = [f for f in FLAGS if f != "-fPIC"]
    subprocess.check_call([HIPCC] + flags + ["-S", "--cuda-device-only", SRC, "-o", out], stderr=subprocess.DEVNULL)
    lines = open(out).read().split("\n")
    starts = [i for i, l in enumerate(lines) if re.match(r"^_ZN3dyn16gemm_bf16_kernel\S*:", l)]
    found = {}
    for n, i in enumerate(starts):
        m = re.search(r"kernelILi(\d+)ELi(\d+)ELb(\d)ELi(\d+)ELb(\d)ELi(\d+)E", lines[i])
        key = tuple(int(x) for x in m.groups())           # BN, MT, INREG, NS, GATED, NW
        found[key] = lines[i:starts[n + 1] if n + 1 < len(starts) else len(lines)]
    return found


def hand_laid_loop(body):
    """Instructions from the head of the loop that holds the assembly MFMAs to the last of them."""
    asm = [j for j, x in enumerate(body) if MFMA in x and "ASMSTART" in body[j - 1]]
    if not asm:
        return None
    head = max([j for j, x in enumerate(body) if "Loop Header" in x and j < asm[0]] or [asm[0]])
    return [x.strip().split()[0] for x in body[head:asm[-1] + 1] if x.strip() and x.strip()[0] not in ";."]


def test_the_kernels_with_256_row_tiles_use_the_hand_laid_loop_and_the_others_do_not(kernels):
    assert len(kernels) >= 12
    for key, body in kernels.items():
        bn, mt, inreg, ns, gated, nw = key
        assert (hand_laid_loop(body) is not None) == (mt >= 256), key


def test_no_copy_spill_or_accumulation_register_traffic_between_a_read_and_its_wait(kernels):
    checked = 0
    for key, body in kernels.items():
        loop = hand_laid_loop(body)
        if loop is None:
            continue
        bn, mt, inreg, ns, gated, nw = key
        c = Counter(loop)
        copies = {k: v for k, v in c.items() if k.startswith(("v_mov", "v_accvgpr", "scratch_", "buffer_store", "buffer_load", "v_swap", "v_perm", "v_readlane", "v_writelane"))}
        assert not copies, (key, copies)
        # one stage: the wave's output tiles times two k halves of MFMAs, and every operand tile read exactly once per k half
        wmw = 4 if (nw == 8 and bn < mt) else 2
        na, nb = bn // (nw // wmw) // 16, mt // (16 * wmw)
        assert c[MFMA] == 2 * na * nb, (key, c[MFMA])
        assert c["ds_read_b128"] == 2 * (na + nb), (key, c["ds_read_b128"])
        assert c["s_barrier"] == 1, key
        checked += 1
    assert checked >= 6
