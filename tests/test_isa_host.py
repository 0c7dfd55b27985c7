"""Host-side checks of the compiled loops that place their own waits (no GPU).

The many-row projection loops and the prefill attention's tile loop issue their LDS operand reads as inline assembly
and place the `s_waitcnt` for them by hand, because the compiler's own wait insertion would serialise reads and matrix
products.  The compiler therefore believes that a read's result is in its registers as soon as the instruction has been
issued.  That is harmless only as long as no instruction touches those registers before the hand-placed wait has retired
the read - and wrong, silently, if the register allocator ever copies or spills one in between, or if a wait count is
off by one.  These tests compile the sources to gfx950 assembly and replay the LDS counter over each loop (LDS
operations retire in issue order; `s_waitcnt lgkmcnt(N)` leaves the N most recent outstanding): every instruction that
names a register of a read that may still be in flight is a failure.  They also pin the instruction counts per stage,
so a change that unrolls or duplicates a loop body shows up here first."""
import os
import re
import subprocess
from collections import Counter

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2605_21603_amd", "csrc")
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
MFMA = "v_mfma_f32_16x16x32_bf16"


def compile_to_isa(tmp, source):
    if not os.path.exists(HIPCC):
        pytest.skip("no ROCm toolchain")
    from paper_2605_21603_amd.build import FLAGS
    out = os.path.join(str(tmp), source + ".s")
    flags = [f for f in FLAGS if f != "-fPIC"]
    subprocess.check_call([HIPCC] + flags + ["-S", "--cuda-device-only", os.path.join(CSRC, source), "-o", out], stderr=subprocess.DEVNULL)
    return open(out).read().split("\n")


def instructions(lines):
    return [x.strip() for x in lines if x.strip() and x.strip()[0] not in ";."]


def registers(operand_text):
    """Vector registers named in an operand list: v7 -> {7}, v[12:15] -> {12..15}."""
    regs = set()
    for a, b in re.findall(r"\bv\[(\d+):(\d+)\]", operand_text):
        regs.update(range(int(a), int(b) + 1))
    for a in re.findall(r"\bv(\d+)\b", operand_text):
        regs.add(int(a))
    return regs


def replay_lds_counter(loop_lines):
    """Walks the loop's text twice (so that reads issued at its end meet their consumers at its start) and returns
    the instructions that name a register of an assembly read that a wait has not yet retired."""
    hand_reads = set()
    marked = []
    for i, x in enumerate(loop_lines):
        s = x.strip()
        if s.startswith("ds_read") and i > 0 and "ASMSTART" in loop_lines[i - 1]:
            hand_reads.add(i)
        if s and s[0] not in ";.":
            marked.append((i, s))
    pending = []               # in issue order: the destination registers of a hand-placed read, or an empty set for any other LDS / scalar-memory operation
    violations = []
    for rep in range(2):
        for i, s in marked:
            op, _, rest = s.partition(" ")
            if op == "s_waitcnt":
                m = re.search(r"lgkmcnt\((\d+)\)", rest)
                if m:
                    keep = int(m.group(1))
                    pending = pending[len(pending) - keep:] if keep else []
                continue
            if op == "s_barrier":
                continue
            in_flight = set().union(*pending) if pending else set()
            if i in hand_reads:
                dst, _, addr = rest.partition(",")
                if registers(addr.split("offset")[0]) & in_flight:
                    violations.append(s)
                pending.append(registers(dst))
                continue
            if in_flight and registers(rest) & in_flight:
                violations.append(s)
            if op.startswith("ds_") or op.startswith("s_load") or op.startswith("s_buffer_load"):
                pending.append(set())
    return violations, len(hand_reads)


@pytest.fixture(scope="module")
def gemm_kernels(tmp_path_factory):
    lines = compile_to_isa(tmp_path_factory.mktemp("isa_gemm"), "kernels_gemm.hip")
    starts = [i for i, l in enumerate(lines) if re.match(r"^_ZN3dyn16gemm_bf16_kernel\S*:", l)]
    found = {}
    for n, i in enumerate(starts):
        m = re.search(r"kernelILi(\d+)ELi(\d+)ELb(\d)ELi(\d+)ELb(\d)ELi(\d+)E", lines[i])
        key = tuple(int(x) for x in m.groups())           # BN, MT, INREG, NS, GATED, NW
        found[key] = lines[i:starts[n + 1] if n + 1 < len(starts) else len(lines)]
    return found


def hand_laid_loop(body):
    """Lines from the head of the loop that holds the assembly MFMAs to the last of them."""
    asm = [j for j, x in enumerate(body) if MFMA in x and "ASMSTART" in body[j - 1]]
    if not asm:
        return None
    head = max([j for j, x in enumerate(body) if "Loop Header" in x and j < asm[0]] or [asm[0]])
    return body[head:asm[-1] + 2]


def test_the_kernels_with_256_row_tiles_use_the_hand_laid_loop_and_the_others_do_not(gemm_kernels):
    assert len(gemm_kernels) >= 12
    for key, body in gemm_kernels.items():
        bn, mt, inreg, ns, gated, nw = key
        assert (hand_laid_loop(body) is not None) == (mt >= 256), key


def test_projection_loops_touch_no_operand_before_its_wait(gemm_kernels):
    checked = 0
    for key, body in gemm_kernels.items():
        loop = hand_laid_loop(body)
        if loop is None:
            continue
        bn, mt, inreg, ns, gated, nw = key
        c = Counter(x.split()[0] for x in instructions(loop))
        copies = {k: v for k, v in c.items() if k.startswith(("v_mov", "v_accvgpr", "scratch_", "v_swap", "v_readlane", "v_writelane"))}
        assert not copies, (key, copies)
        violations, n_reads = replay_lds_counter(loop)
        assert not violations, (key, violations[:5])
        # one stage: the wave's output tiles times two k halves of MFMAs, and every operand tile read exactly once per k half
        wmw = 4 if (nw == 8 and bn < mt) else 2
        na, nb = bn // (nw // wmw) // 16, mt // (16 * wmw)
        assert c[MFMA] == 2 * na * nb, (key, c[MFMA])
        assert n_reads == c["ds_read_b128"] == 2 * (na + nb), (key, n_reads)
        assert c["s_barrier"] == 1, key
        checked += 1
    assert checked >= 6


def test_the_replay_convicts_a_wait_that_is_one_short_and_a_copy_before_the_wait():
    """The checker itself: a stage's shape with a correct wait passes; the same with the wait one read short, or with
    a copy of an operand ahead of the wait, does not."""
    def loop(wait, extra=""):
        text = ["\t;;#ASMSTART", "\tds_read_b128 v[0:3], v40 offset:0", "\t;;#ASMEND",
                "\t;;#ASMSTART", "\tds_read_b128 v[4:7], v40 offset:2048", "\t;;#ASMEND",
                "\t;;#ASMSTART", "\tds_read_b128 v[8:11], v41 offset:0", "\t;;#ASMEND", extra,
                "\ts_waitcnt lgkmcnt(%d)" % wait,
                "\t;;#ASMSTART", "\tv_mfma_f32_16x16x32_bf16 v[20:23], v[0:3], v[4:7], v[20:23]", "\t;;#ASMEND",
                "\ts_waitcnt lgkmcnt(0)",
                "\t;;#ASMSTART", "\tv_mfma_f32_16x16x32_bf16 v[24:27], v[0:3], v[8:11], v[24:27]", "\t;;#ASMEND"]
        return [t for t in text if t]
    assert replay_lds_counter(loop(1))[0] == []
    assert replay_lds_counter(loop(2))[0] != []                         # v[4:7] may still be in flight
    assert replay_lds_counter(loop(1, "\tv_mov_b32_e32 v30, v9"))[0] != []   # a copy of an operand that has not arrived


def test_prefill_attention_loop_touches_no_operand_before_its_wait(tmp_path_factory):
    lines = compile_to_isa(tmp_path_factory.mktemp("isa_prefill"), "kernels_attn_prefill.hip")
    start = next(i for i, l in enumerate(lines) if re.match(r"^_ZN3dyn19attn_prefill_kernel\S*:", l))
    body = lines[start:]
    reads = [j for j, x in enumerate(body) if x.strip().startswith("ds_read") and "ASMSTART" in body[j - 1]]
    assert len(reads) == 4 * 4 + 8 * 4                                   # a tile: four K pages of four operands, eight V groups of four
    head = max(j for j, x in enumerate(body) if "Loop Header" in x and j < reads[0])
    last_mfma = max(j for j, x in enumerate(body) if MFMA in x)
    violations, n = replay_lds_counter(body[head:last_mfma + 1])
    assert n == 48 and not violations, violations[:5]
