"""Static checks on the code hipcc generates for the persistent GEMM kernel (CPU only: cross-compilation).

The kernel names its accumulator registers itself (a[0:255], see csrc/gemm_common.h) instead of handing 64
values to the register allocator.  That is only sound if nothing else in the kernel touches an AGPR, if the
kernel really allocates all 256 of them, and if nothing is spilled to scratch memory; the copy statements
rely on M0 being written and consumed inside one asm statement; and the MFMA statements get no hazard
handling from the compiler.  All of that is a property of the generated
code, so it is checked on the generated code.
"""
import os
import re
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2509_01193_amd", "csrc")
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")


@pytest.fixture(scope="module")
def kernels(tmp_path_factory):
    out = str(tmp_path_factory.mktemp("isa") / "gemm_persistent.s")
    cmd = [HIPCC, "--offload-arch=gfx950", "-O3", "-std=c++17", "-Xclang", "-target-feature", "-Xclang",
           "-packed-fp32-ops", "-I", os.path.join(ROOT, "include"), "-I", CSRC, "-x", "hip", "--cuda-device-only",
           "-S", os.path.join(CSRC, "gemm_persistent.hip"), "-o", out]
    r = subprocess.run(cmd, capture_output=True, text=True, timeout=600)
    assert r.returncode == 0, r.stderr[-3000:]
    text = open(out).read()
    # one entry per kernel: (name, instruction lines, trailer with the resource summary)
    parts = re.split(r"^(_ZN5lobra22gemm_persistent_kernel\w+):", text, flags=re.M)
    ks = []
    for i in range(1, len(parts), 2):
        body = parts[i + 1]
        end = body.index(".end_amdhsa_kernel")
        code = [l.split(";")[0].strip() for l in body[:body.rindex("s_endpgm", 0, end) + 8].split("\n")]
        code = [l for l in code if l and not l.startswith(".")]
        tail = body[end:end + 3000]
        ks.append((parts[i], code, tail))
    assert len(ks) == 2, [k[0] for k in ks]      # forward and backward instantiation
    return ks


def test_only_the_named_statements_touch_agprs(kernels):
    mfma = re.compile(r"v_mfma_f32_16x16x32_bf16 a\[\w+:\w+\], v\[\d+:\d+\], v\[\d+:\d+\], (a\[\w+:\w+\]|0)$")
    rd = re.compile(r"v_accvgpr_read_b32 v\d+, a\[\w+\]$")
    for name, code, _ in kernels:
        users = [l for l in code if re.search(r"\ba(\[|\d)", l)]
        assert len(users) > 300, name
        bad = [l for l in users if not (mfma.match(l) or rd.match(l))]
        assert not bad, (name, bad[:5])
        # an MFMA updates its accumulator in place (or starts it from zero)
        for l in users:
            m = re.match(r"v_mfma_f32_16x16x32_bf16 (a\[\w+:\w+\]), .*, (a\[\w+:\w+\]|0)$", l)
            if m:
                assert m.group(2) in ("0", m.group(1)), l


def test_all_agprs_allocated_and_nothing_spilled(kernels):
    for name, code, tail in kernels:
        assert re.search(r"; NumAgprs: 256\b", tail), (name, tail[:800])
        assert re.search(r"; ScratchSize: 0\b", tail), (name, tail[:800])
        assert not [l for l in code if l.startswith("scratch_")], name
        assert re.search(r"; Occupancy: 1\b", tail), name


def test_m0_is_written_and_consumed_inside_one_statement(kernels):
    for name, code, _ in kernels:
        writes = [i for i, l in enumerate(code) if re.match(r"s_mov_b32 m0,", l)]
        copies = [i for i, l in enumerate(code) if l.startswith("global_load_lds_dwordx4")]
        assert len(copies) >= 48 and len(writes) == len(copies), (name, len(writes), len(copies))
        for w, c in zip(writes, copies):
            assert 0 < c - w <= 2, (name, code[w:c + 1])         # at most the MFMA / s_nop of the statement between
        # nothing else writes M0
        assert not [l for l in code if re.search(r"\bm0\b", l) and not l.startswith(("s_mov_b32 m0,", "global_load_lds"))], name


def _vregs(tok):
    m = re.match(r"v\[(\d+):(\d+)\]$", tok)
    if m:
        return set(range(int(m.group(1)), int(m.group(2)) + 1))
    m = re.match(r"v(\d+)$", tok)
    return {int(m.group(1))} if m else set()


def test_no_mfma_reads_a_register_a_vector_alu_instruction_has_just_written(kernels):
    """The MFMAs are asm statements and the compiler's hazard pass does not look into those: an MFMA needs two
    wait states between a vector ALU write of one of its operand registers and its own read of it (operands that
    come from LDS or memory are covered by the waitcnt the compiler does insert)."""
    for name, code, _ in kernels:
        for i, l in enumerate(code):
            if not l.startswith("v_mfma"):
                continue
            ops = [t.strip() for t in l.split(None, 1)[1].split(",")]
            src = _vregs(ops[1]) | _vregs(ops[2])
            states, k = 0, i - 1
            while states < 2 and k >= 0:
                pl = code[k]
                if pl.startswith("v_") and not pl.startswith(("v_mfma", "v_accvgpr")):
                    dst = pl.split(None, 1)[1].split(",")[0].strip()
                    assert not (_vregs(dst) & src), (name, code[k:i + 1])
                m = re.match(r"s_nop (\d+)$", pl)
                states += int(m.group(1)) + 1 if m else 1
                k -= 1


def test_main_loop_has_no_instruction_clumps(kernels):
    """A wave issues one instruction per four cycles and an MFMA holds its pipe for 16: more than a dozen other
    instructions between two MFMAs of the main loop drain the matrix pipe."""
    for name, code, _ in kernels:
        idx = [i for i, l in enumerate(code) if l.startswith("v_mfma")]
        # the longest run of MFMAs at most 13 instructions apart must cover a whole K tile (128 MFMAs) and more
        best = run = 1
        for a, b in zip(idx, idx[1:]):
            run = run + 1 if b - a <= 13 else 1
            best = max(best, run)
        assert best >= 128, (name, best)


# ---------------------------------------------------------------------------------------------------------
# The K-sliced rank-r kernel keeps several items' copies in flight and waits for them by count.  That only
# works if the compiler adds no wait of its own that drains them: its tables must be read with scalar loads
# (which the vector-memory counter does not see), the item barrier must come without a fence, and the copies
# must be the direct-to-LDS kind with M0 written right in front of each.
# ---------------------------------------------------------------------------------------------------------
@pytest.fixture(scope="module")
def sliced_kernels(tmp_path_factory):
    out = str(tmp_path_factory.mktemp("isa") / "skinny_mfma.s")
    cmd = [HIPCC, "--offload-arch=gfx950", "-O3", "-std=c++17", "-Xclang", "-target-feature", "-Xclang",
           "-packed-fp32-ops", "-I", os.path.join(ROOT, "include"), "-I", CSRC, "-x", "hip", "--cuda-device-only",
           "-S", os.path.join(CSRC, "skinny_mfma.hip"), "-o", out]
    r = subprocess.run(cmd, capture_output=True, text=True, timeout=600)
    assert r.returncode == 0, r.stderr[-3000:]
    text = open(out).read()
    parts = re.split(r"^(_ZN5lobra20shrink_sliced_kernel\w+):", text, flags=re.M)
    ks = []
    for i in range(1, len(parts), 2):
        body = parts[i + 1]
        end = body.index(".end_amdhsa_kernel")
        code = [l.split(";")[0].strip() for l in body[:end].split("\n")]
        code = [l for l in code if l and not l.startswith(".")]
        ks.append((parts[i], code, body[end:end + 3000]))
    assert len(ks) == 2, [k[0] for k in ks]      # projection alone, projection with dB
    return ks


def test_sliced_kernel_waits_for_its_copies_by_count(sliced_kernels):
    for name, code, tail in sliced_kernels:
        fused = "ILb1E" in name
        assert re.search(r"; ScratchSize: 0\b", tail), name
        copies = [i for i, l in enumerate(code) if l.startswith("global_load_lds_dwordx4")]
        assert len(copies) >= 16, (name, len(copies))
        for c in copies:            # M0 is written inside the copy's own asm statement
            assert any(re.match(r"s_mov_b32 m0,", code[k]) for k in range(max(0, c - 2), c)), (name, code[c - 3:c + 1])
        # the steady-state wait leaves the copies of three younger items in flight (wave 0 of the fused form
        # has a fifth copy per item), the drain at the end counts down
        waits = {int(m.group(1)) for l in code for m in [re.match(r"s_waitcnt vmcnt\((\d+)\)$", l)] if m}
        assert {12, 8, 4} <= waits, (name, sorted(waits))
        if fused:
            assert {15, 10, 5} <= waits, (name, sorted(waits))
        # ordinary vector loads: only the adapter rows (16 bytes per lane), never the tables
        plain = [l for l in code if re.match(r"global_load_(dword|dwordx2|dwordx3|ubyte|ushort|sbyte|sshort)\b", l)]
        assert not plain, (name, plain[:4])
        assert [l for l in code if l.startswith("s_load_dwordx4") or l.startswith("s_load_dwordx2")], name
        # no barrier drags a full vector-memory wait along (what a fenced barrier would do)
        for i, l in enumerate(code):
            if l == "s_barrier":
                assert not any(re.match(r"s_waitcnt.*vmcnt\(0\)", code[k]) for k in range(max(0, i - 3), i)), (name, code[i - 4:i + 1])
