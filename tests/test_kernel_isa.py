"""Static checks on the code hipcc generates for the persistent GEMM kernel (CPU only: cross-compilation).

The kernel names its accumulator registers itself (a[0:255], see csrc/gemm_common.h) instead of handing 64
values to the register allocator.  That is only sound if nothing else in the kernel touches an AGPR, if the
kernel really allocates all 256 of them, and if nothing is spilled to scratch memory; and the copy statements
rely on M0 being written and consumed inside one asm statement.  All of that is a property of the generated
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
        code = [l.split(";")[0].strip() for l in body[:body.index("s_endpgm") + 8].split("\n")]
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
