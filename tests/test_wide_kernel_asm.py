"""The steady-state loop of prefill_kernel_wide issues its MFMAs as assembly, which the compiler cannot see into: it
adds no wait states for instructions of its own that would read such an MFMA's result.  The kernel is written so that
the compiler has no reason to place any there (no spill, no copy between the register files, no move); this test
compiles the kernel and checks that it did not."""
import collections
import os
import re
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2502_12574_amd", "csrc")


def steady_state_loop(asm, mangled):
    st = asm.index(mangled + ":")
    body = asm[st:asm.index(".Lfunc_end", st)].split("\n")
    labels = {}
    for i, line in enumerate(body):
        m = re.match(r"(\.LBB\d+_\d+):", line)
        if m:
            labels[m.group(1)] = i
    best = None
    for i, line in enumerate(body):
        m = re.match(r"\s*s_c?branch\S*\s+(\.LBB\d+_\d+)", line)
        if m and m.group(1) in labels and labels[m.group(1)] < i:
            seg = body[labels[m.group(1)]:i]
            if sum("v_mfma" in x for x in seg) == 512 and (best is None or len(seg) < len(best)):
                best = seg
    return best


@pytest.fixture(scope="module")
def asm(tmp_path_factory):
    hipcc = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    if not os.path.exists(hipcc):
        pytest.skip("no hipcc")
    from paper_2502_12574_amd.build import HIPCC_FLAGS
    out = str(tmp_path_factory.mktemp("asm") / "hi_prefill.s")
    flags = [f for f in HIPCC_FLAGS if f != "-fPIC"]
    r = subprocess.run([hipcc, *flags, "-x", "hip", "-I", os.path.join(ROOT, "include"), "-I", CSRC, "-S",
                        "--cuda-device-only", os.path.join(CSRC, "hi_prefill.hip"), "-o", out],
                       stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    assert r.returncode == 0, r.stdout[-2000:]
    return open(out).read()


@pytest.mark.parametrize("prescaled", [1, 0])
def test_nothing_of_the_compilers_reads_an_mfma_result_inside_the_loop(asm, prescaled):
    loop = steady_state_loop(asm, f"_ZN2hi19prefill_kernel_wideILb{prescaled}EEEvNS_11PrefillArgsE")
    assert loop is not None, "no loop of four tiles (512 MFMAs) found"
    ops = collections.Counter(x.split()[0] for x in (l.strip() for l in loop) if x and not x.startswith((".", ";")))
    assert not [o for o in ops if o.startswith("scratch_")], ops           # no spill, no reload
    assert not [o for o in ops if o.startswith("v_accvgpr")], ops         # no copy between the register files
    assert ops["v_mov_b32_e32"] + ops["v_mov_b64_e32"] <= 6, ops          # (the loop's own flag and counter)
    # the instructions the loop is made of: four tiles of 128 MFMAs, 64 exponentials, 32 conversions, 48 LDS reads
    assert ops["v_mfma_f32_16x16x32_bf16"] == 512 and ops["v_exp_f32_e32"] == 256
    assert ops["v_cvt_pk_bf16_f32"] == 128 and ops["ds_read_b64_tr_b16"] == 128 and ops["ds_read_b128"] == 64
    assert ops["global_load_lds_dwordx4"] == 32 and ops["s_barrier"] == 4
    # the vector ALU instructions that touch score registers are the exponentials (and, for plain queries, the
    # multiplications in front of them); everything else works on their results
    allowed = {"v_mfma_f32_16x16x32_bf16", "v_exp_f32_e32", "v_add_f32_e32", "v_cvt_pk_bf16_f32", "v_mul_f32_e32",
               "v_cmp_nge_f32_e32", "v_cmp_nge_f32_e64", "v_cndmask_b32_e64", "v_cmp_ne_u32_e64", "v_mov_b32_e32",
               "v_mov_b64_e32", "v_readfirstlane_b32"}
    assert not [o for o in ops if o.startswith("v_") and o not in allowed], ops
