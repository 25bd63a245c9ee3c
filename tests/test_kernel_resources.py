"""What the compiler made of the merge kernels, checked where it once went wrong unnoticed: no kernel may need
scratch memory (a merge kernel that does takes about 18 us longer to launch), the merge kernels must fit four
workgroups of 256 threads per compute unit (at most 128 vector registers), and column_merge, which is a function
of its own, must reach its LDS columns with ds_ instructions and the table with global_ ones (left to itself the
compiler uses flat instructions for pointer arguments of an out-of-line function: 64-byte pieces then took 96
instead of 56 us).  One device-only compilation of csrc/bpe_encode.hip to assembly; no GPU."""
import os
import re
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2603_02597_amd", "csrc")


@pytest.fixture(scope="module")
def compiled(tmp_path_factory):
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    if not os.path.exists(hipcc):
        pytest.skip("no hipcc")
    from paper_2603_02597_amd.build import FLAGS
    out = str(tmp_path_factory.mktemp("isa") / "bpe_encode.s")
    flags = [f for f in FLAGS if f not in ("-shared", "-fPIC")]
    r = subprocess.run([hipcc, *flags, "-I", os.path.join(ROOT, "include"), "-I", CSRC, "-S", "--cuda-device-only",
                        "-Rpass-analysis=kernel-resource-usage", os.path.join(CSRC, "bpe_encode.hip"), "-o", out],
                       capture_output=True, text=True, timeout=900)
    assert r.returncode == 0, r.stderr[-3000:]
    return open(out).read(), r.stderr


def _usage(remarks):
    """{kernel: {"VGPRs": n, "ScratchSize": n, ...}} from the resource-usage remarks."""
    usage, name = {}, None
    for line in remarks.splitlines():
        m = re.search(r"Function Name: (\S+)", line)
        if m:
            name = m.group(1)
            usage[name] = {}
            continue
        m = re.search(r"remark:\s+([A-Za-z ]+?)(?: \[[^\]]*\])?: (\d+)", line)
        if m and name:
            usage[name][m.group(1).strip()] = int(m.group(2))
    return usage


def test_no_kernel_needs_scratch_memory_and_merge_kernels_fit_four_workgroups(compiled):
    _, remarks = compiled
    assert "loop not unrolled" not in remarks, "an unrolled loop over a register array was left as a loop"
    usage = _usage(remarks)
    merge = [k for k in usage if re.search(r"merge_\w*kernel|encode_kernel", k) and "merge_wide" not in k]
    assert len(merge) >= 8, sorted(usage)
    for k, u in usage.items():
        assert u.get("ScratchSize", 0) == 0, (k, u)
        assert u.get("VGPRs Spill", 0) == 0, (k, u)
    for k in merge:
        assert usage[k]["VGPRs"] + usage[k].get("AGPRs", 0) <= 128, (k, usage[k])


def test_column_merge_names_its_address_spaces(compiled):
    asm, _ = compiled
    m = re.search(r"^(_ZN3bpe12column_mergeILi64E\w*):.*?^\.Lfunc_end\d+:", asm, re.S | re.M)
    if not m:     # inlined everywhere: then the kernels' own address spaces apply
        assert "column_merge" not in asm
        return
    body = m.group(0)
    count = lambda pat: len(re.findall(r"^\s+" + pat, body, re.M))
    assert count(r"ds_read_b128") >= 16 and count(r"ds_write_b32") >= 32      # the columns
    assert count(r"global_load_dwordx2") >= 4                                  # the slots of two pairs
    assert count(r"flat_load_dwordx4") <= 3 and count(r"flat_store") == 0      # (the parameter block itself is read flat)
    assert count(r"scratch_") == 0
