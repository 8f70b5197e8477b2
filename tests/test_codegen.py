"""Properties of the generated gfx950 code that the measured rates depend on.

The streaming hint of the copy kernels (cache-policy bits "sc0 sc1 nt") is worth
2-10 % of their rate and has been lost once to an optimiser merge of a hinted and
a plain access of the same address; nothing else would notice.  The test compiles the copy
kernels' own source to assembly text (no GPU needed) and checks the modifier on
every 16-byte access of the instantiations the library ships.
"""
import os
import re
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2501_06709_amd", "csrc")
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")


@pytest.fixture(scope="module")
def copy_asm(tmp_path_factory):
    out = tmp_path_factory.mktemp("asm") / "kvm_copy.s"
    cmd = [HIPCC, "--offload-arch=gfx950", "-O3", "-std=c++17", "-Xclang", "-target-feature", "-Xclang",
           "-packed-fp32-ops", "-I" + os.path.join(ROOT, "include"), "-I" + CSRC, "-x", "hip", "-S",
           "--cuda-device-only", os.path.join(CSRC, "kvm_copy.hip"), "-o", str(out)]
    subprocess.run(cmd, check=True, stdout=subprocess.DEVNULL, stderr=subprocess.DEVNULL)
    return out.read_text()


def body(asm, mangled_prefix):
    m = re.search(r"^(%s\w*):.*?s_endpgm" % re.escape(mangled_prefix), asm, re.S | re.M)
    assert m, "kernel %s not found" % mangled_prefix
    return m.group(0)


def wide_accesses(text):
    return [ln.strip() for ln in text.splitlines()
            if re.match(r"\s*global_(load|store)_dwordx4\b", ln)]


@pytest.mark.parametrize("prefix", [
    "_ZN3kvm11copy_kernelILi0ELb1EEE",      # fused migrate, hinted
    "_ZN3kvm11copy_kernelILi2ELb1EEE",      # unpack
    "_ZN3kvm11copy_kernelILi1ELb1EEE",      # pack, block-cut
    "_ZN3kvm12stage_kernelILb1ELb1ELb1EEE",  # pack, staging order, uniform block id
    "_ZN3kvm12stage_kernelILb1ELb1ELb0EEE",
    "_ZN3kvm12stage_kernelILb0ELb1ELb1EEE",
])
def test_shipped_copy_kernels_carry_the_streaming_hint(copy_asm, prefix):
    acc = wide_accesses(body(copy_asm, prefix))
    assert len(acc) >= 2
    assert all(a.endswith(" sc0 sc1 nt") for a in acc), [a for a in acc if not a.endswith(" sc0 sc1 nt")]


def test_plain_instantiation_has_no_hint(copy_asm):
    acc = wide_accesses(body(copy_asm, "_ZN3kvm11copy_kernelILi0ELb0EEE"))
    assert acc and not any(a.endswith(" nt") for a in acc)


def test_no_scratch_in_copy_kernels(copy_asm):
    sizes = re.findall(r"\.private_segment_fixed_size:\s*(\d+)", copy_asm)
    assert sizes and all(int(s) == 0 for s in sizes)
