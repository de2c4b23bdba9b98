"""The benchmark's issue model counts vector-ALU instructions per wavefront by class (bench.KERNEL_MIX).
This test recounts them from a fresh compiler listing of the kernels (no GPU needed), so that the
table cannot drift away from the code it describes."""
import collections
import os
import re
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)


@pytest.fixture(scope="module")
def listing(tmp_path_factory):
    from paper_2509_07003_amd import build
    out = str(tmp_path_factory.mktemp("listing") / "kernels.s")
    flags = [f for f in build.FLAGS if f not in ("-shared", "-fPIC")]
    cmd = [build.HIPCC] + flags + ["-S", "--cuda-device-only", "-x", "hip", os.path.join(build.CSRC, "kernels.hip"), "-o", out]
    subprocess.run(cmd, check=True, stdout=subprocess.PIPE, stderr=subprocess.STDOUT)
    return open(out).read().split("\n")


def histogram(listing, mangled_fragment):
    """Mnemonic -> count over the body of the kernel whose mangled name contains the fragment."""
    start = next(i for i, l in enumerate(listing) if l.startswith("_ZN") and mangled_fragment in l and ": " in l + " ")
    counts = collections.Counter()
    for l in listing[start + 1:]:
        if l.startswith(".Lfunc_end"):
            break
        t = l.split(";")[0].strip()
        if not t or t.startswith(".") or t.endswith(":"):
            continue
        counts[t.split()[0]] += 1
    return counts


def mangled(kernel):
    """'aligned_kernel<2, 1, unsigned int, 1, true>' -> the Itanium fragment 'aligned_kernelILi2ELi1EjLi1ELb1EE'."""
    name, args = re.match(r"(\w+)<(.*)>", kernel).groups()
    code = {"unsigned int": "j", "unsigned long": "m", "true": "Lb1E", "false": "Lb0E"}
    enc = "".join(code.get(a.strip(), "Li%sE" % a.strip()) for a in args.split(","))
    return "%sI%sE" % (name, enc)


def test_instruction_mix_table_matches_the_compiler_listing(listing):
    import bench
    straight_line = {"aligned normal bf16", "aligned normal f32", "aligned dropout bf16"}
    for tag, mix in bench.KERNEL_MIX.items():
        h = histogram(listing, mangled(mix["kernel"]))
        valu = sum(c for m, c in h.items() if m.startswith("v_"))
        trans = sum(c for m, c in h.items() if re.match(r"v_(log|sqrt|sin|cos|exp|rcp|rsq)_f32", m))
        passes = mix.get("loop_iterations", 1)   # the staging kernel's generator loop runs this often per wave
        assert h["v_mad_u64_u32"] * passes == mix["mad_u64_u32"], tag
        assert h["v_bitop3_b32"] * passes == mix["bitop3_b32"], tag
        assert trans * passes == mix["trans"], tag
        total = mix["mad_u64_u32"] + mix["bitop3_b32"] + mix["trans"] + mix["other"]
        if passes > 1:
            # A loop: the per-wave total is the hardware counter's (checked against the committed profile below);
            # it must at least cover the generator classes and stay under `passes` times the whole listing.
            assert mix["other"] > 0 and total < passes * valu, (tag, valu, total)
        elif tag in straight_line:
            assert valu == total, (tag, valu, total)          # no branches: the listing is what a wave executes
        else:
            # Branchy kernels (a wave-uniform choice between two conversions; edge paths): a wave executes
            # one side, so the table (the hardware counter's per-wave count) lies below the listing's total.
            assert 0.7 * valu <= total <= valu, (tag, valu, total)
    # The generator is 19 or more products (the first round's second product is by a zero counter word)
    # and 20 three-way XORs per block; nothing else in it is a vector instruction.
    h = histogram(listing, mangled("aligned_kernel<0, 0, unsigned int, 0, false>"))
    assert h["v_mad_u64_u32"] >= 19 and h["v_bitop3_b32"] == 20 and h["v_xor_b32_e32"] == 0


def test_instruction_mix_table_matches_the_committed_counter_profile():
    """The per-wave totals of bench.KERNEL_MIX are what the hardware counters read (SQ_INSTS_VALU / SQ_WAVES in
    profiles/counters_bench_kernels.txt, written from a rocprofv3 --pmc run of bench.py --counters-pass)."""
    import bench
    text = open(os.path.join(ROOT, "profiles", "counters_bench_kernels.txt")).read()
    line = next(l for l in text.splitlines() if l.startswith("valu_per_wave:"))
    measured = {}
    for item in line.split(":", 1)[1].split(";"):
        name, value = item.rsplit("=", 1)
        measured.setdefault(name.split("@")[0].strip(), []).append(float(value))
    seen = 0
    for tag, mix in bench.KERNEL_MIX.items():
        total = mix["mad_u64_u32"] + mix["bitop3_b32"] + mix["trans"] + mix["other"]
        for value in measured.get(mix["kernel"], []):
            assert abs(value - total) <= 1.0, (tag, value, total)
            seen += 1
    assert seen >= 5
