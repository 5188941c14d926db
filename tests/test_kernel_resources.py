"""What the compiler reported for the kernels of the library as built (paper_2510_26692_amd/libkda.resources.json,
written by every build): the kernels of the bench workloads must not touch scratch memory.  In the one-kernel
prefill a scratch access waits behind the write-through slot stores in the same queue (a chunk took 22 instead of
14 microseconds with a handful of spilled registers), and an array indexed by the wave number, which the compiler
places in scratch, cost the 2^20-token workload 5 % before it was noticed."""
import json
import os

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
REPORT = os.path.join(ROOT, "paper_2510_26692_amd", "libkda.resources.json")


@pytest.fixture(scope="module")
def resources():
    if not os.path.exists(REPORT):
        pytest.skip("no resource report: build the library first (python -m paper_2510_26692_amd.build)")
    with open(REPORT) as f:
        return json.load(f)


def _kernels(resources, *fragments):
    return {k: v for k, v in resources.items() if all(f in k for f in fragments)}


def test_report_covers_the_kernels_of_the_hot_path(resources):
    assert len(_kernels(resources, "kda_prefill_kernel")) == 10          # raw x bf16-out x gate, scalar x bf16-out
    assert _kernels(resources, "kda_step_kernel") and _kernels(resources, "kda_fused_fill_kernel")


def test_prefill_kernels_use_no_scratch_outside_the_gated_variants(resources):
    # template arguments <kRaw, kScalar, kOutBf16, kGate>
    every = _kernels(resources, "kda_prefill_kernel")
    for name, r in every.items():
        gate = name.endswith("Lb1EEEvNS0_9FusedArgsE")
        assert r["VGPRs"] <= 256 and r["Occupancy [waves/SIMD]"] >= 2, (name, r)
        if not gate:
            assert r["ScratchSize [bytes/lane]"] == 0 and r["VGPRs Spill"] == 0, (name, r)
        else:
            # (the gated variants keep a few dwords outside the scan loop)
            assert r["VGPRs Spill"] <= 16, (name, r)


def test_decode_kernels_use_no_scratch(resources):
    for name, r in _kernels(resources, "kda_step_kernel").items():
        assert r["ScratchSize [bytes/lane]"] == 0 and r["VGPRs Spill"] == 0, (name, r)
