"""Register budget of the kernels the headline workload runs (host-side check, no GPU).

The attention main kernel, the samplers and the distillation row kernel are tuned to fit the 256
vector registers a wave gets at one 512-thread work-group per compute unit.  A spill in them costs more than its
instructions: a scratch reload is a vector memory operation and waits for every store issued
before it.  hipcc reports registers and scratch per kernel (-Rpass-analysis=kernel-resource-usage);
this test compiles the sources for the device only and reads that report.
"""
import os
import re
import shutil
import subprocess
from concurrent.futures import ThreadPoolExecutor

import pytest

from paper_2510_26475_amd import build

# (source, mangled-name fragment, what it is)
NO_SCRATCH = [
    ("respec_attention.hip", "attn_bf16_kernelILi128ELi1EtLi1E", "attention, D=128, one column tile"),
    ("respec_attention.hip", "attn_bf16_kernelILi128ELi2EtLi1E", "attention, D=128, two column tiles (B=256, k=3 at the 7B shape)"),
    ("respec_attention.hip", "attn_bf16_kernelILi128ELi2EtLi2E", "attention, D=128, two consumers per range"),
    ("respec_attention.hip", "attn_bf16_kernelILi128ELi2EtLi4E", "attention, D=128, four consumers per range"),
    ("respec_attention.hip", "attn_bf16_kernelILi128ELi1EtLi4E", "attention, D=128, four consumers, narrow block"),
    ("respec_sampler.hip", "rejection_sample_kernelILb1ELb1ELb1ELb0E", "chain sampler, bf16, one work-group per sequence"),
    ("respec_sampler.hip", "rejection_sample_kernelILb1ELb1ELb1ELb1E", "chain sampler, bf16, sequences shared by several work-groups"),
    ("respec_tree_sampler.hip", "tree_rejection_sample_kernelILb1ELb1ELb1E", "tree sampler, bf16, temperature 1"),
    ("respec_kd.hip", "kd_stream_kernelILb1E", "distillation rows, bf16"),
]


def _report(source):
    cmd = [build.HIPCC] + [f for f in build.FLAGS if f not in ("-shared", "-fPIC")] + [
        "-c", os.path.join(build.CSRC, source), "-o", os.devnull, "--offload-device-only",
        "-Rpass-analysis=kernel-resource-usage"]
    res = subprocess.run(cmd, capture_output=True, text=True)
    assert res.returncode == 0, res.stderr[-2000:]
    kernels, name = {}, None
    for line in res.stderr.splitlines():
        m = re.search(r"Function Name: (\S+)", line)
        if m:
            name = m.group(1)
            kernels[name] = {}
            continue
        m = re.search(r"remark:\s+(VGPRs|ScratchSize \[bytes/lane\]): (\d+)", line)
        if m and name:
            kernels[name][m.group(1)] = int(m.group(2))
    return kernels


@pytest.fixture(scope="module")
def reports():
    if not (os.path.exists(build.HIPCC) or shutil.which(build.HIPCC)):
        pytest.skip("no hipcc")
    sources = sorted({s for s, _, _ in NO_SCRATCH})
    with ThreadPoolExecutor(len(sources)) as pool:
        return dict(zip(sources, pool.map(_report, sources)))


@pytest.mark.parametrize("source,fragment,what", NO_SCRATCH, ids=[w for _, _, w in NO_SCRATCH])
def test_headline_kernels_keep_their_state_in_registers(reports, source, fragment, what):
    hits = {k: v for k, v in reports[source].items() if fragment in k}
    assert len(hits) == 1, f"{what}: expected one kernel matching {fragment}, found {sorted(hits)}"
    (name, usage), = hits.items()
    assert usage.get("VGPRs", 0) <= 256, (name, usage)
    assert usage.get("ScratchSize [bytes/lane]", -1) == 0, f"{what} spills: {usage}"
