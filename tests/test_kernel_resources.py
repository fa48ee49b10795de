"""Build-time check of the compiled kernels (no GPU): the production instances of the attention kernel must not
use scratch memory. A staging lambda that stops being inlined keeps its register arrays in scratch without any
spill being reported, and the kernel then runs at half its speed; the compiler's resource remarks show it."""
import os
import re
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")


@pytest.mark.skipif(not os.path.exists(HIPCC), reason="hipcc not found")
def test_attention_kernels_use_no_scratch(tmp_path):
    from paper_2605_00342_amd import build as b
    src = os.path.join(b.CSRC, "layer_kernels.hip")
    cmd = [HIPCC, *b.FLAGS, "-Rpass-analysis=kernel-resource-usage", "-c", src, "-o", str(tmp_path / "lk.o")]
    out = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, check=True).stdout
    name, seen = None, {}
    for line in out.splitlines():
        m = re.search(r"Function Name: (\S+)", line)
        if m:
            name = m.group(1)
        m = re.search(r"ScratchSize \[bytes/lane\]: (\d+)", line)
        if m and name:
            seen[name] = int(m.group(1))
    attn = {k: v for k, v in seen.items() if "attn_partial_mfma_kernel" in k}
    assert len(attn) == 8, sorted(attn)  # head dimension 64 / 128 x 4 / 8 wavefronts x contiguous / paged
    assert all(v == 0 for v in attn.values()), attn
    router = {k: v for k, v in seen.items() if "router_logits_kernel" in k and "4BF16" in k}
    assert router and all(v <= 128 for v in router.values()), router
