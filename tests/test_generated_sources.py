"""The generated assembly that the kernels include (csrc/*.inc, committed) is what the committed generators write."""
import os
import subprocess
import sys

import pytest

CSRC = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "paper_2508_06447_amd", "csrc")


@pytest.mark.parametrize("generator,outputs", [
    ("gen_attn_asm.py", ("attn_bf16_body.inc", "attn_bf16_clobbers.inc")),
    ("gen_gemm_asm.py", ("gemm_bf16_mainloops.inc",)),
])
def test_generated_files_are_current(tmp_path, generator, outputs):
    subprocess.run([sys.executable, os.path.join(CSRC, generator), str(tmp_path)], check=True, stdout=subprocess.DEVNULL,
                   stderr=subprocess.DEVNULL)
    for name in outputs:
        fresh, kept = open(tmp_path / name).read(), open(os.path.join(CSRC, name)).read()
        assert fresh == kept, f"{name} is stale: run `python {generator}` in csrc/ and rebuild"
