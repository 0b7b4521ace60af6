"""The build refuses register spills in the streaming decode kernels (host logic of paper_2410_21271_amd/build.py:
the compiler's resource remarks are parsed per kernel)."""
import importlib.util
import os

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _build_module():
    spec = importlib.util.spec_from_file_location("eora_build", os.path.join(ROOT, "paper_2410_21271_amd", "build.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    return mod


REMARKS = """\
a.hip:10:1: remark: Function Name: _ZN4eora15resident_kernelILi1ELi5ELi5ELi8EEEvNS_10StreamArgsE [-Rpass-analysis=kernel-resource-usage]
a.hip:10:1: remark:     VGPRs: 128 [-Rpass-analysis=kernel-resource-usage]
a.hip:10:1: remark:     ScratchSize [bytes/lane]: %d [-Rpass-analysis=kernel-resource-usage]
a.hip:90:1: remark: Function Name: _ZN4eora12other_kernelEv [-Rpass-analysis=kernel-resource-usage]
a.hip:90:1: remark:     ScratchSize [bytes/lane]: %d [-Rpass-analysis=kernel-resource-usage]
"""


def test_spill_in_a_streaming_kernel_fails_the_build():
    b = _build_module()
    b._check_resources("stream.hip", REMARKS % (0, 0))
    b._check_resources("stream.hip", REMARKS % (0, 64))          # another kernel of the file may use scratch
    with pytest.raises(RuntimeError) as e:
        b._check_resources("stream.hip", REMARKS % (36, 0))
    assert "resident_kernel" in str(e.value) and "36 bytes" in str(e.value)


def test_every_source_is_listed_once():
    b = _build_module()
    on_disk = sorted(f for f in os.listdir(b.CSRC) if f.endswith((".hip", ".cpp")))
    assert sorted(b.SOURCES) == on_disk
    assert set(b.NO_SPILL) <= set(b.SOURCES)
