"""Checks on the generated gfx950 code of the kernels that fill LDS from inline assembly (no GPU needed: hipcc
cross-compiles).  The buffer resource of such a load has to sit in scalar registers and the hot loops must not touch
scratch memory; a source change that looks harmless can lose either (a descriptor chosen by a run-time index ends up in
vector registers and in scratch), and nothing at run time reports it."""
import os
import re
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2108_01624_amd", "csrc")


def _hipcc():
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", shutil.which("hipcc")):
        if cand and os.path.exists(cand):
            return cand
    return None


def _isa(src, tmp_path):
    hipcc = _hipcc()
    if hipcc is None:
        pytest.skip("hipcc not found")
    from paper_2108_01624_amd.build import HIPCC_FLAGS

    out = tmp_path / (src + ".s")
    flags = [f for f in HIPCC_FLAGS if f != "-fPIC"]
    r = subprocess.run([hipcc] + flags + ["--cuda-device-only", "-S", os.path.join(CSRC, src), "-o", str(out)],
                       capture_output=True, text=True)
    assert r.returncode == 0, r.stderr[-2000:]
    return out.read_text()


def _kernels(text):
    """name -> (body, metadata block) for every kernel of the translation unit."""
    out = {}
    for m in re.finditer(r"\.amdhsa_kernel (\S+)(.*?)\.end_amdhsa_kernel", text, re.S):
        name, meta = m.group(1), m.group(2)
        start = text.find("\n" + name + ":")
        end = text.find("s_endpgm", start)
        out[name] = (text[start:end], meta)
    return out


@pytest.mark.parametrize("src,hot", [("dp_gram.hip", ("gram_dma_kernel", "gram_units_kernel", "gram_small_dma_kernel")),
                                     ("dp_wgemm.hip", ("wgemm_dma16_kernel",))])
def test_lds_filling_kernels_keep_descriptors_scalar_and_use_no_scratch(src, hot, tmp_path):
    kernels = _kernels(_isa(src, tmp_path))
    seen = 0
    for name, (body, meta) in kernels.items():
        if not any(h in name for h in hot):
            continue
        seen += 1
        scratch = int(re.search(r"\.amdhsa_private_segment_fixed_size (\d+)", meta).group(1))
        assert scratch == 0, f"{name} uses {scratch} bytes of scratch per lane"
        assert "scratch_" not in body, f"{name} has scratch instructions"
        loads = re.findall(r"buffer_load_dwordx4 (\S+), (\S+), (\S+) offen(?: nt)? lds", body)
        assert loads, f"{name}: no LDS-filling loads found"
        for vaddr, rsrc, soff in loads:
            assert vaddr.startswith("v") and rsrc.startswith("s[") and soff.startswith("s"), (name, vaddr, rsrc, soff)
        assert "v_pk_mul_f32" not in body and "v_pk_fma_f32" not in body and "v_pk_add_f32" not in body, name
    assert seen >= len(hot) and all(any(h in name for name in kernels) for h in hot)
