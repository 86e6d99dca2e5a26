"""Properties of the generated gfx950 code that the attention kernel's hand-written LDS
transfers rely on (CPU only: hipcc cross-compiles the device code to assembly).

The transfer statement writes M0 itself and the kernel assumes that nothing else does:
no register-indirect indexing (v_movrel / s_movrel set M0), no other M0 user in between.
"""
import os
import re
import subprocess

import pytest

from paper_2503_16257_amd import build as B

SRC = os.path.join(B.CSRC, "decode_attn_mfma.hip")


@pytest.fixture(scope="module")
def attention_isa(tmp_path_factory):
    out = tmp_path_factory.mktemp("isa") / "decode_attn_mfma.s"
    flags = [f for f in B.FLAGS if f not in ("-fPIC", "-Wall", "-Wno-unused-function")]
    cmd = [B._hipcc(), *flags, "-w", "-S", "--cuda-device-only", SRC, "-o", str(out)]
    r = subprocess.run(cmd, capture_output=True, text=True)
    assert r.returncode == 0, r.stderr[-2000:]
    return out.read_text()


def test_m0_is_written_only_by_the_transfer_statements(attention_isa):
    transfers = len(re.findall(r"^\s*global_load_lds_dwordx4\b", attention_isa, re.M))
    m0_lines = [l for l in attention_isa.splitlines() if re.search(r"\bm0\b", l) and not l.lstrip().startswith(";")]
    assert transfers > 0
    # every mention of M0 is the s_mov of one transfer statement
    assert all(re.match(r"\s*s_mov_b32 m0, s\d+", l) for l in m0_lines), \
        [l for l in m0_lines if not re.match(r"\s*s_mov_b32 m0, s\d+", l)][:5]
    assert len(m0_lines) == transfers
    assert "movrel" not in attention_isa


def test_no_register_spills_in_the_headline_variants(attention_isa):
    """n_a = 16 (the long-video and serving shapes), all three protected-row modes."""
    found = 0
    for m in re.finditer(r"\.name:\s+(\S+).*?\.vgpr_spill_count:\s+(\d+)", attention_isa, re.S):
        name, spills = m.group(1), int(m.group(2))
        if re.search(r"attn_mfma_kernelILi2ELi[012]ELb1E", name):
            found += 1
            assert spills == 0, (name, spills)
    assert found == 3
