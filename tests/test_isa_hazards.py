"""The backward kernels issue their score MFMAs from assembly statements, for which the compiler
adds no wait states.  tests/isa_lint.py checks the emitted gfx950 assembly for results read too
early; here it is first shown to reject planted mistakes, then run on the real kernels."""
import os
import subprocess

import pytest

from paper_2503_12964_amd import build
from tests import isa_lint as L

MFMA_V = "v_mfma_f32_32x32x16_bf16 v[0:15], v[20:23], a[0:3], 0"
MFMA_V_ACC = "v_mfma_f32_32x32x16_bf16 v[0:15], v[24:27], a[4:7], v[0:15]"
OTHER = "v_mfma_f32_32x32x16_bf16 v[32:47], v[20:23], a[0:3], 0"


def _asm(*lines):
    out = []
    for l in lines:
        if l.startswith("!"):                  # an assembly statement
            out += ["\t;;#ASMSTART", "\t" + l[1:], "\t;;#ASMEND"]
        elif l.endswith(":"):
            out.append(l)
        else:
            out.append("\t" + l)
    return "\n".join(out) + "\n\ts_endpgm\n"


def test_reader_directly_behind_the_mfma_is_reported():
    bad = L.check(_asm("!" + MFMA_V, "v_add_f32_e32 v60, v3, v61"))
    assert len(bad) == 1 and "v_add_f32_e32" in bad[0]


def test_writer_of_one_register_of_the_tuple_is_reported():
    assert len(L.check(_asm("!" + MFMA_V, "v_mov_b32_e32 v15, 0"))) == 1
    assert L.check(_asm("!" + MFMA_V, "v_mov_b32_e32 v16, 0")) == []
    assert L.check(_asm("!" + MFMA_V, "v_accvgpr_write_b32 a3, v99")) == []      # the other register file


def test_one_mfma_between_is_not_enough_two_are():
    assert len(L.check(_asm("!" + MFMA_V, OTHER, "v_exp_f32_e32 v70, v7"))) == 1
    assert L.check(_asm("!" + MFMA_V, OTHER, OTHER.replace("32:47", "48:63"), "v_exp_f32_e32 v70, v7")) == []


def test_wait_states_count():
    assert L.check(_asm("!" + MFMA_V, "s_nop 15", "v_exp_f32_e32 v70, v7")) == []
    assert len(L.check(_asm("!" + MFMA_V, "s_nop 13", "v_exp_f32_e32 v70, v7"))) == 1
    body = ["v_mov_b32_e32 v%d, 0" % (100 + i) for i in range(16)]
    assert L.check(_asm("!" + MFMA_V, *body, "v_exp_f32_e32 v70, v7")) == []
    assert len(L.check(_asm("!" + MFMA_V, *body[:12], "v_exp_f32_e32 v70, v7"))) == 1


def test_accumulation_chain_is_allowed_but_its_end_is_checked():
    assert L.check(_asm("!" + MFMA_V, "!" + MFMA_V_ACC, "s_nop 15", "v_exp_f32_e32 v70, v7")) == []
    bad = L.check(_asm("!" + MFMA_V, "!" + MFMA_V_ACC, "v_exp_f32_e32 v70, v7"))
    assert len(bad) == 1 and "line 7" in bad[0]
    # an MFMA that reads the tuple as its A operand is a reader, not a link of the chain
    reads_a = "v_mfma_f32_32x32x16_bf16 v[32:47], v[0:3], a[0:3], 0"
    assert len(L.check(_asm("!" + MFMA_V, reads_a))) == 1


def test_reader_at_the_top_of_a_loop_is_found_through_the_branch():
    loop = ["loop:", "v_exp_f32_e32 v70, v7", OTHER, OTHER, "!" + MFMA_V, "s_cbranch_scc1 loop", OTHER, OTHER]
    bad = L.check(_asm(*loop))
    assert len(bad) == 1 and "v_exp_f32_e32" in bad[0]
    safe = ["loop:", OTHER, OTHER, "v_exp_f32_e32 v70, v7", "!" + MFMA_V, "s_cbranch_scc1 loop", OTHER, OTHER]
    assert L.check(_asm(*safe)) == []
    jump = ["!" + MFMA_V, "s_branch away", OTHER, OTHER, "away:", "v_exp_f32_e32 v70, v7"]
    assert len(L.check(_asm(*jump))) == 1


def test_compiler_selected_mfmas_are_left_to_the_compiler():
    assert L.check(_asm(MFMA_V, "v_add_f32_e32 v60, v3, v61")) == []


def test_backward_kernels_keep_the_rule(tmp_path):
    out = tmp_path / "attn_bwd.s"
    cmd = [build.HIPCC, *build.FLAGS, "--cuda-device-only", "-S", os.path.join(build.CSRC, "attn_bwd.hip"), "-o", str(out)]
    res = subprocess.run(cmd, capture_output=True, text=True)
    assert res.returncode == 0, res.stderr[-2000:]
    text = out.read_text()
    prog = L.parse(text)
    n_asm = sum(1 for i in prog.insts if i.from_asm and i.mnemonic.startswith("v_mfma"))
    assert n_asm >= 500, n_asm          # the markers were recognised: the dK/dV and dQ kernels hold hundreds
    bad = L.check(text)
    assert bad == [], "\n".join(bad[:20])


@pytest.mark.parametrize("src", [s for s in build.SOURCES if s not in ("attn_bwd.hip", "vfm_api.hip")])
def test_no_other_kernel_file_issues_mfmas_from_assembly(src):
    # were one to start doing so, it has to be added to the check above
    text = open(os.path.join(build.CSRC, src)).read()
    assert 'asm volatile("v_mfma' not in text and "mfma32_v(" not in text and "mfma32_acc(" not in text
