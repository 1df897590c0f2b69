"""The build check for lane masks formed under a partial exec mask (see codegen_audit)."""
import os
import time

import codegen_audit as audit

# A kernel in the assembler's output format: a loop (BB0_2) forms a mask from a wave-uniform
# condition with a vector compare, a later loop (BB0_5) tests it.
_BAD = """\
_Z6kernelv:
; %bb.0:
\ts_cselect_b64 s[12:13], -1, 0
.LBB0_2:                                ; =>This Inner Loop Header: Depth=1
\tv_cndmask_b32_e64 v13, 0, 1, s[12:13]
\tv_cmp_ne_u32_e64 s[26:27], 1, v13
\ts_andn2_b64 exec, exec, s[14:15]
\ts_cbranch_execnz .LBB0_2
; %bb.3:
\ts_or_b64 exec, exec, s[14:15]
.LBB0_5:                                ; =>This Inner Loop Header: Depth=1
\ts_and_b64 vcc, exec, s[26:27]
\ts_cbranch_vccz .LBB0_5
\ts_endpgm
.Lfunc_end0:
"""

# the same mask, formed and tested inside one loop body: nothing to report
_GOOD = _BAD.replace(".LBB0_5:                                ; =>This Inner Loop Header: Depth=1\n", "") \
            .replace("; %bb.3:\n\ts_or_b64 exec, exec, s[14:15]\n", "") \
            .replace("\ts_andn2_b64 exec, exec, s[14:15]\n\ts_cbranch_execnz .LBB0_2\n", "") \
            .replace("\ts_cbranch_vccz .LBB0_5\n", "\ts_cbranch_vccz .LBB0_2\n")


def test_audit_reports_a_mask_formed_in_one_loop_and_tested_in_another(tmp_path):
    p = tmp_path / "bad.s"
    p.write_text(_BAD)
    found = audit.findings(str(p))
    assert len(found) == 1
    fn, d, u = found[0]
    assert fn == "_Z6kernelv" and d[1] == "BB0_2" and u[1] == "BB0_5" and "s[26:27]" in u[2]


def test_audit_accepts_a_mask_formed_and_tested_in_the_same_loop(tmp_path):
    p = tmp_path / "good.s"
    p.write_text(_GOOD)
    assert audit.findings(str(p)) == []


def test_audit_reports_per_peer_stores_that_each_drain_the_memory_pipeline(tmp_path):
    body = "".join("\ts_waitcnt vmcnt(0)\n\tglobal_store_dwordx4 v[50:51], v[6:9], off sc1 nt\n\ts_nop 1\n" for _ in range(8))
    p = tmp_path / "slow.s"
    p.write_text("_Z4slowv:\n" + body + "\ts_endpgm\n.Lfunc_end0:\n")
    assert audit.serialised_store_findings(str(p)) == [("_Z4slowv", 8, 8)]
    good = "\ts_waitcnt vmcnt(0)\n" + "".join("\tglobal_store_dwordx4 v[50:51], v[6:9], off sc1 nt\n\ts_nop 1\n" for _ in range(8))
    p.write_text("_Z4fastv:\n" + good + "\ts_endpgm\n.Lfunc_end0:\n")
    assert audit.serialised_store_findings(str(p)) == []


def test_device_code_has_no_partial_exec_uniform_masks(tmp_path):
    # the scan knows this compiler's idioms only: with any other it must be validated again (compile the
    # kernels without per_lane() and check that the scan finds the masks) before its silence means anything
    assert audit.VALIDATED_COMPILER in audit.compiler_version(), "codegen audit not validated for this hipcc"
    t0 = time.time()
    path = audit.device_assembly(str(tmp_path / "msx_device.s"))
    assert os.path.getsize(path) > 100000
    found = audit.findings(path)
    assert found == [], found[:3]
    slow = audit.serialised_store_findings(path)
    assert slow == [], slow
    print(f"audit: {time.time() - t0:.0f} s")
