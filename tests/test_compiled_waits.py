"""The compiled kernels, as assembly: every workgroup barrier is preceded, on every path from an LDS
store or atomic of the same wave, by a wait that empties lgkmcnt.  (One loop of the block-mass kernel
once lacked it: the compiler had dropped the LDS part of the wait that __syncthreads() asks for, and
partial sums were read stale now and then.)  Runs on the CPU, on what the build keeps in _build/."""
import os

from paper_2605_19726_amd import build, lds_wait_audit as audit


def _asm_files():
    files = audit.default_files()
    if len(files) < len(build.SOURCES):
        build.build(verbose=False)
        files = audit.default_files()
    return files


def test_every_source_has_its_assembly_and_none_lacks_the_wait():
    files = _asm_files()
    names = {os.path.basename(f).split("-hip-")[0] + ".hip" for f in files}
    assert names == set(build.SOURCES), names
    assert audit.audit_files(files) == []


def test_the_audit_sees_a_missing_wait_across_a_loop_edge_and_accepts_the_repaired_form():
    # the shape that was found: the store sits in a conditional tail of the loop body, the barrier at the
    # top of the next iteration has a wait for vmcnt only
    broken = """_Zkernel:
	s_mov_b32 s0, 0
.LBB0_1:
	s_waitcnt vmcnt(0)
	s_barrier
	ds_read_b32 v1, v0
	s_waitcnt lgkmcnt(0)
	s_cbranch_execz .LBB0_3
.LBB0_2:
	ds_write_b32 v3, v2
.LBB0_3:
	s_add_i32 s0, s0, 1
	s_cmp_lt_i32 s0, 8
	s_cbranch_scc1 .LBB0_1
	s_endpgm
.Lfunc_end0:
""".split("\n")
    (name, body), = list(audit._functions(broken))
    found = audit.audit_function(body)
    assert found == [(".LBB0_1", "ds_write_b32 v3, v2", ".LBB0_2")]
    fixed = [l.replace("s_waitcnt vmcnt(0)", "s_waitcnt vmcnt(0) lgkmcnt(0)") for l in broken]
    (name, body), = list(audit._functions(fixed))
    assert audit.audit_function(body) == []
