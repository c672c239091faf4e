"""The compiler's output is searched for spill stores that run under a narrowed exec mask (host only).

One build of the scan kernel lost the target side's scale factor that way (see
paper_2506_05632_amd/audit.py); the checker is pinned on small listings with and without the
pattern, then run over the assembly of every source of the library as it is built."""
from paper_2506_05632_amd import audit

FAULTY = """
_Z6kernelv:
\tv_mul_f32_e32 v113, s4, v2
.LBB0_1:
\tv_cmp_eq_u32_e32 vcc, 4, v0
\ts_and_saveexec_b64 s[4:5], s[10:11]
; %bb.179:
\tv_writelane_b32 v127, s58, 37
\tscratch_store_dword off, v113, off offset:8 ; 4-byte Folded Spill
\tv_writelane_b32 v127, s59, 38
\ts_or_b64 exec, exec, s[4:5]
\tscratch_load_dword v58, off, off offset:8 ; 4-byte Folded Reload
\ts_endpgm
"""

# the store comes before the narrowing; a value made inside the narrowed stretch is stored there;
# the mask is whole again before the store; another stretch of code begins before the store
SOUND = """
_Z6kernelv:
\tv_mul_f32_e32 v113, s4, v2
\tscratch_store_dword off, v113, off offset:8 ; 4-byte Folded Spill
\ts_and_saveexec_b64 s[4:5], s[10:11]
\tv_add_f32_e32 v7, v1, v2
\tscratch_store_dword off, v7, off offset:12 ; 4-byte Folded Spill
\tv_fma_f64 v[20:21], v[2:3], v[4:5], v[6:7]
\tscratch_store_dwordx2 off, v[20:21], off offset:16 ; 8-byte Folded Spill
\ts_or_b64 exec, exec, s[4:5]
\tscratch_store_dword off, v113, off offset:20 ; 4-byte Folded Spill
\ts_and_saveexec_b64 s[4:5], s[10:11]
\ts_cbranch_execz .LBB0_3
.LBB0_2:
\tscratch_store_dword off, v113, off offset:24 ; 4-byte Folded Spill
.LBB0_3:
\ts_or_b64 exec, exec, s[4:5]
\ts_endpgm
"""


def test_the_checker_finds_the_pattern_and_only_the_pattern():
    found = audit.spill_stores_under_narrowed_exec(FAULTY)
    assert len(found) == 1
    kernel, line, narrowing, store = found[0]
    assert kernel == "_Z6kernelv" and narrowing.startswith("s_and_saveexec_b64") and "v113" in store
    assert audit.spill_stores_under_narrowed_exec(SOUND) == []
    # a pair of registers counts if either half was made before the narrowing
    pair = FAULTY.replace("scratch_store_dword off, v113,", "scratch_store_dwordx2 off, v[112:113],")
    assert len(audit.spill_stores_under_narrowed_exec(pair)) == 1


def test_no_kernel_of_the_library_stores_a_spill_under_a_narrowed_exec_mask():
    bad = audit.audit()
    assert bad == {}, bad
