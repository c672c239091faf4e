"""Host-side checks of the C ABI that need no GPU: symbols, struct layout, argument errors."""
import ctypes
import os
import re
import subprocess
import sys

import pytest

import paper_2506_05632_amd as llc
from paper_2506_05632_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "llc.h")


def declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(llc_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = llc.load()
    names = declared_functions()
    assert set(names) == set(binding.EXPORTS)
    for name in names:
        assert getattr(lib, name) is not None
    assert llc.llc_version() == 110
    assert llc.llc_status_string(0) == "ok"
    assert "workspace" in llc.llc_status_string(-6)


def test_probe_library_exports_its_declared_symbol_and_its_header_is_plain_c(tmp_path):
    # the machine probes of the benchmark live in a library of their own (no compute call here)
    text = re.sub(r"/\*.*?\*/", "", open(os.path.join(ROOT, "include", "llc_probe.h")).read(), flags=re.S)
    names = sorted(set(re.findall(r"\b(llc_[a-z_]+)\s*\(", text)))
    assert names == ["llc_probe_run"]
    lib = ctypes.CDLL(os.path.join(ROOT, "paper_2506_05632_amd", "libllc_probe.so"))
    for name in names:
        assert getattr(lib, name) is not None
    src = tmp_path / "probe.c"
    src.write_text('#include "llc_probe.h"\nint main(void){ return LLC_PROBE_PHILOX_READ == 6 ? 0 : 1; }\n')
    exe = tmp_path / "probe"
    subprocess.run(["gcc", "-std=c99", "-Wall", "-Werror", "-pedantic", "-I", os.path.join(ROOT, "include"),
                    str(src), "-o", str(exe)], check=True)
    assert subprocess.run([str(exe)]).returncode == 0


def test_header_is_plain_c_and_matches_the_binding_layout(tmp_path):
    src = tmp_path / "layout.c"
    src.write_text(
        '#include <stdio.h>\n#include <stddef.h>\n#include "llc.h"\n'
        "int main(void){printf(\"%zu %zu %zu %zu %zu %zu %zu %zu %zu %zu\\n\", sizeof(llc_couple_args),"
        " sizeof(llc_couple_is_args), sizeof(llc_stats), offsetof(llc_couple_args, temp_draft),"
        " offsetof(llc_couple_args, workspace), offsetof(llc_couple_args, ev_scan_begin),"
        " offsetof(llc_couple_is_args, workspace), sizeof(llc_verify_args),"
        " offsetof(llc_verify_args, tokens), offsetof(llc_verify_args, workspace));"
        " printf(\"%zu %zu %zu\\n\", sizeof(llc_couple_topm_args), offsetof(llc_couple_topm_args, temp_draft),"
        " offsetof(llc_couple_topm_args, stream));"
        " printf(\"%zu %zu %zu\\n\", sizeof(llc_compress_select_args), offsetof(llc_compress_select_args, bins),"
        " offsetof(llc_compress_select_args, workspace));"
        " printf(\"%zu %zu %zu %zu\\n\", sizeof(llc_lml_args), offsetof(llc_lml_args, k),"
        " offsetof(llc_lml_args, bound), offsetof(llc_lml_args, ev_begin)); return 0;}\n")
    exe = tmp_path / "layout"
    subprocess.run(["gcc", "-std=c99", "-Wall", "-Werror", "-pedantic", "-I", os.path.join(ROOT, "include"),
                    str(src), "-o", str(exe)], check=True)
    got = [int(v) for v in subprocess.run([str(exe)], capture_output=True, text=True, check=True).stdout.split()]
    want = [ctypes.sizeof(binding.CoupleArgs), ctypes.sizeof(binding.CoupleIsArgs),
            ctypes.sizeof(binding.LlcStats), binding.CoupleArgs.temp_draft.offset,
            binding.CoupleArgs.workspace.offset, binding.CoupleArgs.ev_scan_begin.offset,
            binding.CoupleIsArgs.workspace.offset, ctypes.sizeof(binding.VerifyArgs),
            binding.VerifyArgs.tokens.offset, binding.VerifyArgs.workspace.offset,
            ctypes.sizeof(binding.TopmArgs), binding.TopmArgs.temp_draft.offset, binding.TopmArgs.stream.offset,
            ctypes.sizeof(binding.CompressSelectArgs), binding.CompressSelectArgs.bins.offset,
            binding.CompressSelectArgs.workspace.offset,
            ctypes.sizeof(binding.LmlArgs), binding.LmlArgs.k.offset, binding.LmlArgs.bound.offset,
            binding.LmlArgs.ev_begin.offset]
    assert got == want


def _args(**kw):
    a = binding.CoupleArgs()
    a.B, a.K, a.V = 4, 2, 64
    a.dtype, a.kind = binding.F32, binding.LOGITS
    a.draft = a.target = 0x1000
    a.draft_stride_b = a.target_stride_b = 64
    a.temp_target = a.temp_draft_all = 1.0
    a.X = a.Y = a.accept = 0x2000
    a.workspace, a.workspace_bytes = 0x4000, 1 << 30
    for k, v in kw.items():
        setattr(a, k, v)
    return a


@pytest.mark.parametrize("kw,code", [
    (dict(draft=None), -1), (dict(Y=None), -1),
    (dict(K=0), -2), (dict(V=0), -2), (dict(B=-1), -2), (dict(K=70000), -2), (dict(V=1 << 31), -2),
    (dict(draft_stride_b=-1), -2),
    (dict(temp_target=0.0), -3), (dict(temp_target=float("nan")), -3), (dict(temp_draft_all=-1.0), -3),
    (dict(dtype=7), -4), (dict(kind=5), -4),
    (dict(draft=0x1002), -5),
    (dict(workspace=None), -6), (dict(workspace=0x4010), -6), (dict(workspace_bytes=16), -6),
    (dict(flags=64), -8), (dict(flags=2), -8), (dict(v_chunks=5000), -8), (dict(k_tile=3), -8),
])
def test_argument_errors_are_reported_before_any_launch(kw, code):
    # every one of these returns on the host: no kernel runs, no GPU is needed
    lib = llc.load()
    assert lib.llc_couple(ctypes.byref(_args(**kw))) == code


def test_a_launch_of_more_than_2_to_the_24_workgroups_is_refused_up_front():
    lib = llc.load()
    a = _args(B=1 << 21, K=15, V=8, draft_stride_b=8, target_stride_b=8, k_tile=2, flags=binding.FLAG_DRY_RUN)
    assert lib.llc_couple(ctypes.byref(a)) == -2
    a = _args(B=1 << 21, K=15, V=8, draft_stride_b=8, target_stride_b=8, k_tile=4, flags=binding.FLAG_DRY_RUN,
              workspace_bytes=1 << 34)
    assert lib.llc_couple(ctypes.byref(a)) == 0


def test_null_struct_and_empty_batch():
    lib = llc.load()
    assert lib.llc_couple(None) == -1
    assert lib.llc_couple_is(None) == -1
    assert lib.llc_couple(ctypes.byref(_args(B=0, draft=None, X=None))) == 0
    assert llc.llc_couple_workspace_size(0, 1, 1) > 0
    assert llc.llc_couple_workspace_size(4, 0, 64) == 0
    big = llc.llc_couple_workspace_size(1024, 8, 128256)
    assert 0 < big < 64 << 20


def test_probability_kind_ignores_temperatures():
    # temperatures are not validated for kinds that do not use them; a bad workspace then is the first error
    lib = llc.load()
    assert lib.llc_couple(ctypes.byref(_args(kind=binding.PROBS, temp_target=0.0, workspace=None))) == -6


def test_product_does_not_import_the_oracle():
    code = ("import sys; import paper_2506_05632_amd; "
            "assert not any(m == 'oracle' or m.startswith('oracle.') for m in sys.modules), 'oracle imported'")
    subprocess.run([sys.executable, "-c", code], check=True, cwd=ROOT)


def test_missing_library_fails_loudly(tmp_path, monkeypatch):
    code = ("import paper_2506_05632_amd as m\n"
            "m.binding.LIB_PATH = '/nonexistent/libllc_hip.so'\n"
            "try:\n    m.load()\nexcept RuntimeError as e:\n    print('raised')\n")
    out = subprocess.run([sys.executable, "-c", code], capture_output=True, text=True, cwd=ROOT)
    assert "raised" in out.stdout


def _verify_args(**kw):
    a = binding.VerifyArgs()
    a.S, a.L, a.K, a.V = 3, 2, 2, 64
    a.dtype, a.kind = binding.F32, binding.LOGITS
    a.target = 0x1000
    a.stride_s, a.stride_j, a.stride_k = 3 * 2 * 64, 2 * 64, 64
    a.temp_target = 1.0
    a.tokens, a.tok_stride_s, a.tok_stride_j = 0x3000, 4, 2
    a.row_stride_s, a.row_stride_j = 3, 1
    a.Y = a.n_out = 0x2000
    a.workspace, a.workspace_bytes = 0x4000, 1 << 30
    for k, v in kw.items():
        setattr(a, k, v)
    return a


@pytest.mark.parametrize("kw,code", [
    (dict(target=None), -1), (dict(Y=None), -1), (dict(n_out=None), -1), (dict(tokens=None), -1),
    (dict(K=65), -2), (dict(K=0), -2), (dict(L=-1), -2), (dict(S=-1), -2), (dict(V=0), -2),
    (dict(stride_j=-1), -2), (dict(row_stride_s=-1), -2),
    (dict(temp_target=0.0), -3),
    (dict(kind=binding.PROBS), -4), (dict(dtype=9), -4),
    (dict(target=0x1002), -5),
    (dict(workspace=None), -6), (dict(workspace_bytes=1024), -6),
    (dict(k_tile=5), -8), (dict(flags=32), -8),
])
def test_verify_argument_errors_are_reported_before_any_launch(kw, code):
    lib = llc.load()
    assert lib.llc_verify(ctypes.byref(_verify_args(**kw))) == code


def test_verify_null_struct_empty_batch_and_workspace_size():
    lib = llc.load()
    assert lib.llc_verify(None) == -1
    assert lib.llc_verify(ctypes.byref(_verify_args(S=0, target=None, Y=None))) == 0
    assert llc.llc_verify_workspace_size(3, 2, 2, 64) > llc.llc_couple_workspace_size(9, 2, 64)
    assert llc.llc_verify_workspace_size(3, 2, 65, 64) == 0


@pytest.mark.parametrize("S,L,K,V", [
    (128, 4, 8, 128256), (64, 4, 8, 152064),          # draft lengths and list sizes of the paper's runs
    (128, 7, 8, 128256), (1, 4, 8, 151936), (3, 5, 2, 152064), (17, 4, 6, 32000), (1000, 1, 5, 32000),
    (2, 4, 64, 128256), (5, 0, 8, 50000), (256, 4, 4, 1000), (9, 12, 9, 40000), (33, 3, 16, 262144),
])
@pytest.mark.parametrize("bf16", [False, True])
def test_verify_takes_exactly_the_workspace_it_asks_for_in_both_forms(S, L, K, V, bf16):
    """Every launch of the call is planned before the first one (the dry run stops there): the
    one-shot scan over S(L+1) rows with per-draft rows, and, in the strong form, the scans of the
    later positions over S rows in the shared-proposal layout, which split V over more workgroups."""
    lib = llc.load()
    need = llc.llc_verify_workspace_size(S, L, K, V)
    assert need > 0
    shape = dict(S=S, L=L, K=K, V=V, stride_k=V, stride_j=K * V, stride_s=(L + 1) * K * V,
                 tok_stride_j=K, tok_stride_s=L * K, row_stride_s=L + 1,
                 dtype=binding.BF16 if bf16 else binding.F32)
    for flags in (binding.FLAG_DRY_RUN, binding.FLAG_DRY_RUN | binding.FLAG_STRONG):
        for kt in (0, 2, 4, 8):
            for vc in (0, 1, 16):
                a = _verify_args(workspace_bytes=need, flags=flags, k_tile=kt, v_chunks=vc, **shape)
                assert lib.llc_verify(ctypes.byref(a)) == 0, (flags, kt, vc)
        a = _verify_args(workspace_bytes=1024, flags=flags, **shape)
        assert lib.llc_verify(ctypes.byref(a)) == -6


def test_dry_run_plans_the_other_calls_too():
    lib = llc.load()
    for B, K, V in [(1024, 8, 128256), (512, 16, 152064), (1, 8, 128256), (7, 65535, 37), (256, 4, 32000)]:
        need = llc.llc_couple_workspace_size(B, K, V)
        for sk in (0, V):
            for kt in (0, 2, 4, 8):
                for vc in (0, 1, 16):
                    a = _args(B=B, K=K, V=V, draft_stride_b=max(sk * K, V), draft_stride_k=sk, target_stride_b=V,
                              workspace_bytes=need, flags=binding.FLAG_DRY_RUN, k_tile=kt, v_chunks=vc)
                    assert lib.llc_couple(ctypes.byref(a)) == 0, (B, K, V, sk, kt, vc)
        a = _args(B=B, K=K, V=V, draft_stride_b=V, target_stride_b=V, workspace_bytes=512,
                  flags=binding.FLAG_DRY_RUN)
        assert lib.llc_couple(ctypes.byref(a)) == -6


def test_the_draft_only_flag_needs_neither_target_nor_target_side_outputs():
    lib = llc.load()
    do = binding.FLAG_DRAFT_ONLY | binding.FLAG_DRY_RUN
    a = _args(flags=do, target=None, Y=None, accept=None, target_stride_b=0)
    assert lib.llc_couple(ctypes.byref(a)) == 0
    assert lib.llc_couple(ctypes.byref(_args(flags=do | binding.FLAG_MIN_FIRST, target=None, Y=None, accept=None))) == 0
    assert lib.llc_couple(ctypes.byref(_args(flags=do, draft=None))) == -1
    assert lib.llc_couple(ctypes.byref(_args(flags=do, X=None))) == -1
    assert lib.llc_couple(ctypes.byref(_args(flags=binding.FLAG_DRY_RUN, target=None))) == -1   # without the flag
    assert lib.llc_couple(ctypes.byref(_args(flags=do, temp_target=0.0, target=None, Y=None, accept=None))) == 0
    assert lib.llc_couple(ctypes.byref(_args(flags=do, temp_draft_all=0.0))) == -3
    a = _verify_args(flags=binding.FLAG_DRAFT_ONLY)
    assert lib.llc_verify(ctypes.byref(a)) == -8


def test_the_min_first_flag_is_planned_like_the_default_and_refused_where_it_is_not_built():
    lib = llc.load()
    mf = binding.FLAG_MIN_FIRST | binding.FLAG_DRY_RUN
    for B, K, V in [(1024, 8, 128256), (512, 16, 152064), (7, 65535, 37)]:
        need = llc.llc_couple_workspace_size(B, K, V)
        for sk in (0, V):
            a = _args(B=B, K=K, V=V, draft_stride_b=max(sk * K, V), draft_stride_k=sk, target_stride_b=V,
                      workspace_bytes=need, flags=mf)
            assert lib.llc_couple(ctypes.byref(a)) == 0
    a = _verify_args(flags=mf)
    a.workspace_bytes = llc.llc_verify_workspace_size(a.S, a.L, a.K, a.V)
    assert lib.llc_verify(ctypes.byref(a)) == 0
    a = _verify_args(flags=mf | binding.FLAG_STRONG)
    a.workspace_bytes = llc.llc_verify_workspace_size(a.S, a.L, a.K, a.V)
    assert lib.llc_verify(ctypes.byref(a)) == 0
    # the binned passes draw one word per (index, draft) only
    assert lib.llc_compress_select(ctypes.byref(_select_args(flags=mf))) == -8


def _topm_args(**kw):
    a = binding.TopmArgs()
    a.B, a.K, a.Md, a.Mt = 4, 2, 8, 8
    a.dtype, a.kind = binding.F32, binding.LOGITS
    a.draft_ids = a.target_ids = 0x1000
    a.draft_val = a.target_val = 0x3000
    a.draft_stride_b = a.target_stride_b = 8
    a.temp_target = a.temp_draft_all = 1.0
    a.X = a.Y = a.accept = 0x2000
    for k, v in kw.items():
        setattr(a, k, v)
    return a


@pytest.mark.parametrize("kw,code", [
    (dict(draft_ids=None), -1), (dict(target_val=None), -1), (dict(accept=None), -1),
    (dict(K=0), -2), (dict(K=1025), -2), (dict(Md=0), -2), (dict(Mt=70000), -2), (dict(B=-1), -2),
    (dict(target_stride_b=-8), -2),
    (dict(temp_draft_all=0.0), -3), (dict(temp_target=float("inf")), -3),
    (dict(dtype=3), -4), (dict(kind=-1), -4),
    (dict(draft_val=0x3002), -5), (dict(target_ids=0x1001), -5),
])
def test_topm_argument_errors_are_reported_before_any_launch(kw, code):
    lib = llc.load()
    assert lib.llc_couple_topm(ctypes.byref(_topm_args(**kw))) == code
    assert lib.llc_couple_topm(None) == -1
    assert lib.llc_couple_topm(ctypes.byref(_topm_args(B=0, draft_ids=None, X=None))) == 0


def _select_args(**kw):
    a = binding.CompressSelectArgs()
    a.B, a.L, a.N = 4, 2, 64
    a.logw_enc = a.logw_dec = 0x1000
    a.enc_stride_b, a.dec_stride_b, a.dec_stride_l = 64, 128, 64
    a.bins, a.bins_stride_b = 0x5000, 64
    a.X = a.Y = a.accept = 0x2000
    a.workspace, a.workspace_bytes = 0x4000, 1 << 30
    for k, v in kw.items():
        setattr(a, k, v)
    return a


@pytest.mark.parametrize("kw,code", [
    (dict(bins=None), -1), (dict(logw_dec=None), -1), (dict(Y=None), -1),
    (dict(L=0), -2), (dict(N=0), -2), (dict(bins_stride_b=-1), -2),
    (dict(logw_enc=0x1002), -5),
    (dict(workspace=None), -6), (dict(workspace_bytes=8), -6),
    (dict(flags=2), -8), (dict(k_tile=7), -8),
])
def test_compress_select_argument_errors_are_reported_before_any_launch(kw, code):
    lib = llc.load()
    assert lib.llc_compress_select(ctypes.byref(_select_args(**kw))) == code
    assert lib.llc_compress_select(None) == -1
    assert lib.llc_compress_select(ctypes.byref(_select_args(B=0, bins=None, X=None))) == 0


def _lml_args(**kw):
    a = binding.LmlArgs()
    a.B, a.V = 4, 64
    a.dtype, a.kind = binding.F32, binding.LOGITS
    a.draft = a.target = 0x1000
    a.draft_stride_b = a.target_stride_b = 64
    a.temp_target = a.temp_draft = 1.0
    a.n_k = 2
    a.k[0], a.k[1] = 1, 8
    a.bound = 0x2000
    a.workspace, a.workspace_bytes = 0x4000, 1 << 30
    for k, v in kw.items():
        setattr(a, k, v)
    return a


@pytest.mark.parametrize("kw,code", [
    (dict(draft=None), -1), (dict(bound=None), -1),
    (dict(V=0), -2), (dict(B=-1), -2), (dict(target_stride_b=-1), -2), (dict(V=(1 << 28) + 1), -2),
    (dict(temp_draft=0.0), -3), (dict(temp_target=float("nan")), -3),
    (dict(dtype=2), -4), (dict(kind=9), -4),
    (dict(target=0x1001), -5),
    (dict(workspace=None), -6), (dict(workspace=0x4008), -6), (dict(workspace_bytes=1000), -6),
    (dict(n_k=0), -8), (dict(n_k=9), -8),
])
def test_lml_argument_errors_are_reported_before_any_launch(kw, code):
    lib = llc.load()
    assert lib.llc_lml_bound(ctypes.byref(_lml_args(**kw))) == code
    assert lib.llc_lml_bound(None) == -1
    bad_k = _lml_args()
    bad_k.k[1] = 0
    assert lib.llc_lml_bound(ctypes.byref(bad_k)) == -8
    assert lib.llc_lml_bound(ctypes.byref(_lml_args(B=0, draft=None, bound=None))) == 0
    assert llc.llc_lml_workspace_size(4, 64) >= 4 * 64 * 24
    assert llc.llc_lml_workspace_size(4, 0) == 0
    assert llc.llc_lml_workspace_size(100000, 128256) == llc.llc_lml_workspace_size(512, 128256)   # capped
    assert llc.llc_lml_workspace_size(1, 1 << 28) >= 24 << 28 and llc.llc_lml_workspace_size(1, (1 << 28) + 1) == 0
