"""Host-side checks of the C-ABI library that need no GPU: it loads, exports every symbol the
header declares, sizes its workspaces, and rejects bad arguments before launching anything."""
import ctypes
import os
import re

import pytest

from paper_2503_15798_amd import binding as mb

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
A16 = 0x1000   # a fake, 16-byte aligned, non-null address: validation must fail before any use


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "mole.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(mole_[a-z_]+)\s*\(", text)))


def test_library_loads_and_exports_every_declared_symbol():
    lib = mb.lib()
    syms = declared_symbols()
    assert set(syms) == set(mb.EXPORTS)
    for s in syms:
        assert getattr(lib, s) is not None
    assert mb.mole_version() == 2
    assert mb.mole_last_error() == ""


def test_workspace_sizes():
    assert mb.mole_dedup_workspace(0, 50304) > 0
    w1, w2 = mb.mole_dedup_workspace(256, 50304), mb.mole_dedup_workspace(16384, 50304)
    assert 0 < w1 < w2 and w2 % 16 == 0
    assert mb.mole_dedup_workspace(-1, 50304) == 0
    ws = mb.mole_build_lut_workspace(50304, 1024, 4096, 16, mb.MOLE_BF16)
    assert 2 * 16 * 1024 * 4096 * 2 < ws < 16 * 2 ** 30
    assert mb.mole_build_lut_workspace(1024, 64, 256, 4, mb.MOLE_F32) >= 1024 * 4 * 256 * 4
    assert mb.mole_build_lut_workspace(1024, 60, 256, 4, mb.MOLE_F32) == 0      # d not a multiple of 16


def fwd(**kw):
    a = dict(table=A16, ids=A16, slot=None, h=A16, W_r=A16, shared_out=A16, residual=None, out=A16,
             gates_dbg=None, rows_dbg=None, err_flag=None, T=4, rows=100, d=64, N=4, dtype=mb.MOLE_BF16,
             flags=0, workspace=None, stream=0, workspace_bytes=0)
    a.update(kw)
    return mb.mole_lookup_forward(**a)


@pytest.mark.parametrize("kw,status,needle", [
    (dict(table=None), mb.MOLE_EINVAL, "must not be NULL"),
    (dict(out=None), mb.MOLE_EINVAL, "must not be NULL"),
    (dict(T=-1), mb.MOLE_EINVAL, "bad size"),
    (dict(rows=0), mb.MOLE_EINVAL, "bad size"),
    (dict(d=60), mb.MOLE_EUNSUPPORTED, "multiple of 8"),
    (dict(d=6, dtype=mb.MOLE_F32), mb.MOLE_EUNSUPPORTED, "multiple of 4"),
    (dict(N=0), mb.MOLE_EUNSUPPORTED, "outside 1..64"),
    (dict(N=65), mb.MOLE_EUNSUPPORTED, "outside 1..64"),
    (dict(dtype=7), mb.MOLE_EINVAL, "unknown dtype"),
    (dict(flags=8), mb.MOLE_EINVAL, "unknown flags"),
    (dict(h=A16 + 4), mb.MOLE_EINVAL, "16-byte aligned"),
    (dict(flags=mb.MOLE_FLAG_DEDUP), mb.MOLE_EWORKSPACE, "plan"),
    (dict(flags=mb.MOLE_FLAG_RUNS), mb.MOLE_EINVAL, "MOLE_FLAG_RUNS needs MOLE_FLAG_DEDUP"),
    (dict(flags=mb.MOLE_FLAG_DEDUP, workspace=A16, workspace_bytes=64), mb.MOLE_EWORKSPACE, "plan"),
])
def test_forward_rejects_bad_arguments_without_launching(kw, status, needle):
    with pytest.raises(mb.MoleError) as e:
        fwd(**kw)
    assert e.value.status == status
    assert needle in e.value.message
    assert needle in mb.mole_last_error()


def test_forward_with_no_tokens_is_a_noop():
    fwd(T=0, table=None, ids=None, h=None, W_r=None, out=None)      # MOLE_OK, nothing launched
    assert mb.mole_last_error() == ""


def test_layers_variant_checks_strides():
    with pytest.raises(mb.MoleError) as e:
        mb.mole_lookup_forward_layers(A16, 10, A16, None, A16, A16, None, None, A16, 4 * 64, None, None, None,
                                      L=2, T=4, rows=100, d=64, N=4, dtype=mb.MOLE_BF16, stream=0)
    assert e.value.status == mb.MOLE_EINVAL and "stride" in e.value.message


def test_dedup_rejects_bad_arguments():
    need = mb.mole_dedup_workspace(8, 100)
    cases = [
        (dict(T=-1), mb.MOLE_EINVAL), (dict(V=0), mb.MOLE_EINVAL), (dict(V=1 << 20), mb.MOLE_EUNSUPPORTED),
        (dict(ids=None), mb.MOLE_EINVAL), (dict(n_uniq=None), mb.MOLE_EINVAL),
        (dict(workspace=None), mb.MOLE_EWORKSPACE), (dict(workspace_bytes=need - 1), mb.MOLE_EWORKSPACE),
        (dict(workspace=A16 + 8), mb.MOLE_EINVAL),
    ]
    for kw, status in cases:
        a = dict(ids=A16, T=8, V=100, uniq=A16, inv=A16, n_uniq=A16, err_flag=None, workspace=A16, stream=0,
                 workspace_bytes=need)
        a.update(kw)
        with pytest.raises(mb.MoleError) as e:
            mb.mole_dedup_ids(**a)
        assert e.value.status == status, kw


def test_build_lut_rejects_bad_arguments():
    need = mb.mole_build_lut_workspace(128, 64, 256, 4, mb.MOLE_F32)
    cases = [
        (dict(E=None), mb.MOLE_EINVAL), (dict(LUT=None), mb.MOLE_EINVAL), (dict(V=0), mb.MOLE_EINVAL),
        (dict(N=65), mb.MOLE_EUNSUPPORTED), (dict(D=250), mb.MOLE_EUNSUPPORTED), (dict(act=5), mb.MOLE_EINVAL),
        (dict(workspace=None), mb.MOLE_EWORKSPACE), (dict(workspace_bytes=need - 1), mb.MOLE_EWORKSPACE),
        (dict(W1=A16 + 2), mb.MOLE_EINVAL),
    ]
    for kw, status in cases:
        a = dict(E=A16, W1=A16, b1=None, W2=A16, b2=None, norm_w=None, norm_eps=1e-5, LUT=A16, V=128, d=64,
                 D=256, N=4, dtype=mb.MOLE_F32, act=mb.MOLE_GELU_ERF, workspace=A16, stream=0,
                 workspace_bytes=need)
        a.update(kw)
        with pytest.raises(mb.MoleError) as e:
            mb.mole_build_lut(**a)
        assert e.value.status == status, kw


def test_offload_fetch_rejects_bad_arguments():
    cases = [
        (dict(host_table=None), mb.MOLE_EINVAL), (dict(L=0), mb.MOLE_EINVAL), (dict(d=3, N=1), mb.MOLE_EUNSUPPORTED),
        (dict(staging=A16 + 8), mb.MOLE_EINVAL), (dict(L=2, host_layer_stride=5), mb.MOLE_EINVAL),
    ]
    for kw, status in cases:
        a = dict(host_table=A16, host_layer_stride=0, uniq=A16, n_uniq=A16, staging=A16, staging_layer_stride=0,
                 err_flag=None, L=1, U_cap=8, V=100, d=64, N=4, dtype=mb.MOLE_BF16, stream=0)
        a.update(kw)
        with pytest.raises(mb.MoleError) as e:
            mb.mole_offload_fetch(**a)
        assert e.value.status == status, kw
    a = dict(host_table=A16, host_layer_stride=0, uniq=A16, n_uniq=A16, staging=A16, staging_layer_stride=0,
             err_flag=None, L=1, U_cap=0, V=100, d=64, N=4, dtype=mb.MOLE_BF16, stream=0)
    mb.mole_offload_fetch(**a)      # nothing to fetch: MOLE_OK without a launch


def test_layer_forward_rejects_bad_arguments():
    base = dict(table=A16, table_stride=0, ids=A16, slot=None, x=A16, ln_w=A16, ln_eps=1e-5, W_r=A16,
                shared_out=None, out=A16, act_stride=0, gates_dbg=None, rows_dbg=None, err_flag=None, L=1, T=4,
                rows=10, d=64, N=4, dtype=mb.MOLE_BF16, flags=0, workspace=None, stream=0, workspace_bytes=0)
    cases = [(dict(W_r=None), mb.MOLE_EINVAL), (dict(ln_w=None), mb.MOLE_EINVAL), (dict(ln_eps=-1.0), mb.MOLE_EINVAL),
             (dict(ln_eps=float("nan")), mb.MOLE_EINVAL), (dict(x=None), mb.MOLE_EINVAL),
             (dict(W_r=A16 + 2), mb.MOLE_EINVAL), (dict(ln_w=A16 + 2), mb.MOLE_EINVAL),
             (dict(d=60), mb.MOLE_EUNSUPPORTED),
             (dict(flags=mb.MOLE_FLAG_DEDUP), mb.MOLE_EWORKSPACE)]
    for kw, status in cases:
        a = dict(base)
        a.update(kw)
        with pytest.raises(mb.MoleError) as e:
            mb.mole_layer_forward(**a)
        assert e.value.status == status, kw
    a = dict(base)
    a.update(T=0)
    mb.mole_layer_forward(**a)          # empty batch: MOLE_OK, nothing launched


def test_set_tuning():
    """Knobs are named after their environment variables; an unknown name or a negative value is refused."""
    mb.mole_set_tuning("MOLE_FWD_SPLIT", 2)
    mb.mole_set_tuning("MOLE_FWD_SPLIT", 0)
    for name, value in (("MOLE_NO_SUCH_KNOB", 1), ("MOLE_FWD_WPB", -1)):
        with pytest.raises(mb.MoleError) as e:
            mb.mole_set_tuning(name, value)
        assert e.value.status == mb.MOLE_EINVAL


def test_offload_fetch_idmajor_rejects_bad_arguments():
    base = dict(host_table=A16, uniq=A16, n_uniq=A16, staging=A16, staging_layer_stride=8 * 4 * 64, err_flag=None,
                L=2, U_cap=8, V=100, d=64, N=4, dtype=mb.MOLE_BF16, stream=0)
    cases = [(dict(host_table=None), mb.MOLE_EINVAL), (dict(n_uniq=None), mb.MOLE_EINVAL),
             (dict(staging=None), mb.MOLE_EINVAL), (dict(L=0), mb.MOLE_EINVAL), (dict(dtype=5), mb.MOLE_EINVAL),
             (dict(d=3, N=1), mb.MOLE_EUNSUPPORTED), (dict(host_table=A16 + 4), mb.MOLE_EINVAL),
             (dict(staging_layer_stride=8 * 4 * 64 - 8), mb.MOLE_EINVAL)]
    for kw, status in cases:
        a = dict(base)
        a.update(kw)
        with pytest.raises(mb.MoleError) as e:
            mb.mole_offload_fetch_idmajor(**a)
        assert e.value.status == status, kw
        assert "mole_offload_fetch_idmajor" in e.value.message
    a = dict(base)
    a.update(U_cap=0)
    mb.mole_offload_fetch_idmajor(**a)      # nothing to fetch: MOLE_OK without a launch


def test_layer_forward_nf_rejects_bad_arguments():
    base = dict(codes=A16, codes_stride=0, scales=A16, scales_stride=0, ids=A16, slot=None, x=A16, ln_w=A16,
                ln_eps=1e-5, W_r=A16, shared_out=None, out=A16, act_stride=0, gates_dbg=None, rows_dbg=None, err_flag=None, L=1,
                T=4, rows=10, d=64, N=4, bits=4, block=64, scale_bytes=4, flags=0, workspace=None, stream=0,
                workspace_bytes=0)
    cases = [(dict(ln_eps=-1.0), mb.MOLE_EINVAL), (dict(ln_eps=float("nan")), mb.MOLE_EINVAL),
             (dict(x=None), mb.MOLE_EINVAL), (dict(W_r=None), mb.MOLE_EINVAL), (dict(ln_w=None), mb.MOLE_EINVAL),
             (dict(bits=5), mb.MOLE_EUNSUPPORTED),
             (dict(N=5), mb.MOLE_EUNSUPPORTED), (dict(x=A16 + 2), mb.MOLE_EINVAL),
             (dict(flags=mb.MOLE_FLAG_DEDUP), mb.MOLE_EWORKSPACE)]
    for kw, status in cases:
        a = dict(base)
        a.update(kw)
        with pytest.raises(mb.MoleError) as e:
            mb.mole_layer_forward_nf(**a)
        assert e.value.status == status, kw
        assert "mole_layer_forward_nf" in e.value.message or status == mb.MOLE_EUNSUPPORTED
    a = dict(base)
    a.update(T=0)
    mb.mole_layer_forward_nf(**a)           # empty batch: MOLE_OK, nothing launched


def test_offload_fetch_nf_rejects_bad_arguments():
    V, N, d, U = 100, 4, 64, 8
    base = dict(host_codes=A16, host_codes_stride=V * N * d // 2, host_scales=A16, host_scales_stride=V * N,
                uniq=A16, n_uniq=A16, staging_codes=A16, staging_codes_stride=U * N * d // 2, staging_scales=A16,
                staging_scales_stride=U * N, err_flag=None, L=2, U_cap=U, V=V, d=d, N=N, bits=4, block=64,
                scale_bytes=4, stream=0)
    cases = [(dict(bits=5), mb.MOLE_EUNSUPPORTED), (dict(scale_bytes=3), mb.MOLE_EINVAL), (dict(L=0), mb.MOLE_EINVAL),
             (dict(d=60), mb.MOLE_EUNSUPPORTED), (dict(block=48), mb.MOLE_EUNSUPPORTED),
             (dict(host_codes=None), mb.MOLE_EINVAL), (dict(host_scales=None), mb.MOLE_EINVAL),
             (dict(uniq=None), mb.MOLE_EINVAL), (dict(staging_scales=None), mb.MOLE_EINVAL),
             (dict(host_codes_stride=V * N * d // 2 - 2), mb.MOLE_EINVAL),        # smaller than one layer
             (dict(staging_scales_stride=U * N - 1), mb.MOLE_EINVAL),
             (dict(host_codes=A16 + 1), mb.MOLE_EUNSUPPORTED)]                     # odd address
    for kw, status in cases:
        a = dict(base)
        a.update(kw)
        with pytest.raises(mb.MoleError) as e:
            mb.mole_offload_fetch_nf(**a)
        assert e.value.status == status, kw
        assert "mole_offload_fetch_nf" in e.value.message
    a = dict(base)
    a.update(U_cap=0)
    mb.mole_offload_fetch_nf(**a)           # nothing to fetch: MOLE_OK without a launch


def test_product_package_does_not_import_the_oracle():
    """The product path must never route through the CPU oracle: no import, no path, no dlopen."""
    pkg = os.path.join(ROOT, "paper_2503_15798_amd")
    pat = re.compile(r"^\s*(import|from)\s+oracle\b|libmole_oracle|mole_oracle_|[\"']oracle[\"/']", re.M)
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h", ".cpp")):
                text = open(os.path.join(dirpath, f)).read()
                assert not pat.search(text), f"{f} reaches for the oracle"


def test_bench_refuses_more_than_one_gpu_and_runs_nothing_without_one():
    """bench.py measures one GPU: --gpus N > 1 exits with a message that says so; without a GPU it exits
    before touching the library (no CPU fallback)."""
    import os
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode == 2 and "ONE GPU" in r.stderr and r.stdout.strip() == ""
    import torch
    if not torch.cuda.is_available():
        r = subprocess.run([sys.executable, os.path.join(root, "bench.py")], capture_output=True, text=True)
        assert r.returncode == 3 and "no GPU" in r.stderr and r.stdout.strip() == ""
