"""The C-ABI library loads on a machine without a GPU and exports exactly what the header declares."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "lfps.h")


def _declared():
    src = open(HEADER).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    return sorted(set(re.findall(r"\b(lfps_[a-z_0-9]+)\s*\(", src)))


def test_header_declares_the_named_entry_points():
    names = _declared()
    for must in ("lfps_create", "lfps_candidates", "lfps_score_topk", "lfps_sparse_attn", "lfps_step",
                 "lfps_full_attn_decode", "lfps_exact_topk", "lfps_destroy"):
        assert must in names


def test_library_exports_every_declared_symbol():
    from paper_2506_15704_amd import binding
    lib = ctypes.CDLL(binding.LIB_PATH)
    for name in _declared():
        assert hasattr(lib, name), f"{name} declared in lfps.h but not exported"


def test_binding_covers_every_declared_symbol():
    from paper_2506_15704_amd import binding
    for name in _declared():
        assert hasattr(binding._lib, name)
        assert getattr(binding._lib, name).argtypes is not None, f"{name} has no ctypes signature"


def test_config_validation_without_gpu():
    from paper_2506_15704_amd import binding as b
    good = dict(batch=2, n_q_heads=32, n_kv_heads=8, head_dim=128, kv_dtype=1, max_seq_len=4096, max_k=128,
                radius=2, n_recent=1, n_sink=0, cand_cap=0, device=0)
    assert b.workspace_bytes(**good) > 0
    for bad in (dict(head_dim=64), dict(n_q_heads=24), dict(batch=0), dict(max_k=0), dict(max_k=5000),
                dict(radius=-1), dict(kv_dtype=7), dict(n_q_heads=64), dict(batch=2048)):
        with pytest.raises(b.LfpsError) as ei:
            b.workspace_bytes(**{**good, **bad})
        assert ei.value.code == b.LFPS_EINVAL
    with pytest.raises(b.LfpsError) as ei:
        b.workspace_bytes(**{**good, "max_seq_len": 1_000_000})
    assert ei.value.code == b.LFPS_ECAP
    # table mode: decay in (0, 1), a > 0, radius <= 30; the tables add to the workspace
    tab = {**good, "table_mode": 1, "table_decay": 0.95, "table_a": 0.2}
    assert b.workspace_bytes(**tab) > b.workspace_bytes(**good) + 2 * 32 * 4096 * 12
    for bad in (dict(table_decay=0.0), dict(table_decay=1.0), dict(table_a=0.0), dict(radius=31), dict(table_mode=2)):
        with pytest.raises(b.LfpsError) as ei:
            b.workspace_bytes(**{**tab, **bad})
        assert ei.value.code == b.LFPS_EINVAL
    # FP8 keys / values: flags are 0 or 1 and need the two-byte (bf16) cache description
    assert b.workspace_bytes(**{**good, "k_fp8": 1, "v_fp8": 1}) > 0
    assert b.workspace_bytes(**{**good, "kv_dtype": b.LFPS_F16}) == b.workspace_bytes(**good)   # fp16: same sizes as bf16
    for bad in (dict(k_fp8=2), dict(v_fp8=-1), dict(k_fp8=1, kv_dtype=0), dict(v_fp8=1, kv_dtype=0),
                dict(k_fp8=1, kv_dtype=b.LFPS_F16), dict(kv_dtype=3)):
        with pytest.raises(b.LfpsError) as ei:
            b.workspace_bytes(**{**good, **bad})
        assert ei.value.code == b.LFPS_EINVAL


def test_kernel_names():
    from paper_2506_15704_amd import binding as b
    names = b.kernel_names()
    assert len(names) == b.N_KERNELS and names[0] == "candidates" and "gather_score" in names


def _struct_fields(name):
    """(C type, field name) pairs of `typedef struct { ... } name;` in the header, in order."""
    src = open(HEADER).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    body = re.search(r"typedef struct \{([^}]*)\}\s*" + name + r"\s*;", src).group(1)
    out = []
    for decl in body.split(";"):
        decl = decl.strip()
        if not decl:
            continue
        parts = [p.strip() for p in decl.split(",")]
        m = re.match(r"(.+?[\s\*])([A-Za-z_0-9]+)$", parts[0])      # "<type> <first name>"
        ctype = m.group(1).strip()
        if ctype.endswith("*"):
            ctype = "ptr"
        for n in [m.group(2)] + parts[1:]:
            out.append((ctype, n))
    return out


def test_binding_structs_mirror_the_header_field_by_field():
    from paper_2506_15704_amd import binding as b
    ctype_of = {"int32_t": ctypes.c_int32, "int64_t": ctypes.c_int64, "float": ctypes.c_float, "ptr": ctypes.c_void_p}
    for name, cls in (("lfps_config", b.lfps_config), ("lfps_kv", b.lfps_kv)):
        want = [(n, ctype_of[t]) for t, n in _struct_fields(name)]
        got = [(f[0], f[1]) for f in cls._fields_]
        assert got == want, f"{name}: binding {got} != header {want}"


def test_bench_refuses_more_than_one_gpu():
    """The one-GPU build says so instead of running a multi-GPU job it does not have."""
    import os
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    res = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                         timeout=120)
    assert res.returncode != 0
    assert "one-GPU" in (res.stdout + res.stderr)


def test_binding_raises_without_the_library(tmp_path):
    """No CPU path in the product: a copy of the package without liblfps.so cannot even be imported."""
    import os
    import shutil
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    pkg = tmp_path / "paper_2506_15704_amd"
    pkg.mkdir()
    for name in ("__init__.py", "binding.py"):
        shutil.copy(os.path.join(root, "paper_2506_15704_amd", name), pkg / name)
    res = subprocess.run([sys.executable, "-c", "import paper_2506_15704_amd.binding"], capture_output=True, text=True,
                         cwd=str(tmp_path), env={**os.environ, "PYTHONPATH": str(tmp_path)}, timeout=300)
    assert res.returncode != 0
    assert "ImportError" in res.stderr and "no CPU fallback" in res.stderr
