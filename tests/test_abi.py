"""The C-ABI library loads and exports every symbol include/aircache.h declares; host-side argument
validation answers before anything touches a GPU."""
import ctypes as C
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _lib():
    import paper_2503_23956_amd as A
    from paper_2503_23956_amd import binding

    if not os.path.exists(binding.LIB_PATH):
        from paper_2503_23956_amd.build import build

        build(verbose=False)
    return A.load_library()


def _declared():
    text = open(os.path.join(ROOT, "include", "aircache.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(air_[a-z_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported():
    lib = _lib()
    names = _declared()
    assert len(names) >= 17
    for n in names:
        assert hasattr(lib, n), f"{n} declared in aircache.h but not exported"
    from paper_2503_23956_amd import binding

    assert sorted(binding.EXPORTS) == names
    assert lib.air_version().startswith(b"aircache")


def test_invalid_configs_are_rejected_on_the_host():
    import paper_2503_23956_amd as A

    lib = _lib()
    good = dict(n_layers=2, n_q_heads=4, n_kv_heads=2, head_dim=64, batch=1, max_vis_len=576, max_nonvis_len=80,
                max_window=16, max_decode_steps=1, dtype=A.AIR_F32)
    assert lib.air_workspace_bytes(C.byref(A.make_config(**good))) > 0
    for bad in (dict(head_dim=96), dict(n_q_heads=5), dict(batch=0), dict(batch=65), dict(max_window=100),
                dict(dtype=7), dict(n_layers=0), dict(max_vis_len=0)):
        cfg = A.make_config(**{**good, **bad})
        assert lib.air_workspace_bytes(C.byref(cfg)) == 0, bad
    for kw in (dict(alpha=1.5), dict(retention=0.0), dict(retention=1.2), dict(min_keep=-1), dict(budget_mode=9)):
        assert lib.air_workspace_bytes(C.byref(A.make_config(**good, **kw))) == 0, kw
    # the units of one layer (batch x KV heads) must fit a grid dimension
    assert lib.air_workspace_bytes(C.byref(A.make_config(**{**good, "batch": 64, "n_q_heads": 1024, "n_kv_heads": 1024}))) == 0
    # visual observation window: no Eq.5, so alpha must be 0; the span may then be as long as the visual span
    assert lib.air_workspace_bytes(C.byref(A.make_config(**good, window_kind=A.AIR_WINDOW_VISUAL))) == 0  # alpha 0.9
    assert lib.air_workspace_bytes(C.byref(A.make_config(**good, window_kind=A.AIR_WINDOW_VISUAL, alpha=0.0))) > 0
    assert lib.air_workspace_bytes(C.byref(A.make_config(**{**good, "max_window": 100}, window_kind=A.AIR_WINDOW_VISUAL,
                                                         alpha=0.0))) > 0
    assert lib.air_workspace_bytes(C.byref(A.make_config(**{**good, "max_window": 600}, window_kind=A.AIR_WINDOW_VISUAL,
                                                         alpha=0.0))) == 0
    assert lib.air_workspace_bytes(C.byref(A.make_config(**good, window_kind=2, alpha=0.0))) == 0
    h = C.c_void_p()
    cfg = A.make_config(**good)
    assert lib.air_create(C.byref(cfg), None, 1 << 30, C.byref(h)) == A.binding.AIR_ERR_WORKSPACE
    assert lib.air_create(C.byref(cfg), 256, 16, C.byref(h)) == A.binding.AIR_ERR_WORKSPACE
    assert lib.air_create(C.byref(cfg), 260, 1 << 30, C.byref(h)) == A.binding.AIR_ERR_WORKSPACE  # misaligned
    assert lib.air_create(C.byref(A.make_config(**{**good, "head_dim": 96})), 256, 1 << 30, C.byref(h)) == A.binding.AIR_ERR_SHAPE
    assert lib.air_create(None, 256, 1 << 30, C.byref(h)) == A.binding.AIR_ERR_INVALID_ARG
    assert not h.value
    assert lib.air_destroy(None) == A.binding.AIR_ERR_INVALID_ARG
    assert lib.air_budget(None, None) == A.binding.AIR_ERR_INVALID_ARG
    assert lib.air_set_tuning(None, None) == A.binding.AIR_ERR_INVALID_ARG
    assert lib.air_decode_attn_static(None, None, 0, 1, None, None, None, None) == A.binding.AIR_ERR_INVALID_ARG
    # the in-place cache exists for the bf16 / head_dim 128 kernels only
    assert lib.air_workspace_bytes(C.byref(A.make_config(**good, cache_in_place=1))) == 0
    big = dict(good, head_dim=128, dtype=A.AIR_BF16)
    with_pool = lib.air_workspace_bytes(C.byref(A.make_config(**big)))
    without = lib.air_workspace_bytes(C.byref(A.make_config(**big, cache_in_place=1)))
    assert 0 < without < with_pool


def test_missing_library_fails_loudly(tmp_path):
    import paper_2503_23956_amd as A

    with pytest.raises(FileNotFoundError):
        A.load_library(str(tmp_path / "libaircache.so"))


def test_index_division_by_batch_as_one_multiply():
    """The kernels split a grid index z = b + B * layer (z < 2^16, B <= 64) with the high word of
    z * (floor(2^32 / B) + 1); the quotient must be exact over the whole range."""
    import numpy as np

    z = np.arange(1 << 16, dtype=np.uint64)
    for B in range(2, 65):
        inv = np.uint64((1 << 32) // B + 1)
        assert np.array_equal((z * inv) >> np.uint64(32), z // np.uint64(B)), B


def test_binding_structs_follow_the_header_field_by_field():
    """The ctypes structures of the binding against the struct bodies of include/aircache.h: same fields, same order,
    same C types (a field added on one side only would shift everything behind it without any error)."""
    from paper_2503_23956_amd import binding

    text = open(os.path.join(ROOT, "include", "aircache.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    ctype = {"int32_t": C.c_int32, "int64_t": C.c_int64, "double": C.c_double, "void": C.c_void_p}
    for name in ("air_config", "air_seq", "air_layer", "air_strides", "air_tuning"):
        m = re.search(r"typedef struct\s*\{([^}]*)\}\s*" + name + r"\s*;", text)
        assert m, name
        fields = []
        for decl in m.group(1).split(";"):
            decl = decl.strip()
            if not decl:
                continue
            mm = re.match(r"(?:const\s+)?(\w+)\s+(.*)", decl)
            base, rest = mm.group(1), mm.group(2)
            for var in rest.split(","):
                var = var.strip()
                fields.append((var.lstrip("*").strip(), C.c_void_p if var.startswith("*") else ctype[base]))
        got = [(n, t) for n, t in getattr(binding, name)._fields_]
        assert got == fields, (name, got, fields)
