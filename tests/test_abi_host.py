"""Host-only checks of the C ABI: the library loads, exports every symbol the header declares,
and rejects bad arguments before touching the GPU (no compute call is made here)."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "moe.h")
LIB = os.path.join(ROOT, "paper_1701_06538_amd", "libmoe_hip.so")


@pytest.fixture(scope="module")
def api():
    if not os.path.exists(LIB):
        from paper_1701_06538_amd import build
        build.build()
    from paper_1701_06538_amd import api as _api
    return _api


def declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    names = re.findall(r"\b(moe_[a-z0-9_]+)\s*\(", text)
    return sorted(set(names))


def test_header_declares_the_named_entry_points():
    names = declared_functions()
    for must in ("moe_gate", "moe_route", "moe_expert_ffn", "moe_combine", "moe_aux_losses",
                 "moe_layer_forward"):
        assert must in names


def test_library_exports_every_declared_symbol(api):
    lib = ctypes.CDLL(LIB)
    for name in declared_functions():
        assert hasattr(lib, name), "missing export: " + name


def test_python_binding_has_the_same_names(api):
    for name in declared_functions():
        assert hasattr(api, name), "binding lacks " + name


def test_status_strings_and_version(api):
    assert api.moe_version() >= 100
    for st in (0, -1, -2, -3, -4):
        assert api.moe_strerror(st)
    assert "unknown" in api.moe_strerror(-99)


def test_bad_shapes_are_rejected_on_the_host(api):
    ok = dict(T=64, d=512, h=1024, n=16, k=4)
    assert api.moe_workspace_bytes(api.make_config(**ok)) > 0
    bad = [dict(ok, k=0), dict(ok, k=17, n=32), dict(ok, k=9, n=32), dict(ok, n=0), dict(ok, d=0),
           dict(ok, T=-1), dict(ok, k=5, n=4), dict(ok, expert_dtype=7), dict(ok, a=4, b=3),
           dict(ok, a=4, b=4, k_primary=2, k_secondary=3), dict(ok, n=20000), dict(ok, d=500)]
    for kw in bad:
        cfg = api.make_config(**kw)
        assert api.moe_workspace_bytes(cfg) == 0, kw
        with pytest.raises(api.MoeError):
            api.moe_get_workspace_layout(cfg)
    hier = api.make_config(T=64, d=512, h=1024, n=64, k=4, a=8, b=8, k_primary=2, k_secondary=2)
    assert api.moe_workspace_bytes(hier) > 0


def test_null_pointers_are_rejected_before_any_launch(api):
    cfg = api.make_config(T=64, d=512, h=1024, n=16, k=4)
    for call, nargs in ((api._moe_gate, 12), (api._moe_route, 10), (api._moe_expert_ffn, 11),
                        (api._moe_combine, 5), (api._moe_aux_losses, 6)):
        st = call(ctypes.byref(cfg), *([None] * nargs))
        assert st == api.MOE_EINVAL
    st = api._moe_layer_forward(ctypes.byref(cfg), *([None] * 14), 0, None)
    assert st == api.MOE_EINVAL
    st = api._moe_layer_backward(ctypes.byref(cfg), *([None] * 16), 0, None)
    assert st in (api.MOE_EINVAL, api.MOE_EUNSUPPORTED)
    hier = api.make_config(T=64, d=512, h=1024, n=64, k=4, a=8, b=8, k_primary=2, k_secondary=2)
    assert api._moe_gate_hier(ctypes.byref(hier), *([None] * 10), 0, None) == api.MOE_EINVAL
    assert api._moe_layer_forward_hier(ctypes.byref(hier), *([None] * 16), 0, None) == api.MOE_EINVAL
    assert api._moe_aux_losses_hier(ctypes.byref(hier), *([None] * 4), 0, *([None] * 4)) == api.MOE_EINVAL
    # flat entry points refuse a hierarchical shape and vice versa
    assert api._moe_gate_hier(ctypes.byref(cfg), *([None] * 10), 0, None) == api.MOE_EINVAL


def test_backward_workspace_and_flags(api):
    cfg = api.make_config(T=65536, d=512, h=1024, n=512, k=4)
    assert api.moe_backward_workspace_bytes(cfg) > 2 * 262144 * 1024 * 2
    L0 = api.moe_get_workspace_layout(cfg)
    assert L0.hidden == 2 ** 64 - 1                      # absent without the flag
    cfg1 = api.make_config(T=65536, d=512, h=1024, n=512, k=4, flags=api.MOE_FLAG_SAVE_HIDDEN)
    L1 = api.moe_get_workspace_layout(cfg1)
    assert L1.hidden != 2 ** 64 - 1 and L1.total - L0.total >= 262144 * 1024 * 2
    # the kept input rows: absent without the flag, and their own block after the hidden rows with it
    assert L0.xs == 2 ** 64 - 1
    assert L1.xs >= L1.hidden + 262144 * 1024 * 2 and L1.xs + 262144 * 512 * 2 <= L1.total
    f32s = api.make_config(T=64, d=512, h=1024, n=32, k=4, expert_dtype=api.MOE_DTYPE_F32,
                           flags=api.MOE_FLAG_SAVE_HIDDEN)
    Lf = api.moe_get_workspace_layout(f32s)
    assert Lf.hidden == 2 ** 64 - 1 and Lf.xs == 2 ** 64 - 1
    hs = api.make_config(T=64, d=512, h=1024, n=64, k=4, a=8, b=8, k_primary=2, k_secondary=2,
                         flags=api.MOE_FLAG_SAVE_HIDDEN)
    Lh = api.moe_get_workspace_layout(hs)
    assert Lh.hidden != 2 ** 64 - 1 and Lh.xs == 2 ** 64 - 1
    f32 = api.make_config(T=64, d=512, h=1024, n=32, k=4, expert_dtype=api.MOE_DTYPE_F32)
    assert api.moe_backward_workspace_bytes(f32) > 0
    hier = api.make_config(T=64, d=512, h=1024, n=64, k=4, a=8, b=8, k_primary=2, k_secondary=2)
    assert api.moe_backward_workspace_bytes(hier) == 0   # flat layer only
    # the hierarchical backward workspace grows by the sums of squares when they are asked for
    hm = api.make_config(T=64, d=512, h=1024, n=1024, k=4, a=32, b=32, k_primary=2, k_secondary=2)
    hm2 = api.make_config(T=64, d=512, h=1024, n=1024, k=4, a=32, b=32, k_primary=2, k_secondary=2,
                          flags=api.MOE_FLAG_ADAM_MOMENTS)
    grow = api.moe_backward_hier_workspace_bytes(hm2) - api.moe_backward_hier_workspace_bytes(hm)
    assert api.moe_backward_hier_workspace_bytes(hm) > 0 and grow >= 1024 * (4 * 512 + 2 * 1024) * 2 * 4


def test_layout_struct_of_the_binding_matches_the_library(api):
    """The library fills exactly the fields the binding declares: bytes past the binding's struct stay
    untouched and its last field is written."""
    import ctypes
    size = ctypes.sizeof(api.MoeWorkspaceLayout)
    buf = (ctypes.c_ubyte * (size + 64))(*([0xAB] * (size + 64)))
    cfg = api.make_config(T=8192, d=512, h=1024, n=256, k=4)
    fn = api._lib.moe_get_workspace_layout
    assert fn(ctypes.byref(cfg), ctypes.cast(buf, ctypes.POINTER(api.MoeWorkspaceLayout))) == 0
    assert bytes(buf[size:]) == b"\xab" * 64
    L = api.MoeWorkspaceLayout.from_buffer_copy(bytes(buf[:size]))
    assert L.xs == 2 ** 64 - 1 and L.hidden == 2 ** 64 - 1 and L.total == api.moe_workspace_bytes(cfg)
    fields = [getattr(L, f) for f, _ in api.MoeWorkspaceLayout._fields_]
    assert 0xABABABABABABABAB not in fields
    # the header lists the same fields in the same order
    import re
    from pathlib import Path
    text = Path(__file__).resolve().parents[1].joinpath("include", "moe.h").read_text()
    body = text[text.index("typedef struct moe_workspace_layout {"):text.index("} moe_workspace_layout;")]
    body = re.sub(r"/\*.*?\*/", "", body, flags=re.S)
    names = re.findall(r"\b([a-z_0-9]+)\s*[,;]", body)
    assert names == [f for f, _ in api.MoeWorkspaceLayout._fields_]


def test_workspace_layout_is_ordered_aligned_and_sized(api):
    cfg = api.make_config(T=8192, d=512, h=1024, n=256, k=4)
    L = api.moe_get_workspace_layout(cfg)
    offs = [L.cleanb, L.sp, L.next_idx, L.partials, L.counts, L.offsets, L.perm, L.inv_perm,
            L.tile_expert, L.tile_row0, L.num_tiles, L.route_ws, L.out_sorted, L.ffn_ws, L.aux_ws]
    assert offs == sorted(offs) and all(o % 256 == 0 for o in offs)
    assert L.sp - L.cleanb >= 8192 * 256 * 4
    assert L.total == api.moe_workspace_bytes(cfg)
    assert L.total >= L.out_sorted + 8192 * 4 * 512 * 4
    assert api.moe_max_tiles(cfg) == 8192 * 4 // api.moe_tile_rows(cfg) + 256
    assert api.moe_gate_partial_rows(cfg) == 8192 // 8
    f32 = api.make_config(T=256, d=512, h=1024, n=16, k=4, expert_dtype=api.MOE_DTYPE_F32)
    assert api.moe_ffn_workspace_bytes(f32) == 256 * 4 * 1024 * 4
    assert api.moe_ffn_workspace_bytes(cfg) == 0


def test_widened_entry_points_validate_on_the_host(api):
    """Balanced gating, threshold inference, the hierarchical backward, the Adam step and the combine
    epilogue reject bad shapes and null pointers before anything is launched."""
    flat = api.make_config(T=64, d=512, h=1024, n=16, k=4)
    assert api.moe_balanced_rows_per_expert(flat) == 16
    assert api.moe_balanced_workspace_bytes(flat) > 0
    odd = api.make_config(T=63, d=512, h=1024, n=16, k=3)            # 189 rows do not split over 16 experts
    assert api.moe_balanced_rows_per_expert(odd) == -1 and api.moe_balanced_workspace_bytes(odd) == 0
    assert api._moe_gate_balanced(ctypes.byref(flat), *([None] * 10), 0, None) == api.MOE_EINVAL
    assert api._moe_gate_balanced(ctypes.byref(odd), *([None] * 10), 0, None) == api.MOE_EINVAL
    assert api._moe_layer_forward_balanced(ctypes.byref(flat), *([None] * 13), 0, None) == api.MOE_EINVAL
    assert api.moe_threshold_workspace_bytes(flat, 1000) > api.moe_threshold_workspace_bytes(flat, 10) > 0
    assert api.moe_threshold_workspace_bytes(flat, -1) == 0
    assert api._moe_layer_forward_threshold(ctypes.byref(flat), *([None] * 6), 100, *([None] * 8), 0, None) == api.MOE_EINVAL
    hier = api.make_config(T=64, d=512, h=1024, n=1024, k=4, a=32, b=32, k_primary=2, k_secondary=2)
    assert api.moe_backward_hier_workspace_bytes(hier) > 0
    assert api.moe_backward_hier_workspace_bytes(flat) == 0
    small_groups = api.make_config(T=64, d=512, h=1024, n=64, k=4, a=8, b=8, k_primary=2, k_secondary=2)
    assert api.moe_backward_hier_workspace_bytes(small_groups) == 0   # group counts off the GEMM slabs
    assert api._moe_layer_backward_hier(ctypes.byref(hier), *([None] * 21), 0, None) == api.MOE_EINVAL
    assert api._moe_layer_backward_hier(ctypes.byref(flat), *([None] * 21), 0, None) == api.MOE_EINVAL
    assert api.moe_adam_workspace_bytes(flat) > 0
    hp = api.MoeAdamParams(1e-3, 0.999, 1e-8, 1)
    assert api._moe_expert_adam_step(ctypes.byref(flat), ctypes.byref(hp), *([None] * 12), 0, None) == api.MOE_EINVAL
    assert api._moe_combine_epilogue(ctypes.byref(flat), *([None] * 5), 0.0, None, None) == api.MOE_EINVAL
    # backward with balanced gating: needs a balanced batch, and the flat backward's expert shapes
    assert api.moe_backward_balanced_workspace_bytes(flat) > 0
    assert api.moe_backward_balanced_workspace_bytes(odd) == 0
    assert api._moe_layer_backward_balanced(ctypes.byref(flat), *([None] * 11), 0.0, *([None] * 5), 0, None) == api.MOE_EINVAL
    assert api._moe_layer_backward_balanced(ctypes.byref(odd), *([None] * 11), 0.0, *([None] * 5), 0, None) == api.MOE_EINVAL
    off_tile = api.make_config(T=64, d=384, h=1024, n=16, k=4)          # bf16 experts: d, h multiples of 256
    assert api._moe_layer_backward_balanced(ctypes.byref(off_tile), *([None] * 11), 0.0, *([None] * 5), 0, None) == api.MOE_EUNSUPPORTED
    # fp32 experts and expert counts off the tile sizes are accepted by the flat backward
    assert api.moe_backward_workspace_bytes(api.make_config(T=64, d=64, h=96, n=20, k=2, expert_dtype=api.MOE_DTYPE_F32)) > 0
