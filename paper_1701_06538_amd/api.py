"""ctypes binding of include/moe.h.  Argument marshalling only: tensors are torch CUDA(HIP)
tensors used as device memory; every computation happens inside libmoe_hip.so."""
import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libmoe_hip.so")

MOE_OK, MOE_EINVAL, MOE_EUNSUPPORTED, MOE_EWORKSPACE, MOE_EHIP = 0, -1, -2, -3, -4
MOE_DTYPE_F32, MOE_DTYPE_BF16 = 0, 1
MOE_FLAG_SAVE_HIDDEN = 1
MOE_FLAG_ADAM_MOMENTS = 2

if not os.path.exists(LIB_PATH):
    raise ImportError(
        "libmoe_hip.so is missing: build it with `python -m paper_1701_06538_amd.build` "
        "(there is no CPU fallback)")
_lib = ctypes.CDLL(LIB_PATH)


class MoeConfig(ctypes.Structure):
    _fields_ = [("T", ctypes.c_int32), ("d", ctypes.c_int32), ("h", ctypes.c_int32),
                ("n", ctypes.c_int32), ("k", ctypes.c_int32), ("a", ctypes.c_int32),
                ("b", ctypes.c_int32), ("k_primary", ctypes.c_int32),
                ("k_secondary", ctypes.c_int32), ("expert_dtype", ctypes.c_int32),
                ("w_importance", ctypes.c_float), ("w_load", ctypes.c_float), ("flags", ctypes.c_int32)]


_LAYOUT_FIELDS = ["cleanb", "sp", "next_idx", "partials", "counts", "offsets", "perm", "inv_perm",
                  "tile_expert", "tile_row0", "num_tiles", "route_ws", "out_sorted", "ffn_ws",
                  "aux_ws", "hidden", "total", "p_cleanb", "p_sp", "p_next_idx", "p_partials", "p_idx",
                  "p_gate", "p_counts", "p_offsets", "p_perm", "p_inv_perm", "p_tile_group",
                  "p_tile_row0", "p_num_tiles", "p_tile_offsets", "p_route_ws", "p_aux_ws",
                  "s_idx", "s_gate", "xs"]


class MoeWorkspaceLayout(ctypes.Structure):
    _fields_ = [(name, ctypes.c_size_t) for name in _LAYOUT_FIELDS]


_cfgp = ctypes.POINTER(MoeConfig)
_vp = ctypes.c_void_p


def _proto(name, restype, argtypes):
    fn = getattr(_lib, name)
    fn.restype = restype
    fn.argtypes = argtypes
    return fn


_moe_version = _proto("moe_version", ctypes.c_int, [])
_moe_strerror = _proto("moe_strerror", ctypes.c_char_p, [ctypes.c_int])
_moe_last_hip_error = _proto("moe_last_hip_error", ctypes.c_int, [])
_moe_gate_partial_rows = _proto("moe_gate_partial_rows", ctypes.c_int64, [_cfgp])
_moe_route_workspace_bytes = _proto("moe_route_workspace_bytes", ctypes.c_size_t, [_cfgp])
_moe_tile_rows = _proto("moe_tile_rows", ctypes.c_int32, [_cfgp])
_moe_max_tiles = _proto("moe_max_tiles", ctypes.c_int64, [_cfgp])
_moe_ffn_workspace_bytes = _proto("moe_ffn_workspace_bytes", ctypes.c_size_t, [_cfgp])
_moe_aux_workspace_bytes = _proto("moe_aux_workspace_bytes", ctypes.c_size_t, [_cfgp])
_moe_workspace_bytes = _proto("moe_workspace_bytes", ctypes.c_size_t, [_cfgp])
_moe_get_workspace_layout = _proto("moe_get_workspace_layout", ctypes.c_int,
                                   [_cfgp, ctypes.POINTER(MoeWorkspaceLayout)])
_moe_gate = _proto("moe_gate", ctypes.c_int, [_cfgp] + [_vp] * 12)
_moe_route = _proto("moe_route", ctypes.c_int, [_cfgp] + [_vp] * 10)
_moe_route_static = _proto("moe_route_static", ctypes.c_int, [_cfgp] + [_vp] * 9)
_moe_expert_ffn = _proto("moe_expert_ffn", ctypes.c_int, [_cfgp] + [_vp] * 11)
_moe_combine = _proto("moe_combine", ctypes.c_int, [_cfgp] + [_vp] * 5)
_moe_aux_losses = _proto("moe_aux_losses", ctypes.c_int, [_cfgp] + [_vp] * 6)
_moe_layer_forward = _proto("moe_layer_forward", ctypes.c_int,
                            [_cfgp] + [_vp] * 14 + [ctypes.c_size_t, _vp])


_moe_layer_forward_profiled = _proto("moe_layer_forward_profiled", ctypes.c_int,
                                     [_cfgp] + [_vp] * 14 + [ctypes.c_size_t, ctypes.POINTER(_vp), _vp])


_moe_gate_hier = _proto("moe_gate_hier", ctypes.c_int, [_cfgp] + [_vp] * 10 + [ctypes.c_size_t, _vp])
_moe_aux_losses_hier = _proto("moe_aux_losses_hier", ctypes.c_int,
                              [_cfgp] + [_vp] * 4 + [ctypes.c_size_t] + [_vp] * 4)
_moe_layer_forward_hier = _proto("moe_layer_forward_hier", ctypes.c_int,
                                 [_cfgp] + [_vp] * 16 + [ctypes.c_size_t, _vp])


_moe_layer_forward_hier_profiled = _proto("moe_layer_forward_hier_profiled", ctypes.c_int,
                                          [_cfgp] + [_vp] * 16 + [ctypes.c_size_t, ctypes.POINTER(_vp), _vp])

_moe_backward_workspace_bytes = _proto("moe_backward_workspace_bytes", ctypes.c_size_t, [_cfgp])
_moe_layer_backward = _proto("moe_layer_backward", ctypes.c_int,
                             [_cfgp] + [_vp] * 16 + [ctypes.c_size_t, _vp])

_moe_balanced_rows_per_expert = _proto("moe_balanced_rows_per_expert", ctypes.c_int64, [_cfgp])
_moe_balanced_workspace_bytes = _proto("moe_balanced_workspace_bytes", ctypes.c_size_t, [_cfgp])
_moe_gate_balanced = _proto("moe_gate_balanced", ctypes.c_int, [_cfgp] + [_vp] * 10 + [ctypes.c_size_t, _vp])
_moe_layer_forward_balanced = _proto("moe_layer_forward_balanced", ctypes.c_int,
                                     [_cfgp] + [_vp] * 13 + [ctypes.c_size_t, _vp])
_moe_layer_forward_balanced_profiled = _proto("moe_layer_forward_balanced_profiled", ctypes.c_int,
                                              [_cfgp] + [_vp] * 13 + [ctypes.c_size_t, ctypes.POINTER(_vp), _vp])
_moe_threshold_workspace_bytes = _proto("moe_threshold_workspace_bytes", ctypes.c_size_t, [_cfgp, ctypes.c_int64])
_moe_layer_forward_threshold = _proto("moe_layer_forward_threshold", ctypes.c_int,
                                      [_cfgp] + [_vp] * 6 + [ctypes.c_int64] + [_vp] * 8 + [ctypes.c_size_t, _vp])

_moe_backward_hier_workspace_bytes = _proto("moe_backward_hier_workspace_bytes", ctypes.c_size_t, [_cfgp])
_moe_layer_backward_hier = _proto("moe_layer_backward_hier", ctypes.c_int,
                                  [_cfgp] + [_vp] * 21 + [ctypes.c_size_t, _vp])

_moe_combine_epilogue = _proto("moe_combine_epilogue", ctypes.c_int, [_cfgp] + [_vp] * 5 + [ctypes.c_float, _vp, _vp])

_moe_batchwise_loss_grad = _proto("moe_batchwise_loss_grad", ctypes.c_int, [_cfgp] + [_vp] * 4)
_moe_backward_balanced_workspace_bytes = _proto("moe_backward_balanced_workspace_bytes", ctypes.c_size_t, [_cfgp])
_moe_layer_backward_balanced = _proto("moe_layer_backward_balanced", ctypes.c_int,
                                      [_cfgp] + [_vp] * 11 + [ctypes.c_float] + [_vp] * 5 + [ctypes.c_size_t, _vp])


class MoeAdamParams(ctypes.Structure):
    _fields_ = [("lr", ctypes.c_float), ("beta2", ctypes.c_float), ("eps", ctypes.c_float),
                ("step", ctypes.c_int32)]


_moe_adam_workspace_bytes = _proto("moe_adam_workspace_bytes", ctypes.c_size_t, [_cfgp])
_moe_expert_adam_step = _proto("moe_expert_adam_step", ctypes.c_int,
                               [_cfgp, ctypes.POINTER(MoeAdamParams)] + [_vp] * 12 + [ctypes.c_size_t, _vp])


class MoeError(RuntimeError):
    def __init__(self, status):
        self.status = status
        msg = _moe_strerror(status).decode()
        if status == MOE_EHIP:
            msg += " (hipError %d)" % _moe_last_hip_error()
        super().__init__("moe status %d: %s" % (status, msg))


def _check(status):
    if status != MOE_OK:
        raise MoeError(status)


def make_config(shape=None, **kw) -> MoeConfig:
    """MoeConfig from a moe_workloads.MoEShape-like object and/or keyword overrides."""
    vals = dict(T=0, d=0, h=0, n=0, k=0, a=0, b=0, k_primary=0, k_secondary=0,
                expert_dtype=MOE_DTYPE_BF16, w_importance=0.1, w_load=0.1, flags=0)
    if shape is not None:
        for f in ("T", "d", "h", "n", "k", "a", "b", "k_primary", "k_secondary", "w_importance", "w_load"):
            vals[f] = getattr(shape, f)
        vals["expert_dtype"] = MOE_DTYPE_F32 if shape.expert_dtype == "f32" else MOE_DTYPE_BF16
    vals.update(kw)
    return MoeConfig(**vals)


def _ptr(t):
    if t is None:
        return None
    if isinstance(t, int):
        return t
    assert t.is_contiguous(), "tensors crossing the ABI must be contiguous"
    return t.data_ptr()


def _stream(stream):
    if stream is None:
        return torch.cuda.current_stream().cuda_stream
    if isinstance(stream, int):
        return stream
    return stream.cuda_stream


def moe_version():
    return _moe_version()


def moe_strerror(status):
    return _moe_strerror(status).decode()


def moe_last_hip_error():
    return _moe_last_hip_error()


def moe_gate_partial_rows(cfg):
    return _moe_gate_partial_rows(ctypes.byref(cfg))


def moe_route_workspace_bytes(cfg):
    return _moe_route_workspace_bytes(ctypes.byref(cfg))


def moe_tile_rows(cfg):
    return _moe_tile_rows(ctypes.byref(cfg))


def moe_max_tiles(cfg):
    return _moe_max_tiles(ctypes.byref(cfg))


def moe_ffn_workspace_bytes(cfg):
    return _moe_ffn_workspace_bytes(ctypes.byref(cfg))


def moe_aux_workspace_bytes(cfg):
    return _moe_aux_workspace_bytes(ctypes.byref(cfg))


def moe_workspace_bytes(cfg):
    return _moe_workspace_bytes(ctypes.byref(cfg))


def moe_get_workspace_layout(cfg):
    out = MoeWorkspaceLayout()
    _check(_moe_get_workspace_layout(ctypes.byref(cfg), ctypes.byref(out)))
    return out


def moe_gate(cfg, x, W_g, W_noise, gate_bias, eps, topk_idx, topk_gate, cleanb, sp, next_idx,
             partials, stream=None):
    _check(_moe_gate(ctypes.byref(cfg), _ptr(x), _ptr(W_g), _ptr(W_noise), _ptr(gate_bias),
                     _ptr(eps), _ptr(topk_idx), _ptr(topk_gate), _ptr(cleanb), _ptr(sp),
                     _ptr(next_idx), _ptr(partials), _stream(stream)))


def moe_route(cfg, topk_idx, counts, offsets, perm, inv_perm, tile_expert, tile_row0, num_tiles,
              workspace, stream=None):
    _check(_moe_route(ctypes.byref(cfg), _ptr(topk_idx), _ptr(counts), _ptr(offsets), _ptr(perm),
                      _ptr(inv_perm), _ptr(tile_expert), _ptr(tile_row0), _ptr(num_tiles),
                      _ptr(workspace), _stream(stream)))


MOE_ROUTE_STATIC_MAX_WORKSPACE_BYTES = 4 << 20


def moe_route_static(cfg, topk_idx, counts, offsets, perm, inv_perm, tile_expert, tile_row0, num_tiles,
                     stream=None):
    _check(_moe_route_static(ctypes.byref(cfg), _ptr(topk_idx), _ptr(counts), _ptr(offsets), _ptr(perm),
                             _ptr(inv_perm), _ptr(tile_expert), _ptr(tile_row0), _ptr(num_tiles),
                             _stream(stream)))


def moe_expert_ffn(cfg, x, perm, offsets, tile_expert, tile_row0, num_tiles, W1, W2, out_sorted,
                   workspace, stream=None):
    _check(_moe_expert_ffn(ctypes.byref(cfg), _ptr(x), _ptr(perm), _ptr(offsets), _ptr(tile_expert),
                           _ptr(tile_row0), _ptr(num_tiles), _ptr(W1), _ptr(W2), _ptr(out_sorted),
                           _ptr(workspace), _stream(stream)))


def moe_combine(cfg, out_sorted, topk_gate, inv_perm, y, stream=None):
    _check(_moe_combine(ctypes.byref(cfg), _ptr(out_sorted), _ptr(topk_gate), _ptr(inv_perm),
                        _ptr(y), _stream(stream)))


def moe_aux_losses(cfg, partials, importance, load, losses, workspace, stream=None):
    _check(_moe_aux_losses(ctypes.byref(cfg), _ptr(partials), _ptr(importance), _ptr(load),
                           _ptr(losses), _ptr(workspace), _stream(stream)))


def moe_layer_forward(cfg, x, W_g, W_noise, gate_bias, eps, W1, W2, y, topk_idx, topk_gate,
                      importance, load, losses, workspace, stream=None):
    nbytes = workspace.numel() * workspace.element_size()
    _check(_moe_layer_forward(ctypes.byref(cfg), _ptr(x), _ptr(W_g), _ptr(W_noise),
                              _ptr(gate_bias), _ptr(eps), _ptr(W1), _ptr(W2), _ptr(y),
                              _ptr(topk_idx), _ptr(topk_gate), _ptr(importance), _ptr(load),
                              _ptr(losses), _ptr(workspace), nbytes, _stream(stream)))


def moe_layer_forward_profiled(cfg, x, W_g, W_noise, gate_bias, eps, W1, W2, y, topk_idx, topk_gate,
                               importance, load, losses, workspace, stage_events, stream=None):
    """stage_events: None or a sequence of 10 hipEvent_t handles (ints, 0/None to skip)."""
    nbytes = workspace.numel() * workspace.element_size()
    ev = None
    if stage_events is not None:
        ev = (_vp * 10)(*[(e or None) for e in stage_events])
    _check(_moe_layer_forward_profiled(ctypes.byref(cfg), _ptr(x), _ptr(W_g), _ptr(W_noise),
                                       _ptr(gate_bias), _ptr(eps), _ptr(W1), _ptr(W2), _ptr(y),
                                       _ptr(topk_idx), _ptr(topk_gate), _ptr(importance), _ptr(load),
                                       _ptr(losses), _ptr(workspace), nbytes, ev, _stream(stream)))


def _nbytes(t):
    return t.numel() * t.element_size()


def moe_gate_hier(cfg, x, Wg_p, Wn_p, eps_p, Wg_s, Wn_s, eps_s, topk_idx, topk_gate, workspace,
                  stream=None):
    _check(_moe_gate_hier(ctypes.byref(cfg), _ptr(x), _ptr(Wg_p), _ptr(Wn_p), _ptr(eps_p), _ptr(Wg_s),
                          _ptr(Wn_s), _ptr(eps_s), _ptr(topk_idx), _ptr(topk_gate), _ptr(workspace),
                          _nbytes(workspace), _stream(stream)))


def moe_aux_losses_hier(cfg, topk_gate, perm, offsets, workspace, importance, load, losses, stream=None):
    _check(_moe_aux_losses_hier(ctypes.byref(cfg), _ptr(topk_gate), _ptr(perm), _ptr(offsets),
                                _ptr(workspace), _nbytes(workspace), _ptr(importance), _ptr(load),
                                _ptr(losses), _stream(stream)))


def moe_layer_forward_hier(cfg, x, Wg_p, Wn_p, eps_p, Wg_s, Wn_s, eps_s, W1, W2, y, topk_idx, topk_gate,
                           importance, load, losses, workspace, stream=None):
    _check(_moe_layer_forward_hier(ctypes.byref(cfg), _ptr(x), _ptr(Wg_p), _ptr(Wn_p), _ptr(eps_p),
                                   _ptr(Wg_s), _ptr(Wn_s), _ptr(eps_s), _ptr(W1), _ptr(W2), _ptr(y),
                                   _ptr(topk_idx), _ptr(topk_gate), _ptr(importance), _ptr(load),
                                   _ptr(losses), _ptr(workspace), _nbytes(workspace), _stream(stream)))


def moe_layer_forward_hier_profiled(cfg, x, Wg_p, Wn_p, eps_p, Wg_s, Wn_s, eps_s, W1, W2, y, topk_idx, topk_gate,
                                    importance, load, losses, workspace, stage_events, stream=None):
    """stage_events: None or a sequence of 10 hipEvent_t handles (ints, 0/None to skip)."""
    ev = None
    if stage_events is not None:
        ev = (_vp * 10)(*[(e or None) for e in stage_events])
    _check(_moe_layer_forward_hier_profiled(ctypes.byref(cfg), _ptr(x), _ptr(Wg_p), _ptr(Wn_p), _ptr(eps_p),
                                            _ptr(Wg_s), _ptr(Wn_s), _ptr(eps_s), _ptr(W1), _ptr(W2), _ptr(y),
                                            _ptr(topk_idx), _ptr(topk_gate), _ptr(importance), _ptr(load),
                                            _ptr(losses), _ptr(workspace), _nbytes(workspace), ev,
                                            _stream(stream)))


def moe_backward_workspace_bytes(cfg):
    return _moe_backward_workspace_bytes(ctypes.byref(cfg))


def moe_layer_backward(cfg, x, W_g, W_noise, eps, W1, W2, dy, topk_idx, topk_gate, fwd_workspace, dx,
                       dW_g, dW_noise, dW1, dW2, workspace, stream=None):
    _check(_moe_layer_backward(ctypes.byref(cfg), _ptr(x), _ptr(W_g), _ptr(W_noise), _ptr(eps), _ptr(W1),
                               _ptr(W2), _ptr(dy), _ptr(topk_idx), _ptr(topk_gate), _ptr(fwd_workspace),
                               _ptr(dx), _ptr(dW_g), _ptr(dW_noise), _ptr(dW1), _ptr(dW2), _ptr(workspace),
                               _nbytes(workspace), _stream(stream)))


def moe_balanced_rows_per_expert(cfg):
    return _moe_balanced_rows_per_expert(ctypes.byref(cfg))


def moe_balanced_workspace_bytes(cfg):
    return _moe_balanced_workspace_bytes(ctypes.byref(cfg))


def moe_gate_balanced(cfg, x, W_g, gate_bias, thresholds, gsigma, tokens, kept, denom, loss_batchwise,
                      workspace, stream=None):
    _check(_moe_gate_balanced(ctypes.byref(cfg), _ptr(x), _ptr(W_g), _ptr(gate_bias), _ptr(thresholds),
                              _ptr(gsigma), _ptr(tokens), _ptr(kept), _ptr(denom), _ptr(loss_batchwise),
                              _ptr(workspace), _nbytes(workspace), _stream(stream)))


def moe_layer_forward_balanced(cfg, x, W_g, gate_bias, thresholds, W1, W2, y, gsigma, tokens, kept, denom,
                               loss_batchwise, workspace, stream=None):
    _check(_moe_layer_forward_balanced(ctypes.byref(cfg), _ptr(x), _ptr(W_g), _ptr(gate_bias),
                                       _ptr(thresholds), _ptr(W1), _ptr(W2), _ptr(y), _ptr(gsigma),
                                       _ptr(tokens), _ptr(kept), _ptr(denom), _ptr(loss_batchwise),
                                       _ptr(workspace), _nbytes(workspace), _stream(stream)))


def moe_layer_forward_balanced_profiled(cfg, x, W_g, gate_bias, thresholds, W1, W2, y, gsigma, tokens, kept,
                                        denom, loss_batchwise, workspace, stage_events, stream=None):
    """stage_events: None or a sequence of 5 hipEvent_t handles (ints, 0/None to skip)."""
    ev = None
    if stage_events is not None:
        ev = (_vp * 5)(*[(e or None) for e in stage_events])
    _check(_moe_layer_forward_balanced_profiled(ctypes.byref(cfg), _ptr(x), _ptr(W_g), _ptr(gate_bias),
                                                _ptr(thresholds), _ptr(W1), _ptr(W2), _ptr(y), _ptr(gsigma),
                                                _ptr(tokens), _ptr(kept), _ptr(denom), _ptr(loss_batchwise),
                                                _ptr(workspace), _nbytes(workspace), ev, _stream(stream)))


def moe_threshold_workspace_bytes(cfg, row_capacity):
    return _moe_threshold_workspace_bytes(ctypes.byref(cfg), row_capacity)


def moe_layer_forward_threshold(cfg, x, W_g, gate_bias, thresholds, W1, W2, row_capacity, y, gsigma, counts,
                                tokens, kept, denom, rows_total, workspace, stream=None):
    _check(_moe_layer_forward_threshold(ctypes.byref(cfg), _ptr(x), _ptr(W_g), _ptr(gate_bias),
                                        _ptr(thresholds), _ptr(W1), _ptr(W2), row_capacity, _ptr(y),
                                        _ptr(gsigma), _ptr(counts), _ptr(tokens), _ptr(kept), _ptr(denom),
                                        _ptr(rows_total), _ptr(workspace), _nbytes(workspace), _stream(stream)))


def moe_adam_workspace_bytes(cfg):
    return _moe_adam_workspace_bytes(ctypes.byref(cfg))


def moe_expert_adam_step(cfg, lr, beta2, eps, step, dW1, dW2, W1_master, W2_master, W1_copy, W2_copy, v_row1,
                         v_col1, v_row2, v_col2, workspace, stream=None, backward_workspace=None):
    hp = MoeAdamParams(lr, beta2, eps, step)
    _check(_moe_expert_adam_step(ctypes.byref(cfg), ctypes.byref(hp), _ptr(dW1), _ptr(dW2), _ptr(W1_master),
                                 _ptr(W2_master), _ptr(W1_copy), _ptr(W2_copy), _ptr(v_row1), _ptr(v_col1),
                                 _ptr(v_row2), _ptr(v_col2), _ptr(backward_workspace), _ptr(workspace),
                                 _nbytes(workspace), _stream(stream)))


def moe_backward_hier_workspace_bytes(cfg):
    return _moe_backward_hier_workspace_bytes(ctypes.byref(cfg))


def moe_layer_backward_hier(cfg, x, Wg_p, Wn_p, eps_p, Wg_s, Wn_s, eps_s, W1, W2, dy, topk_idx, topk_gate,
                            fwd_workspace, dx, dWg_p, dWn_p, dWg_s, dWn_s, dW1, dW2, workspace, stream=None):
    _check(_moe_layer_backward_hier(ctypes.byref(cfg), _ptr(x), _ptr(Wg_p), _ptr(Wn_p), _ptr(eps_p), _ptr(Wg_s),
                                    _ptr(Wn_s), _ptr(eps_s), _ptr(W1), _ptr(W2), _ptr(dy), _ptr(topk_idx),
                                    _ptr(topk_gate), _ptr(fwd_workspace), _ptr(dx), _ptr(dWg_p), _ptr(dWn_p),
                                    _ptr(dWg_s), _ptr(dWn_s), _ptr(dW1), _ptr(dW2), _ptr(workspace),
                                    _nbytes(workspace), _stream(stream)))


def moe_combine_epilogue(cfg, out_sorted, topk_gate, inv_perm, x, keep, drop_prob, y, stream=None):
    _check(_moe_combine_epilogue(ctypes.byref(cfg), _ptr(out_sorted), _ptr(topk_gate), _ptr(inv_perm), _ptr(x),
                                 _ptr(keep), drop_prob, _ptr(y), _stream(stream)))


def moe_backward_balanced_workspace_bytes(cfg):
    return _moe_backward_balanced_workspace_bytes(ctypes.byref(cfg))


def moe_layer_backward_balanced(cfg, x, W_g, thresholds, W1, W2, dy, gsigma, tokens, kept, denom, fwd_workspace,
                                w_batchwise, dx, dW_g, dW1, dW2, workspace, stream=None):
    _check(_moe_layer_backward_balanced(ctypes.byref(cfg), _ptr(x), _ptr(W_g), _ptr(thresholds), _ptr(W1),
                                        _ptr(W2), _ptr(dy), _ptr(gsigma), _ptr(tokens), _ptr(kept), _ptr(denom),
                                        _ptr(fwd_workspace), w_batchwise, _ptr(dx), _ptr(dW_g), _ptr(dW1),
                                        _ptr(dW2), _ptr(workspace), _nbytes(workspace), _stream(stream)))


def moe_batchwise_loss_grad(cfg, gsigma, thresholds, dthresholds, stream=None):
    _check(_moe_batchwise_loss_grad(ctypes.byref(cfg), _ptr(gsigma), _ptr(thresholds), _ptr(dthresholds),
                                    _stream(stream)))
