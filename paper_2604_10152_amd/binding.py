"""ctypes binding of libspecmoe.so: same names as the C ABI, argument marshalling only.

Tensors are torch tensors that already live on the GPU (PyTorch owns device memory and
streams); every computation happens in the library's HIP kernels.  There is no CPU or
PyTorch fallback: if the library is missing, or a tensor is not a contiguous GPU tensor of
the expected dtype, the call raises.
"""
from __future__ import annotations

import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB = None

EXPORTED_SYMBOLS = (
    "moe_route_topk", "moe_permute", "moe_grouped_swiglu_workspace_bytes", "moe_grouped_swiglu",
    "moe_grouped_swiglu_static", "moe_pack_weights", "moe_packed_h_bytes",
    "moe_expert_up_swiglu_gather_packed", "moe_expert_down_packed",
    "moe_permute_rows_packed", "moe_expert_up_swiglu_packed",
    "moe_expert_up_swiglu", "moe_expert_up_swiglu_gather", "moe_expert_down", "moe_combine", "spec_accept", "moe_hot_experts", "moe_rmsnorm", "specmoe_status_string", "specmoe_abi_version",
    "moe_affinity_table_workspace_bytes", "moe_affinity_table", "moe_nearest_draft_expert",
    "moe_route_topk_draft", "spec_accept_sample", "spec_greedy_tokens", "moe_active_expert_bytes",
)

F32, BF16 = 0, 1


class SpecMoEError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: status {status} ({status_string(status)})")


def lib_path() -> str:
    return os.path.join(_HERE, "libspecmoe.so")


def load_library(build_if_missing: bool = True):
    """dlopen the in-tree library; build it with hipcc first if it is not there."""
    global _LIB
    if _LIB is not None:
        return _LIB
    path = lib_path()
    if not os.path.exists(path):
        if not build_if_missing:
            raise FileNotFoundError(path)
        from . import build as _build
        _build.build()
    lib = ctypes.CDLL(path)
    vp, ip, fp = ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p
    i, sz = ctypes.c_int, ctypes.c_size_t
    lib.moe_route_topk.argtypes = [vp, vp, fp, i, i, i, i, i, i, ip, fp, vp]
    lib.moe_permute.argtypes = [vp, ip, i, i, i, i, i, vp, ip, ip, ip, vp]
    lib.moe_grouped_swiglu_workspace_bytes.argtypes = [i, i, i, i, i]
    lib.moe_grouped_swiglu_workspace_bytes.restype = sz
    lib.moe_grouped_swiglu.argtypes = [vp, ip, vp, vp, vp, i, i, i, i, i, vp, vp, sz, vp]
    lib.moe_grouped_swiglu_static.argtypes = [vp, ip, vp, vp, vp, i, i, i, i, i, vp, vp]
    lib.moe_expert_up_swiglu.argtypes = [vp, ip, vp, vp, i, i, i, i, i, vp, vp]
    lib.moe_pack_weights.argtypes = [vp, i, i, i, i, vp, vp]
    lib.moe_packed_h_bytes.argtypes = [i, i, i]
    lib.moe_packed_h_bytes.restype = sz
    lib.moe_expert_up_swiglu_gather_packed.argtypes = [vp, ip, i, i, ip, vp, vp, i, i, i, i, i, vp, sz,
                                                       vp, sz, vp]
    lib.moe_expert_down_packed.argtypes = [vp, ip, vp, i, i, i, i, i, vp, vp]
    lib.moe_permute_rows_packed.argtypes = [vp, ip, i, i, ip, i, i, i, i, vp, sz, vp]
    lib.moe_expert_up_swiglu_packed.argtypes = [vp, sz, ip, vp, vp, i, i, i, i, i, vp, sz, i, vp]
    lib.moe_expert_up_swiglu_gather.argtypes = [vp, ip, i, i, ip, vp, vp, i, i, i, i, i, vp, vp]
    lib.moe_expert_down.argtypes = [vp, ip, vp, i, i, i, i, i, vp, vp]
    lib.moe_combine.argtypes = [vp, ip, fp, vp, i, i, i, i, vp, vp]
    lib.spec_accept.argtypes = [ip, ip, i, i, ip, ip, vp]
    lib.moe_hot_experts.argtypes = [ip, i, i, ip, ip, vp]
    lib.moe_rmsnorm.argtypes = [vp, vp, i, i, ctypes.c_float, i, vp, vp]
    lib.moe_affinity_table_workspace_bytes.argtypes = [i]
    lib.moe_affinity_table_workspace_bytes.restype = ctypes.c_size_t
    lib.moe_affinity_table.argtypes = [vp, vp, vp, i, i, i, i, fp, vp, ctypes.c_size_t, vp]
    lib.moe_nearest_draft_expert.argtypes = [fp, i, ip, i, ip, vp]
    lib.moe_route_topk_draft.argtypes = [vp, vp, fp, i, i, i, i, i, i, ip, ip, fp, vp]
    lib.spec_accept_sample.argtypes = [ip, fp, fp, fp, fp, i, i, i, ip, ip, vp]
    lib.spec_greedy_tokens.argtypes = [vp, i, i, i, ip, vp]
    lib.moe_active_expert_bytes.argtypes = [ip, i, ctypes.c_longlong, vp, vp]
    lib.specmoe_status_string.argtypes = [i]
    lib.specmoe_status_string.restype = ctypes.c_char_p
    lib.specmoe_abi_version.restype = i
    for name in ("moe_route_topk", "moe_permute", "moe_grouped_swiglu", "moe_combine",
                 "moe_grouped_swiglu_static", "moe_pack_weights",
                 "moe_expert_up_swiglu_gather_packed", "moe_expert_down_packed",
                 "moe_permute_rows_packed", "moe_expert_up_swiglu_packed",
                 "moe_expert_up_swiglu", "moe_expert_up_swiglu_gather", "moe_expert_down",
                 "moe_hot_experts", "moe_affinity_table", "moe_nearest_draft_expert",
                 "moe_route_topk_draft", "spec_accept_sample", "spec_greedy_tokens",
                 "moe_active_expert_bytes",
                 "spec_accept", "moe_rmsnorm"):
        getattr(lib, name).restype = i
    _LIB = lib
    return lib


def status_string(status: int) -> str:
    return load_library().specmoe_status_string(int(status)).decode()


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return F32
    if t.dtype == torch.bfloat16:
        return BF16
    raise TypeError(f"unsupported dtype {t.dtype}: use float32 or bfloat16")


def _ptr(t, dtype=None, name="tensor"):
    """Device pointer of a contiguous GPU tensor (None -> NULL)."""
    if t is None:
        return None
    if not isinstance(t, torch.Tensor) or not t.is_cuda:
        raise TypeError(f"{name} must be a GPU tensor (no CPU fallback exists)")
    if not t.is_contiguous():
        raise ValueError(f"{name} must be contiguous")
    if dtype is not None and t.dtype != dtype:
        raise TypeError(f"{name} must have dtype {dtype}, got {t.dtype}")
    return ctypes.c_void_p(t.data_ptr())


def _stream(stream):
    if stream is None:
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream)


def _check(status, where):
    if status != 0:
        raise SpecMoEError(status, where)


def moe_route_topk(x, w_router, router_bias, k, renorm, topk_idx, topk_w, stream=None):
    T, d = x.shape
    E = w_router.shape[0]
    dt = _dtype_code(x)
    _check(load_library().moe_route_topk(
        _ptr(x, name="x"), _ptr(w_router, x.dtype, "w_router"),
        _ptr(router_bias, torch.float32, "router_bias"), T, d, E, int(k), int(bool(renorm)), dt,
        _ptr(topk_idx, torch.int32, "topk_idx"), _ptr(topk_w, torch.float32, "topk_w"),
        _stream(stream)), "moe_route_topk")


def moe_permute(x, topk_idx, E, x_perm, expert_offsets, row_src, row_of, stream=None):
    T, d = x.shape
    k = topk_idx.shape[1]
    _check(load_library().moe_permute(
        _ptr(x, name="x"), _ptr(topk_idx, torch.int32, "topk_idx"), T, d, int(E), k,
        _dtype_code(x), _ptr(x_perm, x.dtype, "x_perm"),
        _ptr(expert_offsets, torch.int32, "expert_offsets"), _ptr(row_src, torch.int32, "row_src"),
        _ptr(row_of, torch.int32, "row_of"), _stream(stream)), "moe_permute")


def moe_grouped_swiglu_workspace_bytes(n_rows, d_model, d_ff, E, dtype) -> int:
    code = F32 if dtype == torch.float32 else BF16
    return int(load_library().moe_grouped_swiglu_workspace_bytes(n_rows, d_model, d_ff, E, code))


def moe_grouped_swiglu(x_perm, expert_offsets, w_gate, w_up, w_down, y_perm, workspace,
                       stream=None):
    n_rows, d = x_perm.shape
    E, f, _ = w_gate.shape
    _check(load_library().moe_grouped_swiglu(
        _ptr(x_perm, name="x_perm"), _ptr(expert_offsets, torch.int32, "expert_offsets"),
        _ptr(w_gate, x_perm.dtype, "w_gate"), _ptr(w_up, x_perm.dtype, "w_up"),
        _ptr(w_down, x_perm.dtype, "w_down"), n_rows, d, f, E, _dtype_code(x_perm),
        _ptr(y_perm, x_perm.dtype, "y_perm"), _ptr(workspace, torch.uint8, "workspace"),
        workspace.numel(), _stream(stream)), "moe_grouped_swiglu")


def moe_grouped_swiglu_static(x_perm, expert_offsets, w_gate, w_up, w_down, y_perm, stream=None):
    n_rows, d = x_perm.shape
    E, f, _ = w_gate.shape
    _check(load_library().moe_grouped_swiglu_static(
        _ptr(x_perm, name="x_perm"), _ptr(expert_offsets, torch.int32, "expert_offsets"),
        _ptr(w_gate, x_perm.dtype, "w_gate"), _ptr(w_up, x_perm.dtype, "w_up"),
        _ptr(w_down, x_perm.dtype, "w_down"), n_rows, d, f, E, _dtype_code(x_perm),
        _ptr(y_perm, x_perm.dtype, "y_perm"), _stream(stream)), "moe_grouped_swiglu_static")


def moe_expert_up_swiglu(x_perm, expert_offsets, w_gate, w_up, h, stream=None):
    n_rows, d = x_perm.shape
    E, f, _ = w_gate.shape
    _check(load_library().moe_expert_up_swiglu(
        _ptr(x_perm, name="x_perm"), _ptr(expert_offsets, torch.int32, "expert_offsets"),
        _ptr(w_gate, x_perm.dtype, "w_gate"), _ptr(w_up, x_perm.dtype, "w_up"), n_rows, d, f, E,
        _dtype_code(x_perm), _ptr(h, x_perm.dtype, "h"), _stream(stream)), "moe_expert_up_swiglu")


def moe_expert_up_swiglu_gather(x, row_src, k, expert_offsets, w_gate, w_up, h, stream=None):
    T, d = x.shape
    n_rows = row_src.numel()
    E, f, _ = w_gate.shape
    _check(load_library().moe_expert_up_swiglu_gather(
        _ptr(x, name="x"), _ptr(row_src, torch.int32, "row_src"), T, int(k),
        _ptr(expert_offsets, torch.int32, "expert_offsets"), _ptr(w_gate, x.dtype, "w_gate"),
        _ptr(w_up, x.dtype, "w_up"), n_rows, d, f, E, _dtype_code(x), _ptr(h, x.dtype, "h"),
        _stream(stream)), "moe_expert_up_swiglu_gather")


def moe_pack_weights(w, w_packed, stream=None):
    E, rows, cols = w.shape
    _check(load_library().moe_pack_weights(
        _ptr(w, torch.bfloat16, "w"), E, rows, cols, BF16, _ptr(w_packed, torch.bfloat16, "w_packed"),
        _stream(stream)), "moe_pack_weights")


def moe_packed_h_bytes(n_rows, d_ff, E) -> int:
    return int(load_library().moe_packed_h_bytes(n_rows, d_ff, E))


def moe_expert_up_swiglu_gather_packed(x, row_src, k, expert_offsets, w_gate_packed, w_up_packed,
                                       n_rows, h_packed, x_packed_workspace=None, stream=None):
    T, d = x.shape
    E, f, _ = w_gate_packed.shape
    _check(load_library().moe_expert_up_swiglu_gather_packed(
        _ptr(x, torch.bfloat16, "x"), _ptr(row_src, torch.int32, "row_src"), T, k,
        _ptr(expert_offsets, torch.int32, "expert_offsets"),
        _ptr(w_gate_packed, torch.bfloat16, "w_gate_packed"),
        _ptr(w_up_packed, torch.bfloat16, "w_up_packed"), n_rows, d, f, E, BF16,
        _ptr(h_packed, name="h_packed"), h_packed.numel() * h_packed.element_size(),
        _ptr(x_packed_workspace, name="x_packed_workspace"),
        0 if x_packed_workspace is None else
        x_packed_workspace.numel() * x_packed_workspace.element_size(),
        _stream(stream)), "moe_expert_up_swiglu_gather_packed")


def moe_permute_rows_packed(x, row_src, k, expert_offsets, n_rows, x_packed, stream=None):
    T, d = x.shape
    E = expert_offsets.numel() - 1
    _check(load_library().moe_permute_rows_packed(
        _ptr(x, torch.bfloat16, "x"), _ptr(row_src, torch.int32, "row_src"), T, k,
        _ptr(expert_offsets, torch.int32, "expert_offsets"), n_rows, d, E, BF16,
        _ptr(x_packed, name="x_packed"), x_packed.numel() * x_packed.element_size(),
        _stream(stream)), "moe_permute_rows_packed")


def moe_expert_up_swiglu_packed(x_packed, expert_offsets, w_gate_packed, w_up_packed, n_rows, h,
                                h_row_major=False, stream=None):
    E, f, d = w_gate_packed.shape
    _check(load_library().moe_expert_up_swiglu_packed(
        _ptr(x_packed, name="x_packed"), x_packed.numel() * x_packed.element_size(),
        _ptr(expert_offsets, torch.int32, "expert_offsets"),
        _ptr(w_gate_packed, torch.bfloat16, "w_gate_packed"),
        _ptr(w_up_packed, torch.bfloat16, "w_up_packed"), n_rows, d, f, E, BF16,
        _ptr(h, name="h"), h.numel() * h.element_size(), 1 if h_row_major else 0,
        _stream(stream)), "moe_expert_up_swiglu_packed")


def moe_expert_down_packed(h_packed, expert_offsets, w_down_packed, y_perm, stream=None):
    n_rows, d = y_perm.shape
    E, _, f = w_down_packed.shape
    _check(load_library().moe_expert_down_packed(
        _ptr(h_packed, name="h_packed"), _ptr(expert_offsets, torch.int32, "expert_offsets"),
        _ptr(w_down_packed, torch.bfloat16, "w_down_packed"), n_rows, d, f, E, BF16,
        _ptr(y_perm, torch.bfloat16, "y_perm"), _stream(stream)), "moe_expert_down_packed")


def moe_expert_down(h, expert_offsets, w_down, y_perm, stream=None):
    n_rows, f = h.shape
    E, d, _ = w_down.shape
    _check(load_library().moe_expert_down(
        _ptr(h, name="h"), _ptr(expert_offsets, torch.int32, "expert_offsets"),
        _ptr(w_down, h.dtype, "w_down"), n_rows, d, f, E, _dtype_code(h),
        _ptr(y_perm, h.dtype, "y_perm"), _stream(stream)), "moe_expert_down")


def moe_combine(y_perm, row_of, topk_w, residual, out, stream=None):
    T, k = topk_w.shape
    d = y_perm.shape[1]
    _check(load_library().moe_combine(
        _ptr(y_perm, name="y_perm"), _ptr(row_of, torch.int32, "row_of"),
        _ptr(topk_w, torch.float32, "topk_w"), _ptr(residual, y_perm.dtype, "residual"), T, d, k,
        _dtype_code(y_perm), _ptr(out, y_perm.dtype, "out"), _stream(stream)), "moe_combine")


def spec_accept(draft_ids, target_ids, accept_len, out_tokens, stream=None):
    B, gamma = draft_ids.shape
    if tuple(target_ids.shape) != (B, gamma + 1):
        raise ValueError("target_ids must be [B, gamma+1]")
    _check(load_library().spec_accept(
        _ptr(draft_ids, torch.int32, "draft_ids"), _ptr(target_ids, torch.int32, "target_ids"), B,
        gamma, _ptr(accept_len, torch.int32, "accept_len"),
        _ptr(out_tokens, torch.int32, "out_tokens"), _stream(stream)), "spec_accept")


def moe_hot_experts(expert_offsets, hot_ids, hot_counts=None, stream=None):
    E = expert_offsets.numel() - 1
    _check(load_library().moe_hot_experts(
        _ptr(expert_offsets, torch.int32, "expert_offsets"), E, hot_ids.numel(),
        _ptr(hot_ids, torch.int32, "hot_ids"), _ptr(hot_counts, torch.int32, "hot_counts"),
        _stream(stream)), "moe_hot_experts")


def moe_affinity_table_workspace_bytes(E):
    return int(load_library().moe_affinity_table_workspace_bytes(int(E)))


def moe_affinity_table(w_gate, w_up, w_down, affinity, workspace, stream=None):
    E, f, d = w_gate.shape
    _check(load_library().moe_affinity_table(
        _ptr(w_gate, None, "w_gate"), _ptr(w_up, w_gate.dtype, "w_up"),
        _ptr(w_down, w_gate.dtype, "w_down"), E, d, f, _dtype_code(w_gate),
        _ptr(affinity, torch.float32, "affinity"), _ptr(workspace, None, "workspace"),
        workspace.numel() * workspace.element_size(), _stream(stream)), "moe_affinity_table")


def moe_nearest_draft_expert(affinity, draft_ids, remap, stream=None):
    E = affinity.shape[0]
    _check(load_library().moe_nearest_draft_expert(
        _ptr(affinity, torch.float32, "affinity"), E, _ptr(draft_ids, torch.int32, "draft_ids"),
        draft_ids.numel(), _ptr(remap, torch.int32, "remap"), _stream(stream)),
        "moe_nearest_draft_expert")


def moe_route_topk_draft(x, w_router, bias, k, renorm, remap, topk_idx, topk_w, stream=None):
    T, d = x.shape
    E = w_router.shape[0]
    _check(load_library().moe_route_topk_draft(
        _ptr(x, None, "x"), _ptr(w_router, x.dtype, "w_router"),
        _ptr(bias, torch.float32, "bias"), T, d, E, k, int(bool(renorm)), _dtype_code(x),
        _ptr(remap, torch.int32, "remap"), _ptr(topk_idx, torch.int32, "topk_idx"),
        _ptr(topk_w, torch.float32, "topk_w"), _stream(stream)), "moe_route_topk_draft")


def spec_accept_sample(draft_ids, p_draft, p_target, u_accept, u_sample, accept_len, out_tokens,
                       stream=None):
    B, gp1, V = p_target.shape
    gamma = gp1 - 1
    _check(load_library().spec_accept_sample(
        _ptr(draft_ids, torch.int32, "draft_ids"), _ptr(p_draft, torch.float32, "p_draft"),
        _ptr(p_target, torch.float32, "p_target"), _ptr(u_accept, torch.float32, "u_accept"),
        _ptr(u_sample, torch.float32, "u_sample"), B, gamma, V,
        _ptr(accept_len, torch.int32, "accept_len"), _ptr(out_tokens, torch.int32, "out_tokens"),
        _stream(stream)), "spec_accept_sample")


def spec_greedy_tokens(logits, tokens, stream=None):
    R, V = logits.shape
    _check(load_library().spec_greedy_tokens(
        _ptr(logits, None, "logits"), R, V, _dtype_code(logits),
        _ptr(tokens, torch.int32, "tokens"), _stream(stream)), "spec_greedy_tokens")


def moe_active_expert_bytes(expert_offsets, bytes_per_expert, out_bytes, stream=None):
    E = expert_offsets.numel() - 1
    _check(load_library().moe_active_expert_bytes(
        _ptr(expert_offsets, torch.int32, "expert_offsets"), E, int(bytes_per_expert),
        _ptr(out_bytes, torch.int64, "out_bytes"), _stream(stream)), "moe_active_expert_bytes")


def moe_rmsnorm(x, gain, eps, out, stream=None):
    T, d = x.shape
    _check(load_library().moe_rmsnorm(
        _ptr(x, name="x"), _ptr(gain, x.dtype, "gain"), T, d, float(eps), _dtype_code(x),
        _ptr(out, x.dtype, "out"), _stream(stream)), "moe_rmsnorm")
