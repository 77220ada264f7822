"""Thin Python binding over the C-ABI library (include/tslt.h): argument marshalling only.

Every function takes torch tensors that live on the GPU, allocates the outputs and the workspace
with torch (device memory and streams are torch's job here, nothing else), passes raw device
pointers and the current HIP stream to the library and returns the output tensors.  There is no
fallback: if the library is missing, or a tensor is not on a GPU, the call raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Sequence

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libtslt.so")

F32, BF16, F16 = 0, 1, 2
OP_TRUNCATE, OP_SAMPLE, OP_VERIFY, OP_VERIFY_TREE, OP_VERIFY_TREE_PATH = 0, 1, 2, 3, 4
ROW_NONFINITE, ROW_EMPTY, ROW_TOKEN_NOT_IN_SET, ROW_BAD_SET, ROW_EXACT_PATH = 1, 2, 4, 8, 256
MAX_K_CAP = 1024
PAYLOAD = {"f32": 0, "bf16": 1, "f16": 2}       # tslt_dtype codes of the formats a payload can travel in

EXPORTS = ("tslt_version", "tslt_last_error", "tslt_workspace_bytes", "tslt_truncate", "tslt_truncate_sample", "tslt_sample",
           "tslt_pack_bound_words", "tslt_pack", "tslt_unpack",
           "tslt_verify", "tslt_verify_accept", "tslt_verify_resample", "tslt_verify_staged", "tslt_verify_accept_staged",
           "tslt_verify_static", "tslt_truncation_stats", "tslt_multicandidate_stats", "tslt_calibrate_read", "tslt_verify_tree")

_lib = None


class TsltError(RuntimeError):
    pass


def load(path: Optional[str] = None):
    """Open the library; raises if it has not been built (python -m paper_2512_16273_amd.build)."""
    global _lib
    if _lib is not None and path is None:
        return _lib
    path = path or os.environ.get("TSLT_LIBRARY") or LIB_PATH      # TSLT_LIBRARY: another build of the same ABI
    if not os.path.exists(path):
        raise TsltError(f"{path} not found: build it with `python -m paper_2512_16273_amd.build` "
                        "(there is no CPU fallback)")
    lib = ctypes.CDLL(path)
    c = ctypes
    vp, i32, i64, f32, sz = c.c_void_p, c.c_int32, c.c_int64, c.c_float, c.c_size_t
    lib.tslt_version.restype = c.c_int
    lib.tslt_version.argtypes = []
    lib.tslt_last_error.restype = c.c_char_p
    lib.tslt_last_error.argtypes = []
    lib.tslt_workspace_bytes.restype = sz
    lib.tslt_workspace_bytes.argtypes = [c.c_int, i64, i64, i64, i32]
    lib.tslt_truncate.restype = c.c_int
    lib.tslt_truncate.argtypes = [vp, c.c_int, i64, i64, i64, f32, i32, f32, i32, c.c_int, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.tslt_pack_bound_words.restype = i64
    lib.tslt_pack_bound_words.argtypes = [i64, i32, i64]
    lib.tslt_pack.restype = c.c_int
    lib.tslt_pack.argtypes = [vp, vp, vp, i64, i32, i64, c.c_int, vp, i64, vp, vp]
    lib.tslt_unpack.restype = c.c_int
    lib.tslt_unpack.argtypes = [vp, vp, i64, i32, i64, c.c_int, vp, vp, vp, vp]
    lib.tslt_truncate_sample.restype = c.c_int
    lib.tslt_truncate_sample.argtypes = [vp, c.c_int, i64, i64, i64, f32, i32, f32, i32, c.c_int, vp, vp, vp, vp, vp, vp,
                                         vp, i32, i32, vp, vp, vp, sz, vp]
    lib.tslt_sample.restype = c.c_int
    lib.tslt_sample.argtypes = [vp, vp, vp, i64, i32, vp, i32, i32, vp, vp, vp]
    for fn in (lib.tslt_verify, lib.tslt_verify_accept, lib.tslt_verify_resample):
        fn.restype = c.c_int
        fn.argtypes = [vp, c.c_int, i64, i32, i64, i64, f32, vp, vp, vp, i32, vp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    for fn in (lib.tslt_verify_staged, lib.tslt_verify_accept_staged):
        fn.restype = c.c_int
        fn.argtypes = [vp, c.c_int, i64, i32, i64, i64, f32, vp, vp, vp, i32, vp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp, i32]
    lib.tslt_verify_static.restype = c.c_int
    lib.tslt_verify_static.argtypes = [vp, c.c_int, i64, i32, i64, i64, f32, vp, vp, vp, i32, vp, vp, vp, vp, vp, vp, vp, vp, vp]
    lib.tslt_calibrate_read.restype = c.c_int
    lib.tslt_calibrate_read.argtypes = [vp, sz, i32, vp, vp]
    lib.tslt_truncation_stats.restype = c.c_int
    lib.tslt_truncation_stats.argtypes = [vp, c.c_int, i64, i64, i64, f32, vp, vp, vp, i32, c.POINTER(i32), i32, vp, vp, vp, vp]
    lib.tslt_multicandidate_stats.restype = c.c_int
    lib.tslt_multicandidate_stats.argtypes = [vp, c.c_int, i64, i64, i64, f32, vp, vp, vp, i32, i32, vp, vp, vp, vp]
    lib.tslt_verify_tree.restype = c.c_int
    lib.tslt_verify_tree.argtypes = [vp, c.c_int, i64, i64, i64, f32, i32, c.POINTER(i32), vp, vp, vp, i32, vp, vp,
                                     vp, i32, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    _lib = lib
    return lib


def _check(code: int):
    if code != 0:
        raise TsltError(f"tslt error {code}: {load().tslt_last_error().decode()}")


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return F32
    if t.dtype == torch.bfloat16:
        return BF16
    if t.dtype == torch.float16:
        return F16
    raise TsltError(f"unsupported logits dtype {t.dtype}")


def _dev(t: torch.Tensor, dtype=None, name="tensor", contiguous=True) -> torch.Tensor:
    if not t.is_cuda:
        raise TsltError(f"{name} must live on the GPU (there is no CPU path)")
    if dtype is not None and t.dtype != dtype:
        raise TsltError(f"{name} must be {dtype}, got {t.dtype}")
    if contiguous and not t.is_contiguous():
        raise TsltError(f"{name} must be contiguous")
    return t


def _ptr(t: Optional[torch.Tensor]):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream() -> ctypes.c_void_p:
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _rows_2d(logits: torch.Tensor):
    """[..., V] view as rows with a common stride (the last dimension must be dense)."""
    if logits.stride(-1) != 1:
        raise TsltError("logits must be dense along the vocabulary")
    V = logits.shape[-1]
    if logits.dim() == 1:
        return 1, V, V
    flat = logits.reshape(-1, V) if logits.is_contiguous() else logits
    if flat.dim() != 2:
        raise TsltError("non-contiguous logits must be 2-D [rows, V]")
    return flat.shape[0], V, flat.stride(0)


def workspace_bytes(op: int, n_outer: int, n_inner: int, V: int, k_cap: int) -> int:
    return int(load().tslt_workspace_bytes(op, n_outer, n_inner, V, k_cap))


def _workspace(nbytes: int, device) -> Optional[torch.Tensor]:
    if nbytes == 0:
        return None
    return torch.empty(nbytes, dtype=torch.uint8, device=device)   # torch aligns to >= 256 bytes


def truncate(logits: torch.Tensor, temperature: float, top_k: int, top_p: float, k_cap: int,
             want_prob: bool = True, out: Optional[dict] = None, u: Optional[torch.Tensor] = None,
             payload: str = "f32", without_replacement: bool = False) -> dict:
    """tslt_truncate over logits [..., V].  Returns idx, logit, prob, count, mass, status ([rows, k_cap] /
    [rows]).  With uniforms u [rows, n] it is tslt_truncate_sample: the result also holds token, slot
    [rows, n], n draws from each row's q_hat (i.i.d., or without replacement).  payload = "bf16" / "f16" rounds the kept values to the
    format in which they will travel before q_hat and the draws are computed."""
    lib = load()
    _dev(logits, name="logits", contiguous=False)
    rows, V, stride = _rows_2d(logits)
    dev = logits.device
    if out is None:
        out = {
            "idx": torch.empty(rows, k_cap, dtype=torch.int32, device=dev),
            "logit": torch.empty(rows, k_cap, dtype=torch.float32, device=dev),
            "prob": torch.empty(rows, k_cap, dtype=torch.float32, device=dev) if want_prob else None,
            "count": torch.empty(rows, dtype=torch.int32, device=dev),
            "mass": torch.empty(rows, dtype=torch.float32, device=dev),
            "status": torch.empty(rows, dtype=torch.int32, device=dev),
        }
    if u is None:
        _check(lib.tslt_truncate(_ptr(logits), _dtype_code(logits), rows, V, stride, float(temperature), int(top_k),
                                 float(top_p), int(k_cap), PAYLOAD[payload], _ptr(out["idx"]), _ptr(out["logit"]), _ptr(out.get("prob")),
                                 _ptr(out["count"]), _ptr(out.get("mass")), _ptr(out.get("status")), None, 0, _stream()))
        return out
    _dev(u, torch.float32, "u")
    u2 = u.reshape(rows, -1)
    n = u2.shape[1]
    if "token" not in out:
        out["token"] = torch.empty(rows, n, dtype=torch.int32, device=dev)
        out["slot"] = torch.empty(rows, n, dtype=torch.int32, device=dev)
    _check(lib.tslt_truncate_sample(_ptr(logits), _dtype_code(logits), rows, V, stride, float(temperature), int(top_k),
                                    float(top_p), int(k_cap), PAYLOAD[payload], _ptr(out["idx"]), _ptr(out["logit"]),
                                    _ptr(out.get("prob")), _ptr(out["count"]), _ptr(out.get("mass")),
                                    _ptr(out.get("status")), _ptr(u2), n, 1 if without_replacement else 0,
                                    _ptr(out["token"]), _ptr(out.get("slot")),
                                    None, 0, _stream()))
    return out


def pack(idx: torch.Tensor, logit: torch.Tensor, count: torch.Tensor, V: int, payload: str) -> dict:
    """tslt_pack: truncated sets [rows, k_cap] -> words (uint32, as int32 storage), row_offset [rows + 1] int64."""
    lib = load()
    _dev(idx, torch.int32, "idx"); _dev(logit, torch.float32, "logit"); _dev(count, torch.int32, "count")
    rows, k_cap = idx.shape
    cap = int(lib.tslt_pack_bound_words(rows, k_cap, V))
    words = torch.zeros(max(cap, 1), dtype=torch.int32, device=idx.device)
    offs = torch.empty(rows + 1, dtype=torch.int64, device=idx.device)
    _check(lib.tslt_pack(_ptr(idx), _ptr(logit), _ptr(count), rows, k_cap, int(V), PAYLOAD[payload], _ptr(words), cap,
                         _ptr(offs), _stream()))
    return {"words": words, "row_offset": offs}


def unpack(words: torch.Tensor, row_offset: torch.Tensor, rows: int, k_cap: int, V: int, payload: str) -> dict:
    """tslt_unpack: the inverse of pack -> idx, logit [rows, k_cap], count [rows]."""
    lib = load()
    _dev(words, torch.int32, "words"); _dev(row_offset, torch.int64, "row_offset")
    dev = words.device
    out = {"idx": torch.empty(rows, k_cap, dtype=torch.int32, device=dev),
           "logit": torch.empty(rows, k_cap, dtype=torch.float32, device=dev),
           "count": torch.empty(rows, dtype=torch.int32, device=dev)}
    _check(lib.tslt_unpack(_ptr(words), _ptr(row_offset), rows, k_cap, int(V), PAYLOAD[payload], _ptr(out["idx"]),
                           _ptr(out["logit"]), _ptr(out["count"]), _stream()))
    return out


def sample(idx: torch.Tensor, logit: torch.Tensor, count: torch.Tensor, u: torch.Tensor,
           without_replacement: bool = False, out: Optional[dict] = None) -> dict:
    """tslt_sample: idx/logit [rows, k_cap], count [rows], u [rows, n] -> token, slot [rows, n]."""
    lib = load()
    _dev(idx, torch.int32, "idx"); _dev(logit, torch.float32, "logit"); _dev(count, torch.int32, "count")
    _dev(u, torch.float32, "u")
    rows, k_cap = idx.shape
    u2 = u.reshape(rows, -1)
    n = u2.shape[1]
    if out is None:
        out = {"token": torch.empty(rows, n, dtype=torch.int32, device=idx.device),
               "slot": torch.empty(rows, n, dtype=torch.int32, device=idx.device)}
    _check(lib.tslt_sample(_ptr(idx), _ptr(logit), _ptr(count), rows, k_cap, _ptr(u2), n,
                           1 if without_replacement else 0, _ptr(out["token"]), _ptr(out.get("slot")), _stream()))
    return out


def verify(target: torch.Tensor, temperature: float, q_idx: torch.Tensor, q_logit: torch.Tensor,
           q_count: torch.Tensor, draft_tokens: torch.Tensor, u_accept: torch.Tensor, u_resample: torch.Tensor,
           out: Optional[dict] = None, workspace: Optional[torch.Tensor] = None, phase: str = "both",
           first_stage: int = 0) -> dict:
    """tslt_verify: target [B, gamma+1, V]; sparse sets [B, gamma, k_cap]; returns accept_len [B],
    tokens [B, gamma+1], ratio, beta [B, gamma], status [B].  phase = "accept" / "resample" calls
    tslt_verify_accept / tslt_verify_resample (then `out` and `workspace` must be passed to both).
    first_stage > 0 calls tslt_verify_staged / tslt_verify_accept_staged."""
    lib = load()
    fn = {"both": lib.tslt_verify, "accept": lib.tslt_verify_accept, "resample": lib.tslt_verify_resample}[phase]
    extra = ()
    if first_stage and phase != "resample":
        fn = {"both": lib.tslt_verify_staged, "accept": lib.tslt_verify_accept_staged}[phase]
        extra = (int(first_stage),)
    _dev(target, name="target")
    if target.dim() != 3:
        raise TsltError("target must be [B, gamma+1, V]")
    B, g1, V = target.shape
    gamma = g1 - 1
    _dev(q_idx, torch.int32, "q_idx"); _dev(q_logit, torch.float32, "q_logit"); _dev(q_count, torch.int32, "q_count")
    _dev(draft_tokens, torch.int32, "draft_tokens"); _dev(u_accept, torch.float32, "u_accept")
    _dev(u_resample, torch.float32, "u_resample")
    k_cap = q_idx.shape[-1]
    if q_idx.numel() != B * gamma * k_cap or u_resample.numel() != B * g1 or u_accept.numel() != B * gamma:
        raise TsltError("verify: shapes do not agree")
    dev = target.device
    if out is None:
        out = {"accept_len": torch.empty(B, dtype=torch.int32, device=dev),
               "tokens": torch.empty(B, g1, dtype=torch.int32, device=dev),
               "ratio": torch.empty(B, gamma, dtype=torch.float32, device=dev),
               "beta": torch.empty(B, gamma, dtype=torch.float32, device=dev),
               "status": torch.empty(B, dtype=torch.int32, device=dev)}
    need = workspace_bytes(OP_VERIFY, B, gamma, V, k_cap)
    ws = workspace if workspace is not None else _workspace(need, dev)
    _check(fn(_ptr(target), _dtype_code(target), B, gamma, V, target.stride(1), float(temperature),
              _ptr(q_idx), _ptr(q_logit), _ptr(q_count), k_cap, _ptr(draft_tokens), _ptr(u_accept),
              _ptr(u_resample), _ptr(out["accept_len"]), _ptr(out["tokens"]), _ptr(out.get("ratio")),
              _ptr(out.get("beta")), _ptr(out.get("status")), _ptr(ws), ws.numel() if ws is not None else 0,
              _stream(), *extra))
    return out


STATIC_MAX_POSITIONS = 262144


def verify_static(target: torch.Tensor, temperature: float, q_idx: torch.Tensor, q_logit: torch.Tensor,
                  q_count: torch.Tensor, draft_tokens: torch.Tensor, u_accept: torch.Tensor, u_resample: torch.Tensor,
                  out: dict) -> dict:
    """tslt_verify_static: tslt_verify without a workspace (the library's own static device array holds the
    per-position decisions).  `out` must hold preallocated accept_len, tokens, ratio, beta, status tensors: this
    wrapper allocates nothing either."""
    lib = load()
    _dev(target, name="target")
    if target.dim() != 3:
        raise TsltError("target must be [B, gamma+1, V]")
    B, g1, V = target.shape
    gamma = g1 - 1
    _dev(q_idx, torch.int32, "q_idx"); _dev(q_logit, torch.float32, "q_logit"); _dev(q_count, torch.int32, "q_count")
    _dev(draft_tokens, torch.int32, "draft_tokens"); _dev(u_accept, torch.float32, "u_accept")
    _dev(u_resample, torch.float32, "u_resample")
    k_cap = q_idx.shape[-1]
    if q_idx.numel() != B * gamma * k_cap or u_resample.numel() != B * g1 or u_accept.numel() != B * gamma:
        raise TsltError("verify_static: shapes do not agree")
    if out["accept_len"].numel() != B or out["tokens"].numel() != B * g1:
        raise TsltError("verify_static: output shapes do not agree")
    _check(lib.tslt_verify_static(_ptr(target), _dtype_code(target), B, gamma, V, target.stride(1), float(temperature),
                                  _ptr(q_idx), _ptr(q_logit), _ptr(q_count), k_cap, _ptr(draft_tokens), _ptr(u_accept),
                                  _ptr(u_resample), _ptr(out["accept_len"]), _ptr(out["tokens"]), _ptr(out.get("ratio")),
                                  _ptr(out.get("beta")), _ptr(out.get("status")), _stream()))
    return out


def calibrate_read(src: torch.Tensor, n_blocks: int, sink: torch.Tensor) -> None:
    """tslt_calibrate_read: one read-only streaming launch over the whole of `src` (time it from outside)."""
    _dev(src, name="src"); _dev(sink, name="sink")
    _check(load().tslt_calibrate_read(_ptr(src), src.numel() * src.element_size(), int(n_blocks), _ptr(sink), _stream()))


def truncation_stats(target: torch.Tensor, temperature: float, q_idx: torch.Tensor, q_logit: torch.Tensor,
                     q_count: torch.Tensor, k_list: Sequence[int]) -> dict:
    """tslt_truncation_stats: target [rows, V]; sets [rows, k_cap]; returns keep, beta [rows, len(k_list)] and
    status [rows]."""
    lib = load()
    _dev(target, name="target")
    if target.dim() != 2:
        raise TsltError("target must be [rows, V]")
    rows, V = target.shape
    _dev(q_idx, torch.int32, "q_idx"); _dev(q_logit, torch.float32, "q_logit"); _dev(q_count, torch.int32, "q_count")
    k_cap = q_idx.shape[-1]
    if q_idx.numel() != rows * k_cap or q_logit.numel() != rows * k_cap or q_count.numel() != rows:
        raise TsltError("truncation_stats: shapes do not agree")
    ks = (ctypes.c_int32 * len(k_list))(*[int(k) for k in k_list])
    dev = target.device
    out = {"keep": torch.empty(rows, len(k_list), dtype=torch.float32, device=dev),
           "beta": torch.empty(rows, len(k_list), dtype=torch.float32, device=dev),
           "status": torch.empty(rows, dtype=torch.int32, device=dev)}
    _check(lib.tslt_truncation_stats(_ptr(target), _dtype_code(target), rows, V, target.stride(0), float(temperature),
                                     _ptr(q_idx), _ptr(q_logit), _ptr(q_count), k_cap, ks, len(k_list),
                                     _ptr(out["keep"]), _ptr(out["beta"]), _ptr(out["status"]), _stream()))
    return out


def multicandidate_stats(target: torch.Tensor, temperature: float, q_idx: torch.Tensor, q_logit: torch.Tensor,
                         q_count: torch.Tensor, k: int) -> dict:
    """tslt_multicandidate_stats: target [rows, V]; sets [rows, k_cap]; returns beta [rows, k], theta [rows] and
    status [rows]."""
    lib = load()
    _dev(target, name="target")
    if target.dim() != 2:
        raise TsltError("target must be [rows, V]")
    rows, V = target.shape
    _dev(q_idx, torch.int32, "q_idx"); _dev(q_logit, torch.float32, "q_logit"); _dev(q_count, torch.int32, "q_count")
    k_cap = q_idx.shape[-1]
    if q_idx.numel() != rows * k_cap or q_logit.numel() != rows * k_cap or q_count.numel() != rows:
        raise TsltError("multicandidate_stats: shapes do not agree")
    dev = target.device
    out = {"beta": torch.empty(rows, int(k), dtype=torch.float32, device=dev),
           "theta": torch.empty(rows, dtype=torch.float32, device=dev),
           "status": torch.empty(rows, dtype=torch.int32, device=dev)}
    _check(lib.tslt_multicandidate_stats(_ptr(target), _dtype_code(target), rows, V, target.stride(0), float(temperature),
                                         _ptr(q_idx), _ptr(q_logit), _ptr(q_count), k_cap, int(k), _ptr(out["beta"]),
                                         _ptr(out["theta"]), _ptr(out["status"]), _stream()))
    return out


def verify_tree(target: torch.Tensor, temperature: float, expansion: Sequence[int], q_idx: torch.Tensor,
                q_logit: torch.Tensor, q_count: torch.Tensor, cand_tokens: torch.Tensor, u_accept: torch.Tensor,
                u_resample: torch.Tensor, all_nodes: bool = True, out: Optional[dict] = None,
                workspace: Optional[torch.Tensor] = None, without_replacement: bool = False) -> dict:
    """tslt_verify_tree: target [B, N_nodes, V]; sparse sets [B, N_int, k_cap]; cand_tokens, u_accept
    [B, N_nodes-1]; u_resample [B, N_nodes].  Returns seq [B, depth+1], len [B], node_token / node_slot
    [B, N_nodes] (when all_nodes), ratio and beta [B, N_nodes-1], status [B].  without_replacement selects the rule
    for candidates that were drawn without replacement."""
    lib = load()
    _dev(target, name="target")
    if target.dim() != 3:
        raise TsltError("target must be [B, N_nodes, V]")
    B, n_nodes, V = target.shape
    depth = len(expansion)
    _dev(q_idx, torch.int32, "q_idx"); _dev(q_logit, torch.float32, "q_logit"); _dev(q_count, torch.int32, "q_count")
    _dev(cand_tokens, torch.int32, "cand_tokens"); _dev(u_accept, torch.float32, "u_accept")
    _dev(u_resample, torch.float32, "u_resample")
    k_cap = q_idx.shape[-1]
    dev = target.device
    if out is None:
        out = {"seq": torch.empty(B, depth + 1, dtype=torch.int32, device=dev),
               "len": torch.empty(B, dtype=torch.int32, device=dev),
               "node_token": torch.empty(B, n_nodes, dtype=torch.int32, device=dev) if all_nodes else None,
               "node_slot": torch.empty(B, n_nodes, dtype=torch.int32, device=dev) if all_nodes else None,
               "ratio": torch.empty(B, max(n_nodes - 1, 1), dtype=torch.float32, device=dev),
               "beta": torch.empty(B, max(n_nodes - 1, 1), dtype=torch.float32, device=dev),
               "status": torch.empty(B, dtype=torch.int32, device=dev)}
    need = workspace_bytes(OP_VERIFY_TREE if all_nodes else OP_VERIFY_TREE_PATH, B, n_nodes, V, k_cap)
    ws = workspace if workspace is not None else _workspace(need, dev)
    exp_arr = (ctypes.c_int32 * depth)(*[int(k) for k in expansion])
    _check(lib.tslt_verify_tree(_ptr(target), _dtype_code(target), B, V, target.stride(1), float(temperature), depth,
                                exp_arr, _ptr(q_idx), _ptr(q_logit), _ptr(q_count), k_cap, _ptr(cand_tokens),
                                _ptr(u_accept), _ptr(u_resample), 1 if without_replacement else 0,
                                _ptr(out.get("node_token")),
                                _ptr(out.get("node_slot")), _ptr(out["seq"]), _ptr(out["len"]), _ptr(out.get("ratio")),
                                _ptr(out.get("beta")), _ptr(out.get("status")), _ptr(ws), ws.numel() if ws is not None else 0, _stream()))
    return out
