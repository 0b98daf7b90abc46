"""ctypes binding: same names as the C ABI in include/vlcache.h, argument marshalling only."""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence

import numpy as np

VLC_F32, VLC_BF16 = 0, 1
_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB = None


class VlcError(RuntimeError):
    def __init__(self, code: int, text: str):
        super().__init__("vlcache error %d: %s" % (code, text))
        self.code = code


class Segment(C.Structure):
    _fields_ = [("start", C.c_int32), ("length", C.c_int32), ("is_image", C.c_int32), ("pos", C.c_int32),
                ("old_pos", C.c_int32), ("cache_row", C.c_int32), ("kv_start", C.c_int32)]


class LayerShape(C.Structure):
    _fields_ = [("H", C.c_int32), ("Hq", C.c_int32), ("Hkv", C.c_int32), ("D", C.c_int32), ("I", C.c_int32),
                ("dtype", C.c_int32), ("eps", C.c_float), ("rope_base", C.c_double),
                ("mrope_t", C.c_int32), ("mrope_h", C.c_int32), ("mrope_w", C.c_int32),
                ("n_experts", C.c_int32), ("top_k", C.c_int32)]


class LayerWeights(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("w_ln1", "w_qkv", "b_qkv", "w_o", "w_ln2", "w_gate_up", "w_down",
                                          "w_qnorm", "w_knorm", "w_router")]


class ShiftJob(C.Structure):
    _fields_ = [("k_src", C.c_void_p), ("v_src", C.c_void_p), ("k_dst", C.c_void_p), ("v_dst", C.c_void_p),
                ("src_row", C.c_void_p), ("dst_row", C.c_void_p), ("delta", C.c_void_p), ("n_tok", C.c_int64)]


class LayerPlan(C.Structure):
    _fields_ = [("n_in", C.c_int64), ("n", C.c_int64), ("map", C.c_void_p), ("slot", C.c_void_p),
                ("pos", C.c_void_p), ("row_kv_start", C.c_void_p), ("row_kv_len", C.c_void_p),
                ("kv_rows", C.c_int64), ("n_reuse", C.c_int64), ("reuse_src", C.c_void_p),
                ("reuse_dst", C.c_void_p), ("reuse_delta", C.c_void_p), ("k_pool", C.c_void_p),
                ("v_pool", C.c_void_p), ("pool_rows", C.c_int64), ("pos3", C.c_void_p)]


def lib_path() -> str:
    """libvlcache.so beside this file; VLC_LIB names another build of the same library (e.g. one made with
    `python -m paper_2512_12977_amd.build --tag T --define D` for an ablation measurement)."""
    return os.environ.get("VLC_LIB") or os.path.join(_HERE, "libvlcache.so")


def lib():
    """The loaded library.  There is no fallback: a missing build is an error."""
    global _LIB
    if _LIB is None:
        path = lib_path()
        if not os.path.exists(path):
            raise ImportError("libvlcache.so is not built (%s missing); run "
                              "`python -m paper_2512_12977_amd.build`" % path)
        L = C.CDLL(path)
        L.vlc_last_error.restype = C.c_char_p
        L.vlc_layer_workspace_bytes.restype = C.c_int64
        L.vlc_layer_workspace_bytes.argtypes = [C.c_void_p, C.c_int64]
        L.vlc_plan_layer_rates.argtypes = [C.c_int, C.c_int, C.c_void_p, C.c_int64, C.c_void_p]
        L.vlc_plan_layer_rates_blocks.argtypes = [C.c_int, C.c_int, C.c_void_p, C.c_int64, C.c_void_p]
        L.vlc_plan_token_indices.argtypes = [C.c_int, C.c_void_p, C.c_int, C.c_void_p, C.c_void_p, C.c_int64] + [C.c_void_p] * 6
        L.vlc_plan_next_rows.argtypes = [C.c_int, C.c_void_p, C.c_int, C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p]
        L.vlc_plan_budget_steps.argtypes = [C.c_int, C.c_int, C.c_void_p]
        L.vlc_plan_reuse_rows.argtypes = [C.c_int, C.c_void_p, C.c_int, C.c_void_p, C.c_void_p, C.c_int64] + [C.c_void_p] * 4
        L.vlc_gather_rows.argtypes = [C.c_void_p, C.c_int64, C.c_int64, C.c_void_p, C.c_int64, C.c_void_p, C.c_int, C.c_void_p]
        L.vlc_rope_shift_kv.argtypes = [C.c_void_p] * 7 + [C.c_int64, C.c_int, C.c_int, C.c_double, C.c_int, C.c_void_p]
        L.vlc_rope_shift_kv_layers.argtypes = [C.c_void_p, C.c_int, C.c_int64, C.c_int, C.c_int, C.c_double, C.c_int,
                                               C.c_void_p]
        L.vlc_scatter_kv.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p, C.c_void_p,
                                     C.c_int64, C.c_int, C.c_int, C.c_int, C.c_void_p]
        L.vlc_sparse_q_attention.argtypes = [C.c_void_p] * 5 + [C.c_int64, C.c_int, C.c_int, C.c_int, C.c_float,
                                                                C.c_void_p, C.c_int, C.c_void_p]
        L.vlc_layer_workspace_layout.argtypes = [C.c_void_p, C.c_int64, C.c_void_p]
        L.vlc_mean_squared_error_workspace_bytes.restype = C.c_int64
        L.vlc_mean_squared_error.argtypes = [C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p]
        L.vlc_layer_forward.argtypes = [C.c_void_p] * 8 + [C.c_int64, C.c_void_p]
        L.vlc_layer_forward_timed.argtypes = [C.c_void_p] * 8 + [C.c_int64, C.c_void_p, C.c_void_p]
        L.vlc_layer_forward_chained.argtypes = [C.c_void_p] * 8 + [C.c_int64, C.c_void_p, C.c_int] + [C.c_void_p] * 3
        L.vlc_first_token_workspace_bytes.restype = C.c_int64
        L.vlc_first_token_workspace_bytes.argtypes = [C.c_int, C.c_int64, C.c_int]
        L.vlc_first_token.argtypes = [C.c_void_p, C.c_void_p, C.c_int64, C.c_int, C.c_int64, C.c_float] + \
                                     [C.c_void_p] * 5 + [C.c_int64, C.c_int, C.c_void_p]
        L.vlc_probe_mfma_bf16.argtypes = [C.c_void_p, C.c_int64, C.c_void_p, C.c_int64, C.c_int, C.c_int, C.c_void_p,
                                          C.c_void_p]
        L.vlc_first_token_noalloc_max_bytes.restype = C.c_int64
        L.vlc_first_token_noalloc.argtypes = [C.c_void_p, C.c_void_p, C.c_int64, C.c_int, C.c_int64, C.c_float] + \
                                             [C.c_void_p] * 4 + [C.c_int, C.c_void_p]
        _LIB = L
    return _LIB


def last_error() -> str:
    return lib().vlc_last_error().decode()


def _check(rc: int) -> None:
    if rc != 0:
        raise VlcError(rc, last_error())


def _dev(t) -> Optional[int]:
    """Device pointer of a torch tensor (None stays NULL)."""
    if t is None:
        return None
    if not t.is_cuda:
        raise ValueError("expected a GPU tensor")
    if not t.is_contiguous():
        raise ValueError("expected a contiguous tensor")
    return t.data_ptr()


def _dtype_code(t) -> int:
    import torch
    if t.dtype == torch.float32:
        return VLC_F32
    if t.dtype == torch.bfloat16:
        return VLC_BF16
    raise ValueError("unsupported dtype %s" % t.dtype)


def _stream(stream) -> Optional[int]:
    import torch
    if stream is None:
        return torch.cuda.current_stream().cuda_stream or None
    return getattr(stream, "cuda_stream", stream) or None


def _host_i32(a, name: str) -> np.ndarray:
    a = np.ascontiguousarray(a, dtype=np.int32)
    return a


# ---------------------------------------------------------------------------------------------
# host planning
# ---------------------------------------------------------------------------------------------
def vlc_plan_layer_rates(sens: np.ndarray, budget_steps: int) -> np.ndarray:
    sens = np.ascontiguousarray(sens, dtype=np.float64)
    L, G1 = sens.shape
    k = np.zeros(L, dtype=np.int32)
    _check(lib().vlc_plan_layer_rates(L, G1 - 1, sens.ctypes.data, int(budget_steps), k.ctypes.data))
    return k


def vlc_plan_layer_rates_blocks(sens: np.ndarray, budget_steps: int) -> np.ndarray:
    sens = np.ascontiguousarray(sens, dtype=np.float64)
    L, G1 = sens.shape
    k = np.zeros(L, dtype=np.int32)
    _check(lib().vlc_plan_layer_rates_blocks(L, G1 - 1, sens.ctypes.data, int(budget_steps), k.ctypes.data))
    return k


def _segments(segs: Sequence) -> "C.Array":
    arr = (Segment * len(segs))()
    for i, s in enumerate(segs):
        arr[i] = s if isinstance(s, Segment) else Segment(*s)
    return arr


def vlc_plan_token_indices(segs: Sequence, L: int, k=None, count_override=None, cap: Optional[int] = None):
    """Returns dict of host int32 arrays: n_rows [L], slot/map/pos/kv_start/kv_len [L, cap]."""
    arr = _segments(segs)
    if cap is None:
        cap = sum(s.length for s in arr)
    kk = None if k is None else _host_i32(k, "k")
    oo = None if count_override is None else _host_i32(count_override, "count_override")
    out = {n: np.zeros((L, cap), dtype=np.int32) for n in ("slot", "map", "pos", "kv_start", "kv_len")}
    n_rows = np.zeros(L, dtype=np.int32)
    _check(lib().vlc_plan_token_indices(len(arr), C.addressof(arr), L,
                                        None if kk is None else kk.ctypes.data,
                                        None if oo is None else oo.ctypes.data, cap, n_rows.ctypes.data,
                                        out["slot"].ctypes.data, out["map"].ctypes.data, out["pos"].ctypes.data,
                                        out["kv_start"].ctypes.data, out["kv_len"].ctypes.data))
    out["n_rows"] = n_rows
    return out


def vlc_plan_next_rows(segs: Sequence, L: int, k=None, count_override=None, cap: Optional[int] = None) -> np.ndarray:
    """Host int32 [L, cap]: index of each row of layer l among the rows of layer l + 1 (-1: dropped)."""
    arr = _segments(segs)
    if cap is None:
        cap = sum(s.length for s in arr)
    kk = None if k is None else _host_i32(k, "k")
    oo = None if count_override is None else _host_i32(count_override, "count_override")
    out = np.full((L, cap), -1, dtype=np.int32)
    _check(lib().vlc_plan_next_rows(len(arr), C.addressof(arr), L, None if kk is None else kk.ctypes.data,
                                    None if oo is None else oo.ctypes.data, cap, out.ctypes.data))
    return out


def vlc_plan_budget_steps(mean_rate_bp: int, L: int) -> int:
    steps = C.c_int64()
    _check(lib().vlc_plan_budget_steps(int(mean_rate_bp), int(L), C.addressof(steps)))
    return int(steps.value)


def vlc_plan_reuse_rows(segs: Sequence, L: int, k=None, count_override=None, cap: Optional[int] = None):
    """Returns dict of host int32 arrays: n_reuse [L], src_row/dst_slot/delta [L, cap]."""
    arr = _segments(segs)
    if cap is None:
        cap = max(1, sum(s.length for s in arr if s.is_image))
    kk = None if k is None else _host_i32(k, "k")
    oo = None if count_override is None else _host_i32(count_override, "count_override")
    out = {n: np.zeros((L, cap), dtype=np.int32) for n in ("src_row", "dst_slot", "delta")}
    n_reuse = np.zeros(L, dtype=np.int32)
    _check(lib().vlc_plan_reuse_rows(len(arr), C.addressof(arr), L,
                                     None if kk is None else kk.ctypes.data,
                                     None if oo is None else oo.ctypes.data, cap, n_reuse.ctypes.data,
                                     out["src_row"].ctypes.data, out["dst_slot"].ctypes.data,
                                     out["delta"].ctypes.data))
    out["n_reuse"] = n_reuse
    return out


# ---------------------------------------------------------------------------------------------
# device kernels (torch tensors on the GPU)
# ---------------------------------------------------------------------------------------------
def vlc_gather_rows(src, idx, dst, stream=None) -> None:
    _check(lib().vlc_gather_rows(_dev(src), src.shape[0], src.shape[1], _dev(idx), idx.numel(), _dev(dst),
                                 _dtype_code(src), _stream(stream)))


def vlc_rope_shift_kv(k_src, v_src, k_dst, v_dst, src_row, dst_row, delta, rope_base: float, stream=None) -> None:
    Hkv, D = k_src.shape[-2], k_src.shape[-1]
    _check(lib().vlc_rope_shift_kv(_dev(k_src), _dev(v_src), _dev(k_dst), _dev(v_dst), _dev(src_row),
                                   _dev(dst_row), _dev(delta), src_row.numel(), Hkv, D, float(rope_base),
                                   _dtype_code(k_src), _stream(stream)))


def shift_job_table(jobs) -> np.ndarray:
    """Host bytes of a vlc_shift_job table.  jobs: sequences (k_src, v_src, k_dst, v_dst, src_row, dst_row, delta)
    of GPU tensors (v_src, v_dst may be None); n_tok = src_row.numel().  Copy the result to the GPU
    (torch.from_numpy(table).cuda()) and pass that tensor to vlc_rope_shift_kv_layers; the tensors named here
    must outlive its use."""
    arr = (ShiftJob * max(len(jobs), 1))()
    for i, (ks, vs, kd, vd, src, dst, dl) in enumerate(jobs):
        if not (src.numel() == dst.numel() == dl.numel()):
            raise ValueError("job %d: index arrays differ in length" % i)
        arr[i] = ShiftJob(_dev(ks), _dev(vs), _dev(kd), _dev(vd), _dev(src), _dev(dst), _dev(dl), src.numel())
    return np.frombuffer(bytes(arr), dtype=np.uint8)[:len(jobs) * C.sizeof(ShiftJob)].copy()


def vlc_rope_shift_kv_layers(job_table, n_jobs: int, max_n_tok: int, Hkv: int, D: int, rope_base: float, dtype: int,
                             stream=None) -> None:
    """job_table: GPU uint8 tensor holding n_jobs vlc_shift_job records (see shift_job_table)."""
    if n_jobs and job_table.numel() < n_jobs * C.sizeof(ShiftJob):
        raise ValueError("job table holds fewer than %d jobs" % n_jobs)
    _check(lib().vlc_rope_shift_kv_layers(_dev(job_table), int(n_jobs), int(max_n_tok), int(Hkv), int(D),
                                          float(rope_base), int(dtype), _stream(stream)))


def vlc_scatter_kv(k_new, v_new, dst_row, k_cache, v_cache, stream=None) -> None:
    Hkv, D = k_cache.shape[-2], k_cache.shape[-1]
    _check(lib().vlc_scatter_kv(_dev(k_new), _dev(v_new), _dev(dst_row), dst_row.numel(), _dev(k_cache),
                                _dev(v_cache), k_cache.shape[0], Hkv, D, _dtype_code(k_cache), _stream(stream)))


def vlc_sparse_q_attention(q, k_cache, v_cache, row_kv_start, row_kv_len, scale: float, out, stream=None) -> None:
    n, Hq, D = q.shape
    Hkv = k_cache.shape[-2]
    _check(lib().vlc_sparse_q_attention(_dev(q), _dev(k_cache), _dev(v_cache), _dev(row_kv_start),
                                        _dev(row_kv_len), n, Hq, Hkv, D, float(scale), _dev(out),
                                        _dtype_code(q), _stream(stream)))


def vlc_layer_workspace_bytes(shape: LayerShape, n_rows_max: int) -> int:
    b = lib().vlc_layer_workspace_bytes(C.addressof(shape), int(n_rows_max))
    if b == 0 and n_rows_max > 0:
        raise VlcError(2, last_error())
    return int(b)


WS_FIELDS = ("xn", "qkv", "q", "o", "h1", "n2", "act", "moe_idx", "moe_w", "moe_pos", "moe_y", "moe_logits",
             "moe_offset")


def vlc_layer_workspace_layout(shape: LayerShape, n_rows: int) -> dict:
    off = (C.c_int64 * len(WS_FIELDS))()
    _check(lib().vlc_layer_workspace_layout(C.addressof(shape), int(n_rows), off))
    return dict(zip(WS_FIELDS, [int(v) for v in off]))


def vlc_layer_forward(shape: LayerShape, weights: LayerWeights, plan: LayerPlan, h_in, h_out, k_cache, v_cache,
                      workspace, stream=None) -> None:
    _check(lib().vlc_layer_forward(C.addressof(shape), C.addressof(weights), C.addressof(plan), _dev(h_in),
                                   _dev(h_out), _dev(k_cache), _dev(v_cache), _dev(workspace),
                                   workspace.numel() * workspace.element_size(), _stream(stream)))


LAYER_STAGES = ("rope_shift", "rmsnorm1", "qkv_gemm", "rope_scatter", "attention", "o_gemm", "rmsnorm2",
                "gate_up_swiglu_gemm", "down_gemm")


def vlc_layer_forward_timed(shape: LayerShape, weights: LayerWeights, plan: LayerPlan, h_in, h_out, k_cache,
                            v_cache, workspace, stage_events, stream=None) -> None:
    """stage_events: ctypes array of len(LAYER_STAGES)+1 hipEvent_t handles (c_void_p); NULL entries are skipped."""
    _check(lib().vlc_layer_forward_timed(C.addressof(shape), C.addressof(weights), C.addressof(plan),
                                         _dev(h_in), _dev(h_out), _dev(k_cache), _dev(v_cache), _dev(workspace),
                                         workspace.numel() * workspace.element_size(), _stream(stream),
                                         C.addressof(stage_events)))


def vlc_layer_forward_chained(shape: LayerShape, weights: LayerWeights, plan: LayerPlan, h_in, h_out, k_cache,
                              v_cache, workspace, input_norm_ready: bool, next_w_ln1=None, next_row=None,
                              stage_events=None, stream=None) -> None:
    """next_w_ln1: the input-norm weight of the layer below (device tensor) or None; next_row: int32 [n], the index
    of each row among the rows of the layer below (negative: dropped), None if that layer keeps every row;
    input_norm_ready: the previous call on this workspace was given this layer's weight."""
    if next_row is not None and (next_row.element_size() != 4 or next_row.numel() != plan.n):
        raise ValueError("next_row: int32 tensor with one entry per recomputed row")
    _check(lib().vlc_layer_forward_chained(C.addressof(shape), C.addressof(weights), C.addressof(plan),
                                           _dev(h_in), _dev(h_out), _dev(k_cache), _dev(v_cache), _dev(workspace),
                                           workspace.numel() * workspace.element_size(), _stream(stream),
                                           1 if input_norm_ready else 0,
                                           None if next_w_ln1 is None else _dev(next_w_ln1),
                                           None if next_row is None else _dev(next_row),
                                           None if stage_events is None else C.addressof(stage_events)))


def vlc_first_token_workspace_bytes(H: int, n_req: int, dtype_code: int) -> int:
    b = lib().vlc_first_token_workspace_bytes(int(H), int(n_req), int(dtype_code))
    if b == 0 and n_req > 0:
        raise VlcError(2, last_error())
    return int(b)


def vlc_first_token(h, rows, eps: float, w_norm, w_out, logits, token, workspace, stream=None) -> None:
    """h [n, H]; rows int32 [n_req]; w_out [vocab, H]; logits float32 [n_req, vocab]; token int32 [n_req]."""
    n_req = rows.numel()
    H = h.shape[-1]
    vocab = w_out.shape[0]
    _check(lib().vlc_first_token(_dev(h), _dev(rows), n_req, H, vocab, float(eps), _dev(w_norm), _dev(w_out),
                                 _dev(logits), _dev(token), _dev(workspace),
                                 workspace.numel() * workspace.element_size(), _dtype_code(h), _stream(stream)))


def vlc_first_token_noalloc_max_bytes() -> int:
    return int(lib().vlc_first_token_noalloc_max_bytes())


def vlc_first_token_noalloc(h, rows, eps: float, w_norm, w_out, logits, token, stream=None) -> None:
    """vlc_first_token with the library's built-in scratch array instead of a workspace tensor."""
    _check(lib().vlc_first_token_noalloc(_dev(h), _dev(rows), rows.numel(), h.shape[-1], w_out.shape[0], float(eps),
                                         _dev(w_norm), _dev(w_out), _dev(logits), _dev(token), _dtype_code(h),
                                         _stream(stream)))


def vlc_mean_squared_error(a, b, out, workspace, stream=None) -> None:
    """a, b float32 device tensors of equal size; out float64 [1]; workspace >= vlc_mean_squared_error_workspace_bytes()."""
    assert a.numel() == b.numel()
    _check(lib().vlc_mean_squared_error(_dev(a), _dev(b), a.numel(), _dev(out), _dev(workspace),
                                        workspace.numel() * workspace.element_size(), _stream(stream)))


def vlc_probe_mfma_bf16(operands, out, iters: int, waves_per_simd: int, stream=None) -> float:
    """Enqueues the register-only MFMA loop; returns the flops of the launch (time it with events)."""
    flops = C.c_double()
    _check(lib().vlc_probe_mfma_bf16(_dev(operands), operands.numel() * operands.element_size(), _dev(out), out.numel(),
                                     int(iters), int(waves_per_simd), C.addressof(flops), _stream(stream)))
    return float(flops.value)


def vlc_mean_squared_error_workspace_bytes() -> int:
    return int(lib().vlc_mean_squared_error_workspace_bytes())
