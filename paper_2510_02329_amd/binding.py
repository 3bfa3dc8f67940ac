"""ctypes binding of the C ABI in include/sj.h.  Argument marshalling only: every step of the
verification path runs inside libsj.so's HIP kernels.  There is no fallback: if the library has not
been built (python -m paper_2510_02329_amd.build) loading raises."""
from __future__ import annotations

import ctypes as C
import os
from typing import Callable, Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))

SJ_OK, SJ_EINVAL, SJ_ECAPACITY, SJ_EHIP, SJ_ENOMEM, SJ_ECALLBACK = 0, -1, -2, -3, -4, -5
SJ_MODE_TWO_STAGE, SJ_MODE_ALIGNMENT, SJ_MODE_JUDGE, SJ_MODE_TOPK = 0, 1, 2, 3
SJ_DBG_LOGITS, SJ_DBG_HIDDEN, SJ_DBG_JUDGE_SCORES, SJ_DBG_P_AT_DRAFT, SJ_DBG_ACCEPT_BITS = 0, 1, 2, 3, 4

TENSOR_IDS = {"embed": 0, "attn_norm": 1, "wq": 2, "wk": 3, "wv": 4, "wo": 5, "ffn_norm": 6,
              "w_gate": 7, "w_up": 8, "w_down": 9, "final_norm": 10, "lm_head": 11,
              "judge_w": 12, "judge_b": 13}
_TENSOR_NAMES = {v: k for k, v in TENSOR_IDS.items()}


class SJError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"sj error {code}: {msg}")
        self.code = code


class SJConfig(C.Structure):
    _fields_ = [("n_layers", C.c_int32), ("d_model", C.c_int32), ("n_q_heads", C.c_int32),
                ("n_kv_heads", C.c_int32), ("head_dim", C.c_int32), ("d_ffn", C.c_int32),
                ("vocab", C.c_int32), ("dtype", C.c_int32), ("rope_base", C.c_float),
                ("rms_eps", C.c_float), ("temperature", C.c_float), ("max_gamma", C.c_int32)]


_TENSOR_FN = C.CFUNCTYPE(C.c_int, C.c_void_p, C.c_int32, C.c_int32, C.c_void_p, C.c_size_t)
_lib: Optional[C.CDLL] = None


def lib_path() -> str:
    return os.path.join(_HERE, "libsj.so")


def load_library() -> C.CDLL:
    global _lib
    if _lib is not None:
        return _lib
    path = lib_path()
    if not os.path.exists(path):
        raise SJError(SJ_EINVAL, f"{path} is not built; run `python -m paper_2510_02329_amd.build`")
    # PyTorch owns the caller's device buffers and streams and ships its own HIP runtime: it has to be in the
    # process before this library is, so that both use that one runtime (loaded the other way round, the
    # library brings in the system's copy and its first HIP call finds no device).
    import torch  # noqa: F401
    lib = C.CDLL(path)
    vp, i32, f32, sz = C.c_void_p, C.c_int32, C.c_float, C.c_size_t
    sig = {
        "sj_model_load": (C.c_int, [C.POINTER(SJConfig), _TENSOR_FN, vp, C.POINTER(vp)]),
        "sj_model_free": (C.c_int, [vp]),
        "sj_model_weight_bytes": (C.c_int64, [vp]),
        "sj_kv_create": (C.c_int, [vp, i32, C.POINTER(i32), C.POINTER(vp)]),
        "sj_kv_free": (C.c_int, [vp]),
        "sj_kv_set": (C.c_int, [vp, i32, vp, vp, i32, i32]),
        "sj_kv_set_layer": (C.c_int, [vp, i32, i32, vp, vp, i32]),
        "sj_kv_set_state": (C.c_int, [vp, i32, i32, i32]),
        "sj_kv_read": (C.c_int, [vp, i32, i32, i32, i32, vp, vp]),
        "sj_kv_state": (C.c_int, [vp, C.POINTER(i32), C.POINTER(i32)]),
        "sj_prefill": (C.c_int, [vp, vp, i32, C.POINTER(i32), i32, vp]),
        "sj_verify_step": (C.c_int, [vp, vp, i32, vp, vp, vp, f32, vp, vp, vp]),
        "sj_verify_head": (C.c_int, [vp, vp, i32, vp, vp, vp, vp, f32, vp, vp, vp]),
        "sj_set_temperature": (C.c_int, [vp, f32]),
        "sj_verify_head_static": (C.c_int, [vp, i32, i32, vp, vp, vp, vp, f32, vp, vp, vp]),
        "sj_draft_block": (C.c_int, [vp, vp, i32, vp, i32, vp, vp, vp]),
        "sj_score_block": (C.c_int, [vp, vp, i32, vp, vp, vp, i32, vp, vp]),
        "sj_judge_train": (C.c_int, [vp, vp, C.c_int64, vp, vp, C.c_int64, i32, vp, i32, vp, vp, vp, vp, vp, vp, vp, vp]),
        "sj_set_mode": (C.c_int, [vp, i32]),
        "sj_set_topk": (C.c_int, [vp, i32]),
        "sj_set_operand_planes": (C.c_int, [vp, i32]),
        "sj_kv_rewind": (C.c_int, [vp, C.POINTER(i32), C.POINTER(i32), vp]),
        "sj_set_kernel_timing": (C.c_int, [vp, i32]),
        "sj_get_kernel_timing": (C.c_int, [vp, C.POINTER(C.c_double), C.POINTER(C.c_int64)]),
        "sj_kernel_class_shape": (C.c_int, [vp, C.c_int32, C.c_int32, C.c_char_p, C.c_int32]),
        "sj_time_kernel_class": (C.c_int, [vp, vp, i32, i32, vp, C.POINTER(C.c_double)]),
        "sj_debug_fetch": (C.c_int, [vp, i32, vp, sz]),
        "sj_last_error": (C.c_char_p, []),
        "sj_version": (C.c_char_p, []),
    }
    for name, (res, args) in sig.items():
        fn = getattr(lib, name)
        fn.restype, fn.argtypes = res, args
    _lib = lib
    return lib


def _check(rc: int) -> None:
    if rc != 0:
        raise SJError(rc, load_library().sj_last_error().decode())


def _ptr(x) -> Optional[int]:
    """Device pointer of a torch tensor (or a raw int / None)."""
    if x is None:
        return None
    if isinstance(x, int):
        return x
    return x.data_ptr()


def _stream(stream) -> Optional[int]:
    if stream is None:
        return None
    return stream if isinstance(stream, int) else stream.cuda_stream


def sj_last_error() -> str:
    return load_library().sj_last_error().decode()


def sj_version() -> str:
    return load_library().sj_version().decode()


def sj_model_load(cfg: SJConfig, provider: Callable[[str, int], np.ndarray]) -> int:
    """provider(name, layer) -> contiguous numpy array in the storage dtype (float32, or uint16 bf16
    bits).  Returns the opaque model handle."""
    lib = load_library()
    err = []

    def cb(_user, tid, layer, dst, nbytes):
        try:
            a = np.ascontiguousarray(provider(_TENSOR_NAMES[tid], layer))
            if a.nbytes != nbytes:
                raise ValueError(f"{_TENSOR_NAMES[tid]}[{layer}]: {a.nbytes} bytes, library wants {nbytes}")
            C.memmove(dst, a.ctypes.data, nbytes)
            return 0
        except Exception as e:  # noqa: BLE001 - reported through the error code
            err.append(e)
            return 1

    out = C.c_void_p()
    rc = lib.sj_model_load(C.byref(cfg), _TENSOR_FN(cb), None, C.byref(out))
    if rc == SJ_ECALLBACK and err:
        raise err[0]
    _check(rc)
    return out.value


def sj_model_free(model: int) -> None:
    _check(load_library().sj_model_free(model))


def sj_model_weight_bytes(model: int) -> int:
    return int(load_library().sj_model_weight_bytes(model))


def sj_kv_create(model: int, batch: int, capacity: Optional[Sequence[int]]) -> int:
    out = C.c_void_p()
    cap = None if capacity is None else (C.c_int32 * len(capacity))(*[int(c) for c in capacity])
    _check(load_library().sj_kv_create(model, batch, cap, C.byref(out)))
    return out.value


def sj_kv_free(kv: int) -> None:
    _check(load_library().sj_kv_free(kv))


def _host(a: Optional[np.ndarray]):
    return None if a is None else np.ascontiguousarray(a).ctypes.data


def sj_kv_set(kv: int, seq: int, k_host: np.ndarray, v_host: np.ndarray, length: int, pending: int) -> None:
    k, v = np.ascontiguousarray(k_host), np.ascontiguousarray(v_host)
    _check(load_library().sj_kv_set(kv, seq, k.ctypes.data, v.ctypes.data, length, pending))


def sj_kv_set_layer(kv: int, seq: int, layer: int, k_host: np.ndarray, v_host: np.ndarray, length: int) -> None:
    k, v = np.ascontiguousarray(k_host), np.ascontiguousarray(v_host)
    _check(load_library().sj_kv_set_layer(kv, seq, layer, k.ctypes.data, v.ctypes.data, length))


def sj_kv_set_state(kv: int, seq: int, length: int, pending: int) -> None:
    _check(load_library().sj_kv_set_state(kv, seq, length, pending))


def sj_kv_read(kv: int, seq: int, layer: int, pos0: int, n: int, k_out: np.ndarray, v_out: np.ndarray) -> None:
    assert k_out.flags.c_contiguous and v_out.flags.c_contiguous
    _check(load_library().sj_kv_read(kv, seq, layer, pos0, n, k_out.ctypes.data, v_out.ctypes.data))


def sj_kv_state(kv: int, batch: int):
    ln, pd = (C.c_int32 * batch)(), (C.c_int32 * batch)()
    _check(load_library().sj_kv_state(kv, ln, pd))
    return np.array(ln[:], dtype=np.int32), np.array(pd[:], dtype=np.int32)


def sj_prefill(model: int, kv: int, seq: int, tokens: Sequence[int], stream=None) -> None:
    arr = (C.c_int32 * len(tokens))(*[int(t) for t in tokens])
    _check(load_library().sj_prefill(model, kv, seq, arr, len(tokens), _stream(stream)))


def sj_verify_step(model: int, kv: int, gamma: int, draft_tokens, draft_probs, uniforms, judge_threshold: float,
                   accepted_len, next_token, stream=None) -> None:
    _check(load_library().sj_verify_step(model, kv, gamma, _ptr(draft_tokens), _ptr(draft_probs), _ptr(uniforms),
                                         float(judge_threshold), _ptr(accepted_len), _ptr(next_token), _stream(stream)))


def sj_verify_head(model: int, kv: int, gamma: int, hidden, draft_tokens, draft_probs, uniforms,
                   judge_threshold: float, accepted_len, next_token, stream=None) -> None:
    _check(load_library().sj_verify_head(model, kv, gamma, _ptr(hidden), _ptr(draft_tokens), _ptr(draft_probs),
                                         _ptr(uniforms), float(judge_threshold), _ptr(accepted_len), _ptr(next_token),
                                         _stream(stream)))


def sj_set_temperature(model: int, temperature: float) -> None:
    _check(load_library().sj_set_temperature(model, float(temperature)))


def sj_verify_head_static(model: int, batch: int, gamma: int, hidden, draft_tokens, draft_probs, uniforms,
                          judge_threshold: float, accepted_len, next_token, stream=None) -> None:
    _check(load_library().sj_verify_head_static(model, int(batch), int(gamma), _ptr(hidden), _ptr(draft_tokens),
                                                _ptr(draft_probs), _ptr(uniforms), float(judge_threshold),
                                                _ptr(accepted_len), _ptr(next_token), _stream(stream)))


def sj_draft_block(model: int, kv: int, gamma: int, uniforms, feed_last: bool, draft_tokens, draft_probs, stream=None) -> None:
    _check(load_library().sj_draft_block(model, kv, gamma, _ptr(uniforms), 1 if feed_last else 0, _ptr(draft_tokens),
                                         _ptr(draft_probs), _stream(stream)))


def sj_score_block(model: int, kv: int, n: int, input_tokens, target_tokens, logprob, hidden_row: int = 0, hidden_out=None,
                   stream=None) -> None:
    _check(load_library().sj_score_block(model, kv, n, _ptr(input_tokens), _ptr(target_tokens), _ptr(logprob), int(hidden_row),
                                         _ptr(hidden_out), _stream(stream)))


def sj_judge_train(H_train, y_train, H_val, y_val, C_grid, stream=None) -> dict:
    """Judge training on device tensors (fp32 features [n, d], int32 labels [n]); C_grid is a host sequence.
    Returns the host-side outputs of the C call as a dict."""
    n_train, d = H_train.shape
    n_val = H_val.shape[0]
    grid = np.ascontiguousarray(np.asarray(C_grid, np.float64))
    n_C = grid.size
    w_all = np.zeros((n_C, d + 1), np.float64)
    auc = np.zeros(n_C, np.float64)
    passes = np.zeros(n_C, np.int32)
    w_best = np.zeros(d + 1, np.float64)
    best = C.c_int32(-1)
    th_f1, th_r = C.c_double(0.0), C.c_double(0.0)
    _check(load_library().sj_judge_train(_ptr(H_train), _ptr(y_train), n_train, _ptr(H_val), _ptr(y_val), n_val, d,
                                         grid.ctypes.data, n_C, w_all.ctypes.data, auc.ctypes.data, passes.ctypes.data,
                                         C.byref(best), w_best.ctypes.data, C.byref(th_f1), C.byref(th_r), _stream(stream)))
    return {"w_all": w_all, "auc": auc, "passes": passes, "best_index": best.value, "w": w_best[:d].copy(),
            "b": float(w_best[d]), "theta_f1": th_f1.value, "theta_recall": th_r.value}


def sj_set_mode(kv: int, mode: int) -> None:
    _check(load_library().sj_set_mode(kv, mode))


def sj_set_topk(kv: int, k: int) -> None:
    _check(load_library().sj_set_topk(kv, k))


def sj_kv_rewind(kv: int, lengths: Sequence[int], pending: Sequence[int], stream=None) -> None:
    n = len(lengths)
    ln, pd = (C.c_int32 * n)(*[int(x) for x in lengths]), (C.c_int32 * n)(*[int(x) for x in pending])
    _check(load_library().sj_kv_rewind(kv, ln, pd, _stream(stream)))


def sj_set_kernel_timing(kv: int, kernel_class: int) -> None:
    _check(load_library().sj_set_kernel_timing(kv, kernel_class))


def sj_kernel_class_shape(kv: int, kernel_class: int, rows: int) -> str:
    buf = C.create_string_buffer(256)
    _check(load_library().sj_kernel_class_shape(kv, kernel_class, rows, buf, 256))
    return buf.value.decode()


def sj_get_kernel_timing(kv: int):
    ms, n = C.c_double(), C.c_int64()
    _check(load_library().sj_get_kernel_timing(kv, C.byref(ms), C.byref(n)))
    return ms.value, n.value


def sj_time_kernel_class(model: int, kv: int, kernel_class: int, launches: int, stream=None) -> float:
    ms = C.c_double()
    _check(load_library().sj_time_kernel_class(model, kv, kernel_class, launches, _stream(stream), C.byref(ms)))
    return ms.value


def sj_set_operand_planes(kv: int, planes: int) -> None:
    _check(load_library().sj_set_operand_planes(kv, planes))


def sj_debug_fetch(kv: int, what: int, out: np.ndarray) -> np.ndarray:
    assert out.flags.c_contiguous
    _check(load_library().sj_debug_fetch(kv, what, out.ctypes.data, out.nbytes))
    return out
