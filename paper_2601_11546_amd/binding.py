"""Thin ctypes binding over librelserve.so (argument marshalling only).

Every function here has the name of the C entry point it calls (include/relserve.h).
Device buffers are torch tensors (PyTorch is used for device memory and streams
only); descriptors are numpy int32 arrays.  There is no fallback: if the library
is not built, importing this module raises.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "librelserve.so")

if not os.path.exists(LIB_PATH):
    raise ImportError(f"{LIB_PATH} is missing: build it with `python -m paper_2601_11546_amd.build` "
                      "(there is no CPU or PyTorch fallback for the layer step)")
# PyTorch ships its own HIP runtime; the library must bind to that one (streams and device pointers come
# from torch), so torch is loaded before the library.  Loaded the other way round, the process holds two
# runtimes and every launch on a torch stream fails.
import torch  # noqa: E402,F401

_lib = C.CDLL(LIB_PATH)

PROFILE_SLOTS = 12

EXPORTS = ["relserve_version", "relserve_strerror", "relserve_config_validate", "relserve_layer_create",
           "relserve_layer_destroy", "relserve_batch_validate", "relserve_batch_slots", "relserve_batch_prepare",
           "relserve_batch_destroy", "relserve_batch_get_info", "relserve_workspace_bytes", "relserve_kv_append",
           "relserve_layer_step", "relserve_layer_step_static", "relserve_static_scratch_bytes", "relserve_model_workspace_bytes", "relserve_model_step", "relserve_greedy_sample", "relserve_rmsnorm", "relserve_linear", "relserve_rope_append",
           "relserve_qkv_rope_append",
           "relserve_attention", "relserve_profile_slot_name", "relserve_profile_enable", "relserve_profile_read",
           "relserve_debug_force_gemm_plan", "relserve_peak_probe_mfma", "relserve_peak_probe_stream", "relserve_peak_probe_stream_pattern",
           "relserve_packed_weight_elems", "relserve_pack_weight", "relserve_linear_packed",
           "relserve_duration_fit", "relserve_duration_predict", "relserve_batch_decompose", "relserve_pem_estimate",
           "relserve_aba_decide", "relserve_starved_priority", "relserve_static_priority", "relserve_utok_estimate",
           "relserve_priority_reuse", "relserve_prefill_candidate",
           "relserve_layer_step_w8a8", "relserve_model_step_w8a8", "relserve_rmsnorm_codes", "relserve_quantise_bf16", "relserve_linear_w8a8"]


class RelserveError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {relserve_strerror(status)} ({status})")


class LayerConfig(C.Structure):
    _fields_ = [("hidden", C.c_int32), ("n_q_heads", C.c_int32), ("n_kv_heads", C.c_int32),
                ("head_dim", C.c_int32), ("mlp_dim", C.c_int32), ("page_size", C.c_int32),
                ("rms_eps", C.c_float), ("rope_base", C.c_float)]


class BatchDesc(C.Structure):
    _fields_ = [("num_reqs", C.c_int32), ("max_blocks", C.c_int32), ("q_start", C.c_void_p),
                ("ctx_len", C.c_void_p), ("block_table", C.c_void_p), ("prefix_id", C.c_void_p),
                ("num_prefixes", C.c_int32), ("prefix_len", C.c_void_p), ("num_pages", C.c_int32)]


class KVCache(C.Structure):
    _fields_ = [("k_pages", C.c_void_p), ("v_pages", C.c_void_p), ("num_pages", C.c_int32), ("dtype", C.c_int32),
                ("k_scale", C.c_float), ("v_scale", C.c_float)]


class QuantPool:
    """A cache pool of 8-bit codes (torch uint8 or float8_e4m3fn tensor [num_pages, P, n_kv, d]) and its scale."""

    def __init__(self, codes, scale: float):
        self.codes, self.scale = codes, float(scale)

    def data_ptr(self):
        return self.codes.data_ptr()

    @property
    def shape(self):
        return self.codes.shape


WEIGHT_NAMES = ("w_in_norm", "w_qkv", "w_o", "w_post_norm", "w_gate_up", "w_down")
MATRIX_NAMES = ("w_qkv", "w_o", "w_gate_up", "w_down")


class LayerWeights(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in WEIGHT_NAMES] + [("packed", C.c_int32)]


class LayerWeightsW8A8(C.Structure):
    _fields_ = ([(n, C.c_void_p) for n in ("w_in_norm", "w_qkv", "s_qkv", "w_o", "s_o", "w_post_norm", "w_gate_up", "s_gate_up",
                                            "w_down", "s_down")]
                + [(n, C.c_float) for n in ("a_qkv", "a_o", "a_gate_up", "a_down")] + [("packed", C.c_int32)])


class Model(C.Structure):
    _fields_ = [("n_layers", C.c_int32), ("vocab", C.c_int32), ("embedding", C.c_void_p), ("layers", C.c_void_p),
                ("caches", C.c_void_p), ("w_final_norm", C.c_void_p), ("w_lm_head", C.c_void_p)]


class DurationModel(C.Structure):
    _fields_ = [("alpha", C.c_double), ("beta", C.c_double), ("r2", C.c_double), ("n", C.c_int32)]


class PemLimits(C.Structure):
    _fields_ = [("cap", C.c_int32), ("max_num_seqs", C.c_int32), ("max_num_batched_tokens", C.c_int32)]


class AbaInput(C.Structure):
    _fields_ = [("m_running", C.c_double), ("m_waiting", C.c_double), ("n_running_reqs", C.c_int32),
                ("cand_prefill_reqs", C.c_int32), ("cand_prefill_utok", C.c_int32), ("cand_prefill_out_len", C.c_int32),
                ("n_running_relqueries", C.c_int32), ("n_waiting_relqueries", C.c_int32), ("running_out_len", C.c_void_p)]


class BatchInfo(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("num_tokens", "num_reqs", "num_decode_rows", "num_prefill_rows",
                                         "num_prefix_groups", "num_attn_items")]


_lib.relserve_version.restype = C.c_int32
_lib.relserve_strerror.restype = C.c_char_p
_lib.relserve_strerror.argtypes = [C.c_int32]
_lib.relserve_profile_slot_name.restype = C.c_char_p
_lib.relserve_profile_slot_name.argtypes = [C.c_int32]
for _n, _a in {
    "relserve_config_validate": [C.c_void_p],
    "relserve_layer_create": [C.c_void_p, C.c_void_p],
    "relserve_layer_destroy": [C.c_void_p],
    "relserve_batch_validate": [C.c_void_p, C.c_void_p],
    "relserve_batch_slots": [C.c_void_p, C.c_void_p, C.c_void_p],
    "relserve_batch_prepare": [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p],
    "relserve_batch_destroy": [C.c_void_p],
    "relserve_batch_get_info": [C.c_void_p, C.c_void_p],
    "relserve_workspace_bytes": [C.c_void_p, C.c_int32, C.c_void_p],
    "relserve_kv_append": [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, KVCache, C.c_void_p],
    "relserve_layer_step": [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, KVCache,
                            C.c_void_p, C.c_size_t, C.c_void_p],
    "relserve_layer_step_static": [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, KVCache, C.c_void_p],
    "relserve_static_scratch_bytes": [C.c_void_p],
    "relserve_layer_step_w8a8": [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, KVCache,
                                 C.c_void_p, C.c_size_t, C.c_void_p],
    "relserve_rmsnorm_codes": [C.c_void_p, C.c_int32, C.c_void_p, C.c_float, C.c_int32, C.c_int32, C.c_float, C.c_void_p,
                               C.c_void_p],
    "relserve_quantise_bf16": [C.c_void_p, C.c_int64, C.c_float, C.c_void_p, C.c_void_p],
    "relserve_linear_w8a8": [C.c_void_p, C.c_void_p, C.c_void_p, C.c_float, C.c_int32, C.c_int32, C.c_int32, C.c_int32,
                             C.c_void_p, C.c_void_p, C.c_float, C.c_int32, C.c_void_p],
    "relserve_model_workspace_bytes": [C.c_void_p, C.c_int32, C.c_int32, C.c_void_p],
    "relserve_model_step": [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t,
                            C.c_void_p],
    "relserve_model_step_w8a8": [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t,
                                 C.c_void_p],
    "relserve_greedy_sample": [C.c_void_p, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p],
    "relserve_rmsnorm": [C.c_void_p, C.c_int32, C.c_void_p, C.c_float, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p],
    "relserve_linear": [C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_void_p,
                        C.c_void_p, C.c_void_p],
    "relserve_linear_packed": [C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_void_p,
                               C.c_void_p, C.c_void_p],
    "relserve_packed_weight_elems": [C.c_int32, C.c_int32, C.c_void_p],
    "relserve_pack_weight": [C.c_void_p, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p],
    "relserve_rope_append": [C.c_void_p, C.c_void_p, C.c_void_p, KVCache, C.c_void_p],
    "relserve_qkv_rope_append": [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, KVCache, C.c_void_p],
    "relserve_attention": [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, KVCache, C.c_void_p, C.c_void_p,
                           C.c_size_t, C.c_void_p],
    "relserve_profile_enable": [C.c_void_p, C.c_int32],
    "relserve_debug_force_gemm_plan": [C.c_int32, C.c_int32],
    "relserve_peak_probe_mfma": [C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p],
    "relserve_peak_probe_stream": [C.c_void_p, C.c_size_t, C.c_void_p, C.c_void_p],
    "relserve_peak_probe_stream_pattern": [C.c_void_p, C.c_size_t, C.c_int32, C.c_void_p, C.c_void_p],
    "relserve_profile_read": [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32],
    "relserve_duration_fit": [C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p],
    "relserve_duration_predict": [C.c_void_p, C.c_double, C.c_void_p],
    "relserve_batch_decompose": [C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p,
                                 C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p],
    "relserve_pem_estimate": [C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p],
    "relserve_aba_decide": [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p],
    "relserve_starved_priority": [C.c_double, C.c_double, C.c_int32, C.c_double, C.c_void_p],
    "relserve_static_priority": [C.c_void_p, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p],
    "relserve_utok_estimate": [C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p],
    "relserve_priority_reuse": [C.c_int32, C.c_int32, C.c_int32, C.c_void_p],
    "relserve_prefill_candidate": [C.c_void_p, C.c_int32, C.c_int64, C.c_int32, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p],
}.items():
    getattr(_lib, _n).restype = C.c_int32
    getattr(_lib, _n).argtypes = _a


def _check(rc: int, where: str) -> None:
    if rc != 0:
        raise RelserveError(rc, where)


def _ptr(t):
    """Device pointer of a torch tensor (or None)."""
    return None if t is None else C.c_void_p(t.data_ptr())


def _stream(stream=None):
    import torch
    s = stream if stream is not None else torch.cuda.current_stream()
    return C.c_void_p(s.cuda_stream)


def _config(shape) -> LayerConfig:
    return LayerConfig(shape.hidden, shape.n_q_heads, shape.n_kv_heads, shape.head_dim, shape.mlp_dim,
                       shape.page_size, shape.rms_eps, shape.rope_base)


def _desc(batch):
    """BatchDesc over numpy arrays; returns (desc, keepalive)."""
    keep = [np.ascontiguousarray(batch.q_start, np.int32), np.ascontiguousarray(batch.ctx_len, np.int32),
            np.ascontiguousarray(batch.block_table, np.int32), np.ascontiguousarray(batch.prefix_id, np.int32),
            np.ascontiguousarray(batch.prefix_len, np.int32)]
    bt = keep[2]
    d = BatchDesc(len(keep[1]), bt.shape[1] if bt.ndim == 2 else 0, keep[0].ctypes.data, keep[1].ctypes.data,
                  bt.ctypes.data if bt.size else None, keep[3].ctypes.data if keep[3].size else None,
                  len(keep[4]), keep[4].ctypes.data if keep[4].size else None, int(batch.num_pages))
    return d, keep


def _cache(k_pages, v_pages) -> KVCache:
    if isinstance(k_pages, QuantPool) != isinstance(v_pages, QuantPool):
        raise TypeError("both pools must be 16-bit tensors or both QuantPool")
    if isinstance(k_pages, QuantPool):
        return KVCache(k_pages.data_ptr(), v_pages.data_ptr(), k_pages.shape[0], 1, k_pages.scale, v_pages.scale)
    return KVCache(k_pages.data_ptr(), v_pages.data_ptr(), k_pages.shape[0], 0, 1.0, 1.0)


# ---- entry points, same names as the C ABI ------------------------------------------------
def relserve_version() -> int:
    return int(_lib.relserve_version())


def relserve_strerror(status: int) -> str:
    return _lib.relserve_strerror(int(status)).decode()


def relserve_config_validate(shape) -> int:
    cfg = _config(shape)
    return int(_lib.relserve_config_validate(C.byref(cfg)))


def relserve_batch_validate(shape, batch) -> int:
    cfg = _config(shape)
    d, keep = _desc(batch)
    return int(_lib.relserve_batch_validate(C.byref(cfg), C.byref(d)))


def relserve_batch_slots(shape, batch) -> np.ndarray:
    cfg = _config(shape)
    d, keep = _desc(batch)
    out = np.empty(int(batch.q_start[-1]), np.int32)
    _check(_lib.relserve_batch_slots(C.byref(cfg), C.byref(d), out.ctypes.data), "relserve_batch_slots")
    return out


class Layer:
    """Owns a relserve_layer handle."""

    def __init__(self, shape):
        self.shape = shape
        self.handle = C.c_void_p()
        cfg = _config(shape)
        _check(_lib.relserve_layer_create(C.byref(cfg), C.byref(self.handle)), "relserve_layer_create")

    def close(self):
        if self.handle:
            _lib.relserve_layer_destroy(self.handle)
            self.handle = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def relserve_layer_create(shape) -> Layer:
    return Layer(shape)


class PreparedBatch:
    """Owns a relserve_batch handle."""

    def __init__(self, layer: Layer, batch, stream=None):
        self.handle = C.c_void_p()
        d, keep = _desc(batch)
        _check(_lib.relserve_batch_prepare(layer.handle, C.byref(d), _stream(stream), C.byref(self.handle)),
               "relserve_batch_prepare")
        self.T = int(batch.q_start[-1])

    @property
    def info(self) -> dict:
        bi = BatchInfo()
        _check(_lib.relserve_batch_get_info(self.handle, C.byref(bi)), "relserve_batch_get_info")
        return {n: getattr(bi, n) for n, _ in BatchInfo._fields_}

    def close(self):
        if self.handle:
            _lib.relserve_batch_destroy(self.handle)
            self.handle = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def relserve_batch_prepare(layer: Layer, batch, stream=None) -> PreparedBatch:
    return PreparedBatch(layer, batch, stream)


def relserve_workspace_bytes(layer: Layer, max_tokens: int) -> int:
    out = C.c_size_t()
    _check(_lib.relserve_workspace_bytes(layer.handle, int(max_tokens), C.byref(out)), "relserve_workspace_bytes")
    return int(out.value)


def relserve_kv_append(layer, pbatch, k, v, k_pages, v_pages, stream=None) -> None:
    _check(_lib.relserve_kv_append(layer.handle, pbatch.handle, _ptr(k), _ptr(v), _cache(k_pages, v_pages),
                                   _stream(stream)), "relserve_kv_append")


def _weights(w: dict) -> LayerWeights:
    """w: the six tensors by name; an entry "packed": True marks matrices converted by relserve_pack_weight."""
    return LayerWeights(*[w[n].data_ptr() for n in WEIGHT_NAMES], int(bool(w.get("packed", False))))


def relserve_layer_step(layer, pbatch, weights: dict, x, y, k_pages, v_pages, workspace, stream=None) -> None:
    wt = _weights(weights)
    _check(_lib.relserve_layer_step(layer.handle, pbatch.handle, C.byref(wt), _ptr(x), _ptr(y),
                                    _cache(k_pages, v_pages), _ptr(workspace),
                                    workspace.numel() * workspace.element_size(), _stream(stream)),
           "relserve_layer_step")


def relserve_layer_step_static(layer, pbatch, weights: dict, x, y, k_pages, v_pages, stream=None) -> None:
    wt = _weights(weights)
    _check(_lib.relserve_layer_step_static(layer.handle, pbatch.handle, C.byref(wt), _ptr(x), _ptr(y),
                                           _cache(k_pages, v_pages), _stream(stream)), "relserve_layer_step_static")


def _weights_w8a8(w: dict) -> LayerWeightsW8A8:
    """w: codes w_* (uint8), row scales s_* (fp32), norm weights (bf16) as device tensors, input scales a_* as numbers."""
    return LayerWeightsW8A8(*[w[n].data_ptr() for n, t in LayerWeightsW8A8._fields_ if t is C.c_void_p],
                            *[float(w[n]) for n, t in LayerWeightsW8A8._fields_ if t is C.c_float],
                            int(bool(w.get("packed", False))))


def relserve_layer_step_w8a8(layer, pbatch, weights: dict, x, y, k_pages, v_pages, workspace, stream=None) -> None:
    wt = _weights_w8a8(weights)
    _check(_lib.relserve_layer_step_w8a8(layer.handle, pbatch.handle, C.byref(wt), _ptr(x), _ptr(y),
                                         _cache(k_pages, v_pages), _ptr(workspace),
                                         workspace.numel() * workspace.element_size(), _stream(stream)),
           "relserve_layer_step_w8a8")


def relserve_rmsnorm_codes(x, w, eps: float, scale: float, out, stream=None) -> None:
    import torch
    _check(_lib.relserve_rmsnorm_codes(_ptr(x), int(x.dtype == torch.float32), _ptr(w), float(eps), x.shape[0],
                                       x.shape[1], float(scale), _ptr(out), _stream(stream)), "relserve_rmsnorm_codes")


def relserve_quantise_bf16(values, scale: float, codes, stream=None) -> None:
    _check(_lib.relserve_quantise_bf16(_ptr(values), values.numel(), float(scale), _ptr(codes), _stream(stream)),
           "relserve_quantise_bf16")


def relserve_linear_w8a8(a, w, w_scale, a_scale: float, epilogue: int, residual, out, out_scale: float = 0.0, n: int = 0,
                         stream=None) -> None:
    """a [T, K], w [N, K] uint8 codes (n > 0: w is packed and has n rows), w_scale [N] fp32."""
    _check(_lib.relserve_linear_w8a8(_ptr(a), _ptr(w), _ptr(w_scale), float(a_scale), a.shape[0], int(n) if n else w.shape[0],
                                     a.shape[1], int(epilogue), _ptr(residual), _ptr(out), float(out_scale), int(n > 0),
                                     _stream(stream)), "relserve_linear_w8a8")


def pack_codes(w):
    """An [N, K] uint8 code matrix in the packed layout: relserve_pack_weight on its rows seen as K / 2 two-byte units."""
    import torch
    n, k = w.shape
    packed = torch.empty(relserve_packed_weight_elems(n, k // 2) * 2, dtype=torch.uint8, device=w.device)
    _check(_lib.relserve_pack_weight(_ptr(w), n, k // 2, _ptr(packed), _stream(None)), "relserve_pack_weight")
    return packed


def pack_layer_weights_w8a8(weights: dict) -> dict:
    out = dict(weights)
    for name in MATRIX_NAMES:
        out[name] = pack_codes(weights[name])
    out["packed"] = True
    return out


def relserve_static_scratch_bytes() -> int:
    out = C.c_size_t()
    _check(_lib.relserve_static_scratch_bytes(C.byref(out)), "relserve_static_scratch_bytes")
    return int(out.value)


def relserve_model_workspace_bytes(layer: Layer, max_tokens: int, max_reqs: int) -> int:
    out = C.c_size_t()
    _check(_lib.relserve_model_workspace_bytes(layer.handle, int(max_tokens), int(max_reqs), C.byref(out)),
           "relserve_model_workspace_bytes")
    return int(out.value)


def relserve_model_step(layer, pbatch, model: dict, token_ids, logits, workspace, stream=None) -> None:
    """model = {"embedding", "layers": [weights dict], "caches": [(k_pages, v_pages)], "w_final_norm", "w_lm_head"}
    of torch tensors.  Layers whose dicts carry row scales ("s_qkv") run with quantised projections."""
    n = len(model["layers"])
    w8a8 = n > 0 and "s_qkv" in model["layers"][0]
    lc = (KVCache * n)(*[_cache(k, v) for k, v in model["caches"]])
    if w8a8:
        lw = (LayerWeightsW8A8 * n)(*[_weights_w8a8(w) for w in model["layers"]])
        m = Model(n, model["embedding"].shape[0], model["embedding"].data_ptr(), None,
                  C.cast(lc, C.c_void_p), model["w_final_norm"].data_ptr(), model["w_lm_head"].data_ptr())
        _check(_lib.relserve_model_step_w8a8(layer.handle, pbatch.handle, C.byref(m), C.cast(lw, C.c_void_p), _ptr(token_ids),
                                             _ptr(logits), _ptr(workspace), workspace.numel() * workspace.element_size(),
                                             _stream(stream)), "relserve_model_step_w8a8")
        return
    lw = (LayerWeights * n)(*[_weights(w) for w in model["layers"]])
    m = Model(n, model["embedding"].shape[0], model["embedding"].data_ptr(), C.cast(lw, C.c_void_p),
              C.cast(lc, C.c_void_p), model["w_final_norm"].data_ptr(), model["w_lm_head"].data_ptr())
    _check(_lib.relserve_model_step(layer.handle, pbatch.handle, C.byref(m), _ptr(token_ids), _ptr(logits),
                                    _ptr(workspace), workspace.numel() * workspace.element_size(), _stream(stream)),
           "relserve_model_step")


def relserve_greedy_sample(logits, next_token, stream=None) -> None:
    """logits: device fp32 [rows, vocab]; next_token: device int32 [rows]."""
    _check(_lib.relserve_greedy_sample(_ptr(logits), logits.shape[0], logits.shape[1], _ptr(next_token), _stream(stream)),
           "relserve_greedy_sample")


def relserve_rmsnorm(x, w, eps: float, out, stream=None) -> None:
    import torch
    _check(_lib.relserve_rmsnorm(_ptr(x), int(x.dtype == torch.float32), _ptr(w), float(eps), x.shape[0],
                                 x.shape[1], _ptr(out), _stream(stream)), "relserve_rmsnorm")


def relserve_linear(a, w, epilogue: int, residual, out, stream=None) -> None:
    _check(_lib.relserve_linear(_ptr(a), _ptr(w), a.shape[0], w.shape[0], w.shape[1], int(epilogue),
                                _ptr(residual), _ptr(out), _stream(stream)), "relserve_linear")


def relserve_packed_weight_elems(n: int, k: int) -> int:
    out = C.c_int64(0)
    _check(_lib.relserve_packed_weight_elems(int(n), int(k), C.byref(out)), "relserve_packed_weight_elems")
    return out.value


def relserve_pack_weight(w, out, stream=None) -> None:
    """w: row-major [N, K] device bf16; out: device bf16 with relserve_packed_weight_elems(N, K) elements."""
    _check(_lib.relserve_pack_weight(_ptr(w), w.shape[0], w.shape[1], _ptr(out), _stream(stream)), "relserve_pack_weight")


def relserve_linear_packed(a, w_packed, n: int, epilogue: int, residual, out, stream=None) -> None:
    _check(_lib.relserve_linear_packed(_ptr(a), _ptr(w_packed), a.shape[0], int(n), a.shape[1], int(epilogue),
                                       _ptr(residual), _ptr(out), _stream(stream)), "relserve_linear_packed")


def pack_layer_weights(weights: dict) -> dict:
    """A copy of a layer's weight dict with the four matrices in the packed layout (torch device tensors)."""
    import torch
    out = dict(weights)
    for name in MATRIX_NAMES:
        w = weights[name]
        packed = torch.empty(relserve_packed_weight_elems(w.shape[0], w.shape[1]), dtype=w.dtype, device=w.device)
        relserve_pack_weight(w, packed)
        out[name] = packed
    out["packed"] = True
    return out


def relserve_rope_append(layer, pbatch, qkv, k_pages, v_pages, stream=None) -> None:
    _check(_lib.relserve_rope_append(layer.handle, pbatch.handle, _ptr(qkv), _cache(k_pages, v_pages),
                                     _stream(stream)), "relserve_rope_append")


def relserve_qkv_rope_append(layer, pbatch, h, w_qkv, q_out, k_pages, v_pages, stream=None) -> None:
    _check(_lib.relserve_qkv_rope_append(layer.handle, pbatch.handle, _ptr(h), _ptr(w_qkv), _ptr(q_out),
                                         _cache(k_pages, v_pages), _stream(stream)), "relserve_qkv_rope_append")


def relserve_attention(layer, pbatch, q, q_pitch: int, k_pages, v_pages, out, workspace, stream=None) -> None:
    _check(_lib.relserve_attention(layer.handle, pbatch.handle, _ptr(q), int(q_pitch), _cache(k_pages, v_pages),
                                   _ptr(out), _ptr(workspace), workspace.numel() * workspace.element_size(),
                                   _stream(stream)), "relserve_attention")


def relserve_peak_probe_mfma(sink, iters: int, stream=None) -> float:
    """Enqueues the MFMA issue loop; returns the flop count of the launch."""
    flops = C.c_double(0.0)
    _check(_lib.relserve_peak_probe_mfma(_ptr(sink), int(iters), C.byref(flops), _stream(stream)), "relserve_peak_probe_mfma")
    return flops.value


def relserve_peak_probe_stream(src, nbytes: int, sink, stream=None) -> None:
    _check(_lib.relserve_peak_probe_stream(_ptr(src), int(nbytes), _ptr(sink), _stream(stream)), "relserve_peak_probe_stream")


def relserve_peak_probe_stream_pattern(src, nbytes: int, pattern: int, sink, stream=None) -> None:
    _check(_lib.relserve_peak_probe_stream_pattern(_ptr(src), int(nbytes), int(pattern), _ptr(sink), _stream(stream)),
           "relserve_peak_probe_stream_pattern")


def relserve_debug_force_gemm_plan(tile: int = -1, tail_splits: int = 0) -> None:
    _check(_lib.relserve_debug_force_gemm_plan(int(tile), int(tail_splits)), "relserve_debug_force_gemm_plan")


def relserve_profile_slot_name(slot: int) -> str:
    return _lib.relserve_profile_slot_name(int(slot)).decode()


def relserve_profile_enable(layer, slots=True) -> None:
    """slots: True = every kernel, False = off, or an iterable of slot names / indices."""
    if slots is True:
        mask = -1
    elif not slots:
        mask = 0
    else:
        names = [relserve_profile_slot_name(i) for i in range(PROFILE_SLOTS)]
        mask = 0
        for s in slots:
            mask |= 1 << (names.index(s) if isinstance(s, str) else int(s))
    _check(_lib.relserve_profile_enable(layer.handle, mask), "relserve_profile_enable")


def relserve_profile_read(layer, reset: bool = True) -> dict:
    ms = (C.c_double * PROFILE_SLOTS)()
    n = (C.c_int64 * PROFILE_SLOTS)()
    _check(_lib.relserve_profile_read(layer.handle, ms, n, int(bool(reset))), "relserve_profile_read")
    out = {}
    for i in range(PROFILE_SLOTS):
        if n[i]:
            out[relserve_profile_slot_name(i)] = {"ms_sum": ms[i], "launches": int(n[i])}
    return out


def relserve_duration_fit(units, seconds) -> dict:
    """Eq. 9's coefficients from measured (size, duration) points: {"alpha", "beta", "r2", "n"}."""
    u = np.ascontiguousarray(units, np.float64)
    s = np.ascontiguousarray(seconds, np.float64)
    if u.ndim != 1 or u.shape != s.shape:
        raise ValueError("units and seconds must be vectors of one length")
    m = DurationModel()
    _check(_lib.relserve_duration_fit(u.ctypes.data_as(C.c_void_p), s.ctypes.data_as(C.c_void_p), len(u), C.byref(m)),
           "relserve_duration_fit")
    return {"alpha": m.alpha, "beta": m.beta, "r2": m.r2, "n": m.n}


def relserve_duration_predict(model: dict, units: float) -> float:
    m = DurationModel(model["alpha"], model["beta"], model.get("r2", 0.0), model.get("n", 0))
    out = C.c_double()
    _check(_lib.relserve_duration_predict(C.byref(m), float(units), C.byref(out)), "relserve_duration_predict")
    return out.value


def _pem_inputs(utok, decodes):
    u = np.ascontiguousarray(utok, np.int32)
    d = None if decodes is None else np.ascontiguousarray(decodes, np.uint8)
    if u.ndim != 1 or (d is not None and d.shape != u.shape):
        raise ValueError("utok and decodes must be vectors of one length")
    return u, d


def relserve_batch_decompose(utok, out_len: int, cap: int, max_num_seqs: int, max_num_batched_tokens: int, decodes=None) -> dict:
    """Algorithm 1: {"prefill_batch_of", "decode_group_of", "prefill_utok", "group_req"} (numpy int32 arrays)."""
    u, d = _pem_inputs(utok, decodes)
    n = len(u)
    lim = PemLimits(cap, max_num_seqs, max_num_batched_tokens)
    pb, dg = np.empty(n, np.int32), np.empty(n, np.int32)
    pu, gr = np.empty(max(n, 1), np.int32), np.empty(max(n, 1), np.int32)
    npre, ngrp = C.c_int32(), C.c_int32()
    _check(_lib.relserve_batch_decompose(u.ctypes.data_as(C.c_void_p), None if d is None else d.ctypes.data_as(C.c_void_p), n,
                                         int(out_len), C.byref(lim), pb.ctypes.data_as(C.c_void_p), dg.ctypes.data_as(C.c_void_p),
                                         pu.ctypes.data_as(C.c_void_p), C.byref(npre), gr.ctypes.data_as(C.c_void_p),
                                         C.byref(ngrp)), "relserve_batch_decompose")
    return {"prefill_batch_of": pb, "decode_group_of": dg, "prefill_utok": pu[:npre.value].copy(),
            "group_req": gr[:ngrp.value].copy()}


def relserve_pem_estimate(utok, out_len: int, cap: int, max_num_seqs: int, max_num_batched_tokens: int,
                          prefill_model: dict, decode_model: dict, decodes=None) -> float:
    """Eq. 10: predicted duration of a relQuery from its requests' uncached tokens and the two fitted lines."""
    u, d = _pem_inputs(utok, decodes)
    lim = PemLimits(cap, max_num_seqs, max_num_batched_tokens)
    mp = DurationModel(prefill_model["alpha"], prefill_model["beta"], 0.0, 0)
    md = DurationModel(decode_model["alpha"], decode_model["beta"], 0.0, 0)
    out = C.c_double()
    _check(_lib.relserve_pem_estimate(u.ctypes.data_as(C.c_void_p), None if d is None else d.ctypes.data_as(C.c_void_p), len(u),
                                      int(out_len), C.byref(lim), C.byref(mp), C.byref(md), C.byref(out)), "relserve_pem_estimate")
    return out.value


def relserve_aba_decide(m_running: float, m_waiting: float, n_running_reqs: int, cand_reqs: int, cand_utok: int,
                        cand_out_len: int, running_out_lens, n_waiting: int, prefill_model: dict, decode_model: dict):
    """Sec. 4.3: (decision, delta) with decision 0 = idle, 1 = run the prefill candidate, 2 = run the decode candidate."""
    ol = np.ascontiguousarray(running_out_lens, np.int32)
    inp = AbaInput(m_running, m_waiting, n_running_reqs, cand_reqs, cand_utok, cand_out_len, len(ol), n_waiting,
                   ol.ctypes.data if len(ol) else None)
    mp = DurationModel(prefill_model["alpha"], prefill_model["beta"], 0.0, 0)
    md = DurationModel(decode_model["alpha"], decode_model["beta"], 0.0, 0)
    dec, delta = C.c_int32(), C.c_double()
    _check(_lib.relserve_aba_decide(C.byref(inp), C.byref(mp), C.byref(md), C.byref(dec), C.byref(delta)), "relserve_aba_decide")
    return dec.value, delta.value


def relserve_starved_priority(priority: float, waiting_seconds: float, n_requests_submitted: int, threshold: float) -> float:
    out = C.c_double()
    _check(_lib.relserve_starved_priority(priority, waiting_seconds, n_requests_submitted, threshold, C.byref(out)),
           "relserve_starved_priority")
    return out.value


def _i32(a):
    a = np.ascontiguousarray(a, np.int32)
    return a, (a.ctypes.data_as(C.c_void_p) if a.size else None)


def relserve_static_priority(tok, out_len: int, l1: dict, l2: dict) -> float:
    """Eq. 6-7: sum over the requests of L1(tok) + L2(out_len), both linear ({"alpha", "beta"})."""
    t, tp = _i32(tok)
    m1 = DurationModel(l1["alpha"], l1["beta"], 0.0, 0)
    m2 = DurationModel(l2["alpha"], l2["beta"], 0.0, 0)
    out = C.c_double()
    _check(_lib.relserve_static_priority(tp, len(t), int(out_len), C.byref(m1), C.byref(m2), C.byref(out)), "relserve_static_priority")
    return out.value


def relserve_utok_estimate(tok, sample_tok, sample_utok) -> np.ndarray:
    """Eq. 11: tok x (cache miss ratio of the sample), rounded to integers."""
    t, tp = _i32(tok)
    st, stp = _i32(sample_tok)
    su, sup = _i32(sample_utok)
    out = np.empty(len(t), np.int32)
    _check(_lib.relserve_utok_estimate(tp, len(t), stp, sup, len(st), out.ctypes.data_as(C.c_void_p) if len(t) else None),
           "relserve_utok_estimate")
    return out


def relserve_priority_reuse(n_submitted: int, n_waiting_before: int, n_waiting_now: int) -> bool:
    out = C.c_int32()
    _check(_lib.relserve_priority_reuse(int(n_submitted), int(n_waiting_before), int(n_waiting_now), C.byref(out)),
           "relserve_priority_reuse")
    return bool(out.value)


def relserve_prefill_candidate(utok, tokens_free: int, seqs_free: int, tokens_in_batch: int, max_num_batched_tokens: int):
    """Sec. 4.3: (requests taken from the front of utok, their tokens) under the three limits."""
    u, up = _i32(utok)
    n, toks = C.c_int32(), C.c_int64()
    _check(_lib.relserve_prefill_candidate(up, len(u), int(tokens_free), int(seqs_free), int(tokens_in_batch),
                                           int(max_num_batched_tokens), C.byref(n), C.byref(toks)), "relserve_prefill_candidate")
    return n.value, toks.value

