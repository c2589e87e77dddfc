"""ctypes binding of the plain-C oracle (test infrastructure, not product code).

`build()` compiles oracle/relserve_oracle.c twice with gcc: once with fp32
accumulators (the oracle proper) and once with fp64 accumulators (used to
measure the oracle's own rounding error).  `load()` returns a thin wrapper whose
methods take numpy arrays; bf16 data travel as uint16 bit patterns.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "relserve_oracle.c")
_LIBS = {"f32": os.path.join(_HERE, "librelserve_oracle.so"),
         "f64": os.path.join(_HERE, "librelserve_oracle_f64.so")}


def build(force: bool = False, src: str = _SRC, out: dict | None = None, extra: tuple = ()) -> None:
    out = out or _LIBS
    for acc, lib in out.items():
        if (not force and os.path.exists(lib)
                and os.path.getmtime(lib) >= max(os.path.getmtime(src),
                                                 os.path.getmtime(os.path.join(_HERE, "relserve_oracle.h")))):
            continue
        cmd = ["gcc", "-std=c11", "-O3", "-march=native", "-fopenmp", "-fPIC", "-shared",
               "-Wall", "-Wextra", "-I", _HERE, src, "-o", lib, "-lm", *extra]
        if acc == "f64":
            cmd.insert(1, "-DORACLE_ACC_F64")
        subprocess.run(cmd, check=True)


class _Config(C.Structure):
    _fields_ = [("hidden", C.c_int32), ("n_q_heads", C.c_int32), ("n_kv_heads", C.c_int32),
                ("head_dim", C.c_int32), ("mlp_dim", C.c_int32), ("page_size", C.c_int32),
                ("rms_eps", C.c_float), ("rope_base", C.c_float)]


class _Batch(C.Structure):
    _fields_ = [("num_reqs", C.c_int32), ("max_blocks", C.c_int32),
                ("q_start", C.c_void_p), ("ctx_len", C.c_void_p), ("block_table", C.c_void_p)]


class _Weights(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in
                ("w_in_norm", "w_qkv", "w_o", "w_post_norm", "w_gate_up", "w_down")]


class _WeightsW8A8(C.Structure):
    _fields_ = ([(n, C.c_void_p) for n in ("w_in_norm", "w_qkv", "s_qkv", "w_o", "s_o", "w_post_norm", "w_gate_up", "s_gate_up",
                                            "w_down", "s_down")]
                + [(n, C.c_float) for n in ("a_qkv", "a_o", "a_gate_up", "a_down")])


class _Model(C.Structure):
    _fields_ = [("n_layers", C.c_int32), ("vocab", C.c_int32), ("embedding", C.c_void_p),
                ("layers", C.c_void_p), ("w_final_norm", C.c_void_p), ("w_lm_head", C.c_void_p)]


def _ptr(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _chk(a, dtype, name):
    if a.dtype != dtype or not a.flags["C_CONTIGUOUS"]:
        raise TypeError(f"{name}: want C-contiguous {np.dtype(dtype).name}, got {a.dtype}")
    return a


@dataclass
class StepResult:
    y_f32: np.ndarray
    y_bf16: np.ndarray
    attn_out: np.ndarray
    x1: np.ndarray


class Oracle:
    def __init__(self, lib_path: str):
        self.lib = L = C.CDLL(lib_path)
        L.oracle_bf16_to_f32.restype = C.c_float
        L.oracle_bf16_to_f32.argtypes = [C.c_uint16]
        L.oracle_f32_to_bf16.restype = C.c_uint16
        L.oracle_f32_to_bf16.argtypes = [C.c_float]
        L.oracle_rmsnorm.restype = None
        L.oracle_rmsnorm.argtypes = [C.c_void_p, C.c_void_p, C.c_float, C.c_int32, C.c_int32, C.c_void_p]
        L.oracle_linear.restype = None
        L.oracle_linear.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_void_p, C.c_int32, C.c_void_p]
        L.oracle_rope.restype = None
        L.oracle_rope.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_float]
        L.oracle_kv_append.restype = C.c_int32
        L.oracle_kv_append.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                       C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p]
        L.oracle_attention_token.restype = None
        L.oracle_attention_token.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_int32,
                                             C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
        L.oracle_layer_step.restype = C.c_int32
        L.oracle_layer_step.argtypes = [C.c_void_p] * 6 + [C.c_int32, C.c_void_p, C.c_int32] + [C.c_void_p] * 4
        L.oracle_acc_is_f64.restype = C.c_int32
        L.oracle_model_step.restype = C.c_int32
        L.oracle_model_step.argtypes = [C.c_void_p] * 6 + [C.c_int32, C.c_void_p, C.c_void_p]
        L.oracle_num_threads.restype = C.c_int32
        L.oracle_e4m3_to_f32.restype = C.c_float
        L.oracle_e4m3_to_f32.argtypes = [C.c_uint8]
        L.oracle_f32_to_e4m3.restype = C.c_uint8
        L.oracle_f32_to_e4m3.argtypes = [C.c_float]
        L.oracle_attention_token_fp8kv.restype = None
        L.oracle_attention_token_fp8kv.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p,
                                                   C.c_void_p, C.c_float, C.c_float, C.c_void_p]
        L.oracle_layer_step_fp8kv.restype = C.c_int32
        L.oracle_layer_step_fp8kv.argtypes = ([C.c_void_p] * 6 + [C.c_int32, C.c_float, C.c_float, C.c_void_p, C.c_int32]
                                              + [C.c_void_p] * 4)
        L.oracle_quantise.restype = None
        L.oracle_quantise.argtypes = [C.c_void_p, C.c_int64, C.c_float, C.c_void_p]
        L.oracle_linear_w8a8.restype = None
        L.oracle_linear_w8a8.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_void_p, C.c_float, C.c_int32, C.c_void_p]
        L.oracle_layer_step_w8a8.restype = C.c_int32
        L.oracle_layer_step_w8a8.argtypes = ([C.c_void_p] * 6 + [C.c_int32, C.c_int32, C.c_float, C.c_float, C.c_void_p, C.c_int32]
                                             + [C.c_void_p] * 4)
        L.oracle_model_step_w8a8.restype = C.c_int32
        L.oracle_model_step_w8a8.argtypes = [C.c_void_p] * 7 + [C.c_int32, C.c_void_p, C.c_void_p]
        L.oracle_greedy_sample.restype = None
        L.oracle_greedy_sample.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_void_p]

    # -- marshalling helpers -------------------------------------------------
    @staticmethod
    def _cfg(shape) -> _Config:
        return _Config(shape.hidden, shape.n_q_heads, shape.n_kv_heads, shape.head_dim,
                       shape.mlp_dim, shape.page_size, shape.rms_eps, shape.rope_base)

    @staticmethod
    def _batch(batch):
        keep = (_chk(np.ascontiguousarray(batch.q_start), np.int32, "q_start"),
                _chk(np.ascontiguousarray(batch.ctx_len), np.int32, "ctx_len"),
                _chk(np.ascontiguousarray(batch.block_table), np.int32, "block_table"))
        b = _Batch(len(batch.ctx_len), keep[2].shape[1] if keep[2].ndim == 2 else 0,
                   _ptr(keep[0]), _ptr(keep[1]), _ptr(keep[2]))
        return b, keep

    # -- scalar / elementwise pieces ----------------------------------------
    def bf16_to_f32(self, bits: int) -> float:
        return float(self.lib.oracle_bf16_to_f32(int(bits)))

    def f32_to_bf16(self, f: float) -> int:
        return int(self.lib.oracle_f32_to_bf16(float(f)))

    def rmsnorm(self, x: np.ndarray, w_bits: np.ndarray, eps: float) -> np.ndarray:
        x = _chk(np.ascontiguousarray(x), np.float32, "x")
        w_bits = _chk(np.ascontiguousarray(w_bits), np.uint16, "w")
        out = np.empty_like(x)
        self.lib.oracle_rmsnorm(_ptr(x), _ptr(w_bits), eps, x.shape[0], x.shape[1], _ptr(out))
        return out

    def linear(self, w_bits: np.ndarray, inp: np.ndarray) -> np.ndarray:
        w_bits = _chk(np.ascontiguousarray(w_bits), np.uint16, "W")
        inp = _chk(np.ascontiguousarray(inp), np.float32, "in")
        n, k = w_bits.shape
        assert inp.shape[1] == k
        out = np.empty((inp.shape[0], n), np.float32)
        self.lib.oracle_linear(_ptr(w_bits), n, k, _ptr(inp), inp.shape[0], _ptr(out))
        return out

    def rope(self, vec: np.ndarray, pos: int, base: float) -> np.ndarray:
        out = _chk(np.array(vec, dtype=np.float32, order="C"), np.float32, "vec")
        assert out.ndim == 1
        self.lib.oracle_rope(_ptr(out), out.shape[0], int(pos), base)
        return out

    # -- cache and attention ---------------------------------------------------
    def kv_append(self, shape, batch, k_bits, v_bits, k_pages, v_pages):
        """In-place cache write; returns the slot of every token."""
        cfg = self._cfg(shape)
        b, keep = self._batch(batch)
        for a, n in ((k_bits, "k"), (v_bits, "v"), (k_pages, "k_pages"), (v_pages, "v_pages")):
            _chk(a, np.uint16, n)
        slots = np.full(int(batch.q_start[-1]), -1, np.int32)
        rc = self.lib.oracle_kv_append(C.byref(cfg), C.byref(b), _ptr(k_bits), _ptr(v_bits),
                                       _ptr(k_pages), _ptr(v_pages), k_pages.shape[0], _ptr(slots))
        if rc:
            raise ValueError(f"oracle_kv_append rc={rc}")
        del keep
        return slots

    def attention_token(self, shape, batch, r, pos, q, k_pages, v_pages):
        cfg = self._cfg(shape)
        b, keep = self._batch(batch)
        q = _chk(np.ascontiguousarray(q), np.float32, "q")
        out = np.empty((shape.n_q_heads, shape.head_dim), np.float32)
        self.lib.oracle_attention_token(C.byref(cfg), C.byref(b), int(r), int(pos), _ptr(q),
                                        _ptr(_chk(k_pages, np.uint16, "k_pages")),
                                        _ptr(_chk(v_pages, np.uint16, "v_pages")), _ptr(out))
        del keep
        return out

    def e4m3_to_f32(self, code: int) -> float:
        return float(self.lib.oracle_e4m3_to_f32(int(code)))

    def f32_to_e4m3(self, x: float) -> int:
        return int(self.lib.oracle_f32_to_e4m3(float(x)))

    def attention_token_fp8kv(self, shape, batch, r, pos, q, k_pages, v_pages, k_scale, v_scale):
        cfg = self._cfg(shape)
        b, keep = self._batch(batch)
        q = _chk(np.ascontiguousarray(q), np.float32, "q")
        out = np.empty((shape.n_q_heads, shape.head_dim), np.float32)
        self.lib.oracle_attention_token_fp8kv(C.byref(cfg), C.byref(b), int(r), int(pos), _ptr(q),
                                              _ptr(_chk(k_pages, np.uint8, "k_pages")), _ptr(_chk(v_pages, np.uint8, "v_pages")),
                                              float(k_scale), float(v_scale), _ptr(out))
        del keep
        return out

    def quantise(self, values: np.ndarray, scale: float) -> np.ndarray:
        values = _chk(np.ascontiguousarray(values), np.float32, "values")
        codes = np.empty(values.shape, np.uint8)
        self.lib.oracle_quantise(_ptr(values), values.size, float(scale), _ptr(codes))
        return codes

    def linear_w8a8(self, w_codes: np.ndarray, s_w: np.ndarray, in_codes: np.ndarray, a_scale: float) -> np.ndarray:
        w_codes = _chk(np.ascontiguousarray(w_codes), np.uint8, "W codes")
        s_w = _chk(np.ascontiguousarray(s_w), np.float32, "row scales")
        in_codes = _chk(np.ascontiguousarray(in_codes), np.uint8, "input codes")
        n, k = w_codes.shape
        assert in_codes.shape[1] == k and s_w.shape == (n,)
        out = np.empty((in_codes.shape[0], n), np.float32)
        self.lib.oracle_linear_w8a8(_ptr(w_codes), _ptr(s_w), n, k, _ptr(in_codes), float(a_scale), in_codes.shape[0], _ptr(out))
        return out

    @staticmethod
    def _w8a8_struct(weights: dict):
        dt = {"w_in_norm": np.uint16, "w_post_norm": np.uint16, "w_qkv": np.uint8, "w_o": np.uint8, "w_gate_up": np.uint8,
              "w_down": np.uint8, "s_qkv": np.float32, "s_o": np.float32, "s_gate_up": np.float32, "s_down": np.float32}
        wk = {k: _chk(np.ascontiguousarray(weights[k]), t, k) for k, t in dt.items()}
        w = _WeightsW8A8(*[_ptr(wk[n]) for n, t in _WeightsW8A8._fields_ if t is C.c_void_p],
                         *[float(weights[n]) for n, t in _WeightsW8A8._fields_ if t is C.c_float])
        return w, wk

    def layer_step(self, shape, batch, weights: dict, x_bits, k_pages, v_pages, rows=None, kv_scales=None) -> StepResult:
        """One layer step; k_pages / v_pages are updated in place.  kv_scales = (k_scale, v_scale) selects the
        quantised cache: the pools are then uint8 arrays of 8-bit codes.  Weights with a key "s_qkv" select the
        quantised projections: w_qkv / w_o / w_gate_up / w_down are uint8 codes, s_* their fp32 row scales, a_* the
        scale of each projection's input."""
        cfg = self._cfg(shape)
        b, keep = self._batch(batch)
        w8a8 = "s_qkv" in weights
        if w8a8:
            w, wk = self._w8a8_struct(weights)
        else:
            wk = {k: _chk(np.ascontiguousarray(v), np.uint16, k) for k, v in weights.items()}
            w = _Weights(*[_ptr(wk[n]) for n, _ in _Weights._fields_])
        x_bits = _chk(np.ascontiguousarray(x_bits), np.uint16, "x")
        pool_dtype = np.uint16 if kv_scales is None else np.uint8
        _chk(k_pages, pool_dtype, "k_pages")
        _chk(v_pages, pool_dtype, "v_pages")
        T = int(batch.q_start[-1])
        assert x_bits.shape == (T, shape.hidden), (x_bits.shape, T, shape.hidden)
        if rows is not None:
            rows = _chk(np.ascontiguousarray(rows, dtype=np.int32), np.int32, "rows")
        n_out = T if rows is None or len(rows) == 0 else len(rows)
        y = np.empty((n_out, shape.hidden), np.float32)
        yb = np.empty((n_out, shape.hidden), np.uint16)
        attn = np.empty((n_out, shape.n_q_heads * shape.head_dim), np.float32)
        x1 = np.empty((n_out, shape.hidden), np.float32)
        tail = (_ptr(rows) if rows is not None and len(rows) else None, 0 if rows is None else len(rows),
                _ptr(y), _ptr(yb), _ptr(attn), _ptr(x1))
        if w8a8:
            ks, vs = (1.0, 1.0) if kv_scales is None else kv_scales
            rc = self.lib.oracle_layer_step_w8a8(C.byref(cfg), C.byref(b), C.byref(w), _ptr(x_bits),
                                                 _ptr(k_pages), _ptr(v_pages), k_pages.shape[0],
                                                 0 if kv_scales is None else 1, float(ks), float(vs), *tail)
        elif kv_scales is None:
            rc = self.lib.oracle_layer_step(C.byref(cfg), C.byref(b), C.byref(w), _ptr(x_bits),
                                            _ptr(k_pages), _ptr(v_pages), k_pages.shape[0], *tail)
        else:
            rc = self.lib.oracle_layer_step_fp8kv(C.byref(cfg), C.byref(b), C.byref(w), _ptr(x_bits),
                                                  _ptr(k_pages), _ptr(v_pages), k_pages.shape[0],
                                                  float(kv_scales[0]), float(kv_scales[1]), *tail)
        if rc:
            raise ValueError(f"oracle_layer_step rc={rc}")
        del keep, wk
        return StepResult(y, yb, attn, x1)

    def model_step(self, shape, batch, model: dict, token_ids, k_pages: list, v_pages: list):
        """model = {"embedding", "layers": [weights dict, ...], "w_final_norm", "w_lm_head"}.
        Per-layer cache pools are updated in place.  Returns (logits [B, V] fp32, hidden [T, H] bf16 bits)."""
        cfg = self._cfg(shape)
        b, keep = self._batch(batch)
        n_layers = len(model["layers"])
        w8a8 = n_layers > 0 and "s_qkv" in model["layers"][0]     # quantised projections in every layer
        lw = ((_WeightsW8A8 if w8a8 else _Weights) * n_layers)()
        keep_w = []
        for i, wd in enumerate(model["layers"]):
            if w8a8:
                lw[i], wk = self._w8a8_struct(wd)
            else:
                wk = {k: _chk(np.ascontiguousarray(v), np.uint16, k) for k, v in wd.items()}
                lw[i] = _Weights(*[_ptr(wk[n]) for n, _ in _Weights._fields_])
            keep_w.append(wk)
        emb = _chk(np.ascontiguousarray(model["embedding"]), np.uint16, "embedding")
        fin = _chk(np.ascontiguousarray(model["w_final_norm"]), np.uint16, "w_final_norm")
        head = _chk(np.ascontiguousarray(model["w_lm_head"]), np.uint16, "w_lm_head")
        m = _Model(n_layers, emb.shape[0], _ptr(emb), None if w8a8 else C.cast(lw, C.c_void_p), _ptr(fin), _ptr(head))
        ids = _chk(np.ascontiguousarray(token_ids, dtype=np.int32), np.int32, "token_ids")
        kp = (C.c_void_p * n_layers)(*[_chk(a, np.uint16, "k_pages").ctypes.data for a in k_pages])
        vp = (C.c_void_p * n_layers)(*[_chk(a, np.uint16, "v_pages").ctypes.data for a in v_pages])
        T = int(batch.q_start[-1])
        logits = np.empty((len(batch.ctx_len), emb.shape[0]), np.float32)
        hidden = np.empty((T, shape.hidden), np.uint16)
        if w8a8:
            rc = self.lib.oracle_model_step_w8a8(C.byref(cfg), C.byref(m), C.cast(lw, C.c_void_p), C.byref(b), _ptr(ids), kp, vp,
                                                 k_pages[0].shape[0], _ptr(logits), _ptr(hidden))
        else:
            rc = self.lib.oracle_model_step(C.byref(cfg), C.byref(m), C.byref(b), _ptr(ids), kp, vp,
                                            k_pages[0].shape[0], _ptr(logits), _ptr(hidden))
        if rc:
            raise ValueError(f"oracle_model_step rc={rc}")
        del keep, keep_w
        return logits, hidden

    def greedy_sample(self, logits: np.ndarray) -> np.ndarray:
        logits = _chk(np.ascontiguousarray(logits), np.float32, "logits")
        out = np.empty(logits.shape[0], np.int32)
        self.lib.oracle_greedy_sample(_ptr(logits), logits.shape[0], logits.shape[1], _ptr(out))
        return out

    @property
    def num_threads(self) -> int:
        return int(self.lib.oracle_num_threads())

    @property
    def acc_is_f64(self) -> bool:
        return bool(self.lib.oracle_acc_is_f64())


_CACHE: dict = {}


def load(acc: str = "f32") -> Oracle:
    if acc not in _CACHE:
        build()
        _CACHE[acc] = Oracle(_LIBS[acc])
    return _CACHE[acc]
