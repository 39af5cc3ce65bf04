"""ctypes front end of the C oracle (oracle/ff_oracle.c).  TEST INFRASTRUCTURE ONLY.

Only tests, __graft_entry__.smoke() and bench.py's cpu_baseline leg may import this.  It takes
canonical-layout tensors (as produced by the seeded input generators) as numpy/torch CPU arrays
and evaluates the decoder step definition in fp64.  Nothing here touches the HIP path.
"""
from __future__ import annotations

import ctypes as C

import numpy as np
import torch

from . import build as _build

_lib = None


class Mat(C.Structure):
    _fields_ = [("wdtype", C.c_int32), ("n", C.c_int32), ("k", C.c_int32),
                ("w", C.c_void_p), ("s", C.c_void_p), ("z", C.c_void_p)]


class Config(C.Structure):
    _fields_ = [("n_layers", C.c_int32), ("d_model", C.c_int32), ("n_q_heads", C.c_int32),
                ("n_kv_heads", C.c_int32), ("head_dim", C.c_int32), ("d_ffn", C.c_int32),
                ("vocab", C.c_int32), ("rms_eps", C.c_double), ("rope_theta", C.c_double)]


class Layer(C.Structure):
    _fields_ = [("attn_norm", C.c_void_p), ("ffn_norm", C.c_void_p),
                ("wq", Mat), ("wk", Mat), ("wv", Mat), ("wo", Mat),
                ("w_gate", Mat), ("w_up", Mat), ("w_down", Mat)]


class Head(C.Structure):
    _fields_ = [("embed", C.c_void_p), ("final_norm", C.c_void_p), ("lm_head", Mat)]


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(_build.build())
        L = _lib
        L.ffo_bf16_to_f64.restype = C.c_double
        L.ffo_bf16_to_f64.argtypes = [C.c_uint16]
        L.ffo_f16_to_f64.restype = C.c_double
        L.ffo_f16_to_f64.argtypes = [C.c_uint16]
        L.ffo_f64_to_bf16.restype = C.c_uint16
        L.ffo_f64_to_bf16.argtypes = [C.c_double]
        L.ffo_silu.restype = C.c_double
        L.ffo_silu.argtypes = [C.c_double]
        L.ffo_dequant_int8.restype = C.c_double
        L.ffo_dequant_int8.argtypes = [C.c_int8, C.c_uint16]
        L.ffo_dequant_int4.restype = C.c_double
        L.ffo_dequant_int4.argtypes = [C.c_void_p, C.c_int, C.c_uint16, C.c_uint16]
        L.ffo_rmsnorm.argtypes = [C.c_void_p, C.c_void_p, C.c_int, C.c_double, C.c_void_p]
        L.ffo_rope.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_double]
        L.ffo_attention_head.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int, C.c_int,
                                         C.c_size_t, C.c_double, C.c_void_p, C.c_void_p]
        L.ffo_matvec.argtypes = [C.POINTER(Mat), C.c_void_p, C.c_void_p]
        L.ffo_dequant_matrix.argtypes = [C.POINTER(Mat), C.c_void_p]
        L.ffo_layer_step.argtypes = [C.POINTER(Config), C.POINTER(Layer), C.c_void_p, C.c_void_p,
                                     C.c_void_p, C.c_int]
        L.ffo_embed.argtypes = [C.POINTER(Config), C.POINTER(Head), C.c_int, C.c_void_p]
        L.ffo_logits.argtypes = [C.POINTER(Config), C.POINTER(Head), C.c_void_p, C.c_void_p]
        L.ffo_decode_step.argtypes = [C.POINTER(Config), C.POINTER(Layer), C.POINTER(Head),
                                      C.c_void_p, C.c_void_p, C.c_int, C.c_void_p, C.c_int, C.c_void_p]
        assert L.ffo_sizeof_layer() == C.sizeof(Layer) and L.ffo_sizeof_mat() == C.sizeof(Mat)
    return _lib


def _np(t):
    """torch CPU tensor or numpy array -> contiguous numpy array (bf16/fp16 as uint16 bits)."""
    if isinstance(t, torch.Tensor):
        t = t.detach().cpu().contiguous()
        if t.dtype in (torch.bfloat16, torch.float16):
            return t.view(torch.int16).numpy().view(np.uint16)
        return t.numpy()
    return np.ascontiguousarray(t)


def _ptr(a):
    return a.ctypes.data_as(C.c_void_p)


class _Keep:
    """Holds numpy buffers alive next to the ctypes structs that point into them."""

    def __init__(self):
        self.bufs = []

    def mat(self, m: dict, wdtype: int) -> Mat:
        w = _np(m["w"])
        self.bufs.append(w)
        n = w.shape[0]
        k = w.shape[1] * (2 if wdtype == 2 else 1)
        out = Mat(wdtype, n, k, w.ctypes.data, None, None)
        if "s" in m:
            s = _np(m["s"])
            self.bufs.append(s)
            out.s = s.ctypes.data
        if "z" in m:
            z = _np(m["z"])
            self.bufs.append(z)
            out.z = z.ctypes.data
        return out

    def vec(self, t):
        a = _np(t)
        self.bufs.append(a)
        return a.ctypes.data


def _mat_wdtype(m: dict) -> int:
    w = m["w"]
    dt = w.dtype
    if dt in (torch.bfloat16,):
        return 0
    if dt in (torch.int8, np.int8):
        return 1
    return 2


class OracleModel:
    """A decoder held as canonical-layout CPU tensors; evaluates steps with the C oracle."""

    def __init__(self, shape, layers: list, head: dict):
        self.shape = shape
        self.keep = _Keep()
        self.cfg = Config(len(layers), shape.d_model, shape.n_q_heads, shape.n_kv_heads,
                          shape.head_dim, shape.d_ffn, shape.vocab, shape.rms_eps, shape.rope_theta)
        self.layers = (Layer * max(1, len(layers)))()
        for i, lw in enumerate(layers):
            L = self.layers[i]
            L.attn_norm = self.keep.vec(lw["attn_norm"])
            L.ffn_norm = self.keep.vec(lw["ffn_norm"])
            for name in ("wq", "wk", "wv", "wo", "w_gate", "w_up", "w_down"):
                setattr(L, name, self.keep.mat(lw[name], _mat_wdtype(lw[name])))
        self.head = Head(self.keep.vec(head["embed"]), self.keep.vec(head["final_norm"]),
                         self.keep.mat(head["lm_head"], _mat_wdtype(head["lm_head"])))

    def new_kv(self, batch: int, max_ctx: int) -> np.ndarray:
        """bf16 bits, [n_layers, batch, 2 (K,V), max_ctx, n_kv_heads, head_dim]."""
        s = self.shape
        return np.zeros((self.cfg.n_layers, batch, 2, max_ctx, s.n_kv_heads, s.head_dim), dtype=np.uint16)

    def decode_step(self, tokens, positions, kv: np.ndarray) -> np.ndarray:
        tokens = np.ascontiguousarray(tokens, dtype=np.int32)
        positions = np.ascontiguousarray(positions, dtype=np.int32)
        batch = tokens.shape[0]
        assert kv.shape[1] == batch and kv.flags.c_contiguous
        assert int(positions.max()) < kv.shape[3]
        logits = np.zeros((batch, self.cfg.vocab), dtype=np.float64)
        lib().ffo_decode_step(C.byref(self.cfg), self.layers, C.byref(self.head), _ptr(tokens),
                              _ptr(positions), batch, _ptr(kv), kv.shape[3], _ptr(logits))
        return logits

    def layer_step(self, layer: int, x: np.ndarray, Kc: np.ndarray, Vc: np.ndarray, pos: int) -> None:
        assert x.dtype == np.float64 and Kc.dtype == np.uint16
        lib().ffo_layer_step(C.byref(self.cfg), C.byref(self.layers[layer]), _ptr(x), _ptr(Kc), _ptr(Vc), pos)

    def embed(self, token: int) -> np.ndarray:
        x = np.zeros(self.cfg.d_model, dtype=np.float64)
        lib().ffo_embed(C.byref(self.cfg), C.byref(self.head), int(token), _ptr(x))
        return x

    def logits(self, x: np.ndarray) -> np.ndarray:
        out = np.zeros(self.cfg.vocab, dtype=np.float64)
        lib().ffo_logits(C.byref(self.cfg), C.byref(self.head), _ptr(x), _ptr(out))
        return out


# ---- thin wrappers over the pieces, for the pin tests ----

def rmsnorm(x, gain_bf16, eps):
    x = np.ascontiguousarray(x, dtype=np.float64)
    g = _np(gain_bf16)
    y = np.zeros_like(x)
    lib().ffo_rmsnorm(_ptr(x), _ptr(g), x.shape[0], eps, _ptr(y))
    return y


def rope(v, pos, theta):
    v = np.array(v, dtype=np.float64, copy=True)
    lib().ffo_rope(_ptr(v), v.shape[0], int(pos), float(theta))
    return v


def attention_head(q, K_bf16, V_bf16, alpha, return_probs=False):
    """q fp64 [hd]; K,V bf16 bits [n_keys, hd] (contiguous)."""
    q = np.ascontiguousarray(q, dtype=np.float64)
    K = _np(K_bf16)
    V = _np(V_bf16)
    n, hd = K.shape
    o = np.zeros(hd, dtype=np.float64)
    p = np.zeros(max(n, 1), dtype=np.float64)
    lib().ffo_attention_head(_ptr(q), _ptr(K), _ptr(V), n, hd, hd, float(alpha), _ptr(o), _ptr(p))
    return (o, p[:n]) if return_probs else o


def matvec(m: dict, x):
    keep = _Keep()
    mat = keep.mat(m, _mat_wdtype(m))
    x = np.ascontiguousarray(x, dtype=np.float64)
    y = np.zeros(mat.n, dtype=np.float64)
    lib().ffo_matvec(C.byref(mat), _ptr(x), _ptr(y))
    return y


def dequant_matrix(m: dict) -> np.ndarray:
    keep = _Keep()
    mat = keep.mat(m, _mat_wdtype(m))
    out = np.zeros((mat.n, mat.k), dtype=np.float32)
    lib().ffo_dequant_matrix(C.byref(mat), _ptr(out))
    return out


def silu(z: float) -> float:
    return lib().ffo_silu(float(z))


def bf16_round(x: float) -> int:
    return lib().ffo_f64_to_bf16(float(x))


def bf16_bits_to_f64(a) -> np.ndarray:
    a = np.asarray(a, dtype=np.uint16)
    return (a.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
