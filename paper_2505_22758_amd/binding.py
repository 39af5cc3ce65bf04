"""Thin ctypes binding of include/flashformer.h: argument marshalling only.

Every step of the decode path runs in the HIP kernels of libflashformer.so; torch is used for
device memory (tensors -> data_ptr()) and streams.  There is no fallback: if the library is
missing this module raises at import.
"""
from __future__ import annotations

import ctypes as C
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libflashformer.so")
if not os.path.exists(LIB_PATH):
    raise ImportError(
        f"{LIB_PATH} not found: build it first (python -m paper_2505_22758_amd.build or "
        "__graft_entry__.build()); there is no CPU fallback for the decode path")
_lib = C.CDLL(LIB_PATH)

FF_OK, FF_ERR_ARG, FF_ERR_UNSUPPORTED, FF_ERR_RANGE, FF_ERR_NOMEM, FF_ERR_TIMEOUT, FF_ERR_HIP = 0, -1, -2, -3, -4, -5, -6
FF_W_BF16, FF_W_INT8_PC, FF_W_INT4_G128 = 0, 1, 2
FF_TOKEN_SKIP = -1   # token id of a sequence that sits a decode step out (see include/flashformer.h)
FF_MAT = {"wq": 0, "wk": 1, "wv": 2, "wo": 3, "w_gate": 4, "w_up": 5, "w_down": 6, "lm_head": 7}

EXPORTS = ["ff_last_error", "ff_model_bytes", "ff_model_create", "ff_model_load_layer", "ff_model_load_head",
           "ff_model_load", "ff_model_load_synthetic", "ff_model_free", "ff_kv_bytes", "ff_kv_alloc", "ff_kv_fill", "ff_kv_read", "ff_kv_fill_synthetic", "ff_kv_free",
           "ff_decode_step", "ff_decode_step_static", "ff_decode_step_perop", "ff_status", "ff_debug_dequant", "ff_debug_gemv", "ff_debug_timeline", "ff_debug_stream_read", "ff_debug_stack_linear", "ff_debug_set_overlap", "ff_debug_set_attention_balance", "ff_debug_mute_workgroup",
           "ff_fused_schedule"]


class ff_config(C.Structure):
    _fields_ = [("n_layers", C.c_int32), ("d_model", C.c_int32), ("n_q_heads", C.c_int32), ("n_kv_heads", C.c_int32),
                ("head_dim", C.c_int32), ("d_ffn", C.c_int32), ("vocab", C.c_int32), ("rms_eps", C.c_float),
                ("rope_theta", C.c_float), ("wdtype", C.c_int32), ("max_batch", C.c_int32), ("quant_lm_head", C.c_int32)]


class ff_matrix(C.Structure):
    _fields_ = [("w", C.c_void_p), ("s", C.c_void_p), ("z", C.c_void_p)]


class ff_layer_weights(C.Structure):
    _fields_ = [("attn_norm", C.c_void_p), ("ffn_norm", C.c_void_p), ("wq", ff_matrix), ("wk", ff_matrix), ("wv", ff_matrix),
                ("wo", ff_matrix), ("w_gate", ff_matrix), ("w_up", ff_matrix), ("w_down", ff_matrix)]


class ff_head_weights(C.Structure):
    _fields_ = [("embed", C.c_void_p), ("final_norm", C.c_void_p), ("lm_head", ff_matrix)]


_vp, _i32, _sz = C.c_void_p, C.c_int32, C.c_size_t
_lib.ff_last_error.restype = C.c_char_p
_lib.ff_model_bytes.argtypes = [C.POINTER(ff_config), C.POINTER(_sz), C.POINTER(_sz)]
_lib.ff_model_create.argtypes = [C.POINTER(ff_config), _vp, _sz, _vp, _sz, _vp, C.POINTER(_vp)]
_lib.ff_model_load_layer.argtypes = [_vp, _i32, C.POINTER(ff_layer_weights), _vp]
_lib.ff_model_load_head.argtypes = [_vp, C.POINTER(ff_head_weights), _vp]
_lib.ff_model_load.argtypes = [C.POINTER(ff_config), C.POINTER(ff_layer_weights), C.POINTER(ff_head_weights), _vp, _sz, _vp,
                               _sz, _vp, C.POINTER(_vp)]
_lib.ff_model_load_synthetic.argtypes = [C.POINTER(ff_config), C.c_uint64, _vp, _sz, _vp, _sz, _vp, C.POINTER(_vp)]
_lib.ff_model_free.argtypes = [_vp]
_lib.ff_kv_bytes.argtypes = [_vp, _i32, _i32, C.POINTER(_sz)]
_lib.ff_kv_alloc.argtypes = [_vp, _i32, _i32, _vp, _sz, _vp, C.POINTER(_vp)]
_lib.ff_kv_fill.argtypes = [_vp, _i32, _i32, _i32, _i32, _vp, _vp, _vp]
_lib.ff_kv_read.argtypes = [_vp, _i32, _i32, _i32, _i32, _vp, _vp, _vp]
_lib.ff_kv_fill_synthetic.argtypes = [_vp, C.c_uint64, _i32, _vp]
_lib.ff_debug_stream_read.argtypes = [_vp, _sz, _i32, _vp]
_lib.ff_debug_stack_linear.argtypes = [_vp, _i32, _i32, _vp, _vp, _i32, _vp, _sz, _vp]
_lib.ff_kv_free.argtypes = [_vp]
_lib.ff_decode_step.argtypes = [_vp, _vp, _vp, _vp, _vp, _i32, _vp]
_lib.ff_decode_step_perop.argtypes = [_vp, _vp, _vp, _vp, _vp, _i32, _vp]
_lib.ff_decode_step_static.argtypes = [_vp, _vp, _vp, _vp, _vp, _i32, _vp]
_lib.ff_status.argtypes = [_vp, _vp]
_lib.ff_debug_dequant.argtypes = [_vp, _i32, _i32, _vp, _vp]
_lib.ff_debug_gemv.argtypes = [_vp, _i32, _i32, _vp, _vp, _i32, _i32, _vp]
_lib.ff_debug_timeline.argtypes = [_vp, _vp]
_lib.ff_debug_mute_workgroup.argtypes = [_vp, _i32]
_lib.ff_debug_set_overlap.argtypes = [_vp, _i32]
_lib.ff_debug_set_attention_balance.argtypes = [_vp, _i32]
_lib.ff_fused_schedule.argtypes = [_vp, C.POINTER(_i32), C.POINTER(_i32), C.POINTER(_i32)]


class FFError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        super().__init__(f"{where}: error {code}: {_lib.ff_last_error().decode()}")


def _check(rc: int, where: str) -> None:
    if rc != FF_OK:
        raise FFError(rc, where)


def _ptr(t) -> int | None:
    if t is None:
        return None
    assert t.is_cuda and t.is_contiguous(), "device tensors must be contiguous CUDA/HIP tensors"
    return t.data_ptr()


def _stream(stream=None) -> int:
    s = stream if stream is not None else torch.cuda.current_stream()
    return s.cuda_stream


def make_config(shape, wdtype: int = FF_W_BF16, max_batch: int = 1, quant_lm_head: bool = True) -> ff_config:
    return ff_config(shape.n_layers, shape.d_model, shape.n_q_heads, shape.n_kv_heads, shape.head_dim, shape.d_ffn,
                     shape.vocab, shape.rms_eps, shape.rope_theta, wdtype, max_batch, int(quant_lm_head))


def _matrix(m: dict) -> ff_matrix:
    return ff_matrix(_ptr(m["w"]), _ptr(m.get("s")), _ptr(m.get("z")))


def layer_weights(lw: dict) -> ff_layer_weights:
    return ff_layer_weights(_ptr(lw["attn_norm"]), _ptr(lw["ffn_norm"]), *[_matrix(lw[k]) for k in
                            ("wq", "wk", "wv", "wo", "w_gate", "w_up", "w_down")])


def head_weights(hw: dict) -> ff_head_weights:
    return ff_head_weights(_ptr(hw["embed"]), _ptr(hw["final_norm"]), _matrix(hw["lm_head"]))


# ---- functions mirroring the C ABI one to one ----
def ff_model_bytes(cfg: ff_config):
    a, b = _sz(), _sz()
    _check(_lib.ff_model_bytes(C.byref(cfg), C.byref(a), C.byref(b)), "ff_model_bytes")
    return a.value, b.value


def ff_model_create(cfg: ff_config, packed: torch.Tensor, scratch: torch.Tensor, stream=None) -> int:
    h = _vp()
    _check(_lib.ff_model_create(C.byref(cfg), _ptr(packed), packed.numel() * packed.element_size(), _ptr(scratch),
                                scratch.numel() * scratch.element_size(), _stream(stream), C.byref(h)), "ff_model_create")
    return h.value


def ff_model_load_layer(model: int, layer: int, lw: dict, stream=None) -> None:
    w = layer_weights(lw)
    _check(_lib.ff_model_load_layer(model, layer, C.byref(w), _stream(stream)), "ff_model_load_layer")


def ff_model_load_head(model: int, hw: dict, stream=None) -> None:
    w = head_weights(hw)
    _check(_lib.ff_model_load_head(model, C.byref(w), _stream(stream)), "ff_model_load_head")


def ff_model_load(cfg: ff_config, layers: list, head: dict, packed: torch.Tensor, scratch: torch.Tensor, stream=None) -> int:
    arr = (ff_layer_weights * len(layers))(*[layer_weights(l) for l in layers])
    hw = head_weights(head)
    h = _vp()
    _check(_lib.ff_model_load(C.byref(cfg), arr, C.byref(hw), _ptr(packed), packed.numel() * packed.element_size(),
                              _ptr(scratch), scratch.numel() * scratch.element_size(), _stream(stream), C.byref(h)),
           "ff_model_load")
    return h.value


def ff_model_load_synthetic(cfg: ff_config, seed: int, packed: torch.Tensor, scratch: torch.Tensor, stream=None) -> int:
    h = _vp()
    _check(_lib.ff_model_load_synthetic(C.byref(cfg), seed & 0xFFFFFFFFFFFFFFFF, _ptr(packed), packed.numel() * packed.element_size(),
                                        _ptr(scratch), scratch.numel() * scratch.element_size(), _stream(stream), C.byref(h)),
           "ff_model_load_synthetic")
    return h.value


def ff_model_free(model: int) -> None:
    _check(_lib.ff_model_free(model), "ff_model_free")


def ff_kv_bytes(model: int, batch: int, max_ctx: int) -> int:
    n = _sz()
    _check(_lib.ff_kv_bytes(model, batch, max_ctx, C.byref(n)), "ff_kv_bytes")
    return n.value


def ff_kv_alloc(model: int, batch: int, max_ctx: int, buf: torch.Tensor, stream=None) -> int:
    h = _vp()
    _check(_lib.ff_kv_alloc(model, batch, max_ctx, _ptr(buf), buf.numel() * buf.element_size(), _stream(stream), C.byref(h)),
           "ff_kv_alloc")
    return h.value


def ff_kv_fill(kv: int, layer: int, seq: int, pos0: int, k: torch.Tensor, v: torch.Tensor, stream=None) -> None:
    _check(_lib.ff_kv_fill(kv, layer, seq, pos0, k.shape[0], _ptr(k), _ptr(v), _stream(stream)), "ff_kv_fill")


def ff_kv_read(kv: int, layer: int, seq: int, pos0: int, k_out: torch.Tensor, v_out: torch.Tensor, stream=None) -> None:
    _check(_lib.ff_kv_read(kv, layer, seq, pos0, k_out.shape[0], _ptr(k_out), _ptr(v_out), _stream(stream)), "ff_kv_read")


def ff_kv_fill_synthetic(kv: int, seed: int, n_ctx: int, stream=None) -> None:
    _check(_lib.ff_kv_fill_synthetic(kv, seed & 0xFFFFFFFFFFFFFFFF, n_ctx, _stream(stream)), "ff_kv_fill_synthetic")


def ff_debug_stream_read(buf: torch.Tensor, n_workgroups: int = 256, stream=None) -> None:
    _check(_lib.ff_debug_stream_read(_ptr(buf), buf.numel() * buf.element_size(), n_workgroups, _stream(stream)), "ff_debug_stream_read")


def ff_debug_stack_linear(w: torch.Tensor, x: torch.Tensor, y: torch.Tensor, mode: int, scratch: torch.Tensor, stream=None) -> None:
    assert w.dtype == torch.bfloat16 and w.dim() == 3 and w.shape[1] == w.shape[2] and x.dtype == torch.float32 and y.dtype == torch.float32
    _check(_lib.ff_debug_stack_linear(_ptr(w), w.shape[1], w.shape[0], _ptr(x), _ptr(y), mode, _ptr(scratch),
                                      scratch.numel() * scratch.element_size(), _stream(stream)), "ff_debug_stack_linear")


def ff_kv_free(kv: int) -> None:
    _check(_lib.ff_kv_free(kv), "ff_kv_free")


def ff_decode_step(model: int, tokens: torch.Tensor, positions: torch.Tensor, kv: int, logits: torch.Tensor, batch: int,
                   stream=None) -> None:
    assert tokens.dtype == torch.int32 and positions.dtype == torch.int32 and logits.dtype == torch.float32
    _check(_lib.ff_decode_step(model, _ptr(tokens), _ptr(positions), kv, _ptr(logits), batch, _stream(stream)), "ff_decode_step")


def ff_decode_step_static(model: int, tokens: torch.Tensor, positions: torch.Tensor, kv: int, logits: torch.Tensor, batch: int,
                          stream=None) -> None:
    assert tokens.dtype == torch.int32 and positions.dtype == torch.int32 and logits.dtype == torch.float32
    _check(_lib.ff_decode_step_static(model, _ptr(tokens), _ptr(positions), kv, _ptr(logits), batch, _stream(stream)),
           "ff_decode_step_static")


def ff_decode_step_perop(model: int, tokens: torch.Tensor, positions: torch.Tensor, kv: int, logits: torch.Tensor,
                         batch: int, stream=None) -> None:
    assert tokens.dtype == torch.int32 and positions.dtype == torch.int32 and logits.dtype == torch.float32
    _check(_lib.ff_decode_step_perop(model, _ptr(tokens), _ptr(positions), kv, _ptr(logits), batch, _stream(stream)),
           "ff_decode_step_perop")


def ff_status(model: int, stream=None) -> None:
    _check(_lib.ff_status(model, _stream(stream)), "ff_status")


def ff_debug_dequant(model: int, layer: int, which: str, out: torch.Tensor, stream=None) -> None:
    assert out.dtype == torch.float32
    _check(_lib.ff_debug_dequant(model, layer, FF_MAT[which], _ptr(out), _stream(stream)), "ff_debug_dequant")


def ff_debug_gemv(model: int, layer: int, which: str, x: torch.Tensor, out: torch.Tensor, path: int, stream=None) -> None:
    assert x.dtype == torch.float32 and out.dtype == torch.float32 and x.dim() == 2 and out.shape[0] == x.shape[0]
    _check(_lib.ff_debug_gemv(model, layer, FF_MAT[which], _ptr(x), _ptr(out), x.shape[0], path, _stream(stream)), "ff_debug_gemv")


def ff_debug_timeline(model: int, buf) -> None:
    _check(_lib.ff_debug_timeline(model, _ptr(buf) if buf is not None else None), "ff_debug_timeline")


def ff_debug_set_overlap(model: int, overlap: bool) -> None:
    _check(_lib.ff_debug_set_overlap(model, int(overlap)), "ff_debug_set_overlap")


def ff_debug_set_attention_balance(model: int, by_length: bool) -> None:
    _check(_lib.ff_debug_set_attention_balance(model, int(by_length)), "ff_debug_set_attention_balance")


def ff_debug_mute_workgroup(model: int, workgroup: int) -> None:
    _check(_lib.ff_debug_mute_workgroup(model, workgroup), "ff_debug_mute_workgroup")


def ff_fused_schedule(model: int):
    a, b, c = _i32(), _i32(), _i32()
    _check(_lib.ff_fused_schedule(model, C.byref(a), C.byref(b), C.byref(c)), "ff_fused_schedule")
    return a.value, b.value, c.value


# ---- plumbing helper: owns the torch buffers behind one model + cache ----
class Decoder:
    """Allocates the caller-side device buffers with torch and keeps the handles together."""

    def __init__(self, shape, wdtype=FF_W_BF16, max_batch=1, quant_lm_head=True, device="cuda:0"):
        self.shape, self.device = shape, torch.device(device)
        self.cfg = make_config(shape, wdtype, max_batch, quant_lm_head)
        pb, sb = ff_model_bytes(self.cfg)
        self.packed = torch.empty(pb, dtype=torch.uint8, device=self.device)
        self.scratch = torch.empty(sb, dtype=torch.uint8, device=self.device)
        self.model = ff_model_create(self.cfg, self.packed, self.scratch)
        self.kv = None
        self.kv_buf = None

    @classmethod
    def synthetic(cls, shape, seed: int, wdtype=FF_W_BF16, max_batch=1, quant_lm_head=True, device="cuda:0"):
        """A decoder filled on the device with the seeded synthetic weights (ff_model_load_synthetic)."""
        self = cls.__new__(cls)
        self.shape, self.device = shape, torch.device(device)
        self.cfg = make_config(shape, wdtype, max_batch, quant_lm_head)
        pb, sb = ff_model_bytes(self.cfg)
        self.packed = torch.empty(pb, dtype=torch.uint8, device=self.device)
        self.scratch = torch.empty(sb, dtype=torch.uint8, device=self.device)
        self.model = ff_model_load_synthetic(self.cfg, seed, self.packed, self.scratch)
        self.kv = None
        self.kv_buf = None
        return self

    def load_layer(self, layer: int, lw: dict):
        ff_model_load_layer(self.model, layer, lw)

    def load_head(self, hw: dict):
        ff_model_load_head(self.model, hw)

    def alloc_kv(self, batch: int, max_ctx: int):
        if self.kv is not None:
            ff_kv_free(self.kv)
        self.kv_buf = torch.zeros(ff_kv_bytes(self.model, batch, max_ctx), dtype=torch.uint8, device=self.device)
        self.kv = ff_kv_alloc(self.model, batch, max_ctx, self.kv_buf)
        self.kv_batch, self.max_ctx = batch, max_ctx

    def step(self, tokens, positions, logits, perop=False):
        fn = ff_decode_step_perop if perop else ff_decode_step
        fn(self.model, tokens, positions, self.kv, logits, tokens.shape[0])

    def close(self):
        if self.kv is not None:
            ff_kv_free(self.kv)
            self.kv = None
        if self.model is not None:
            ff_model_free(self.model)
            self.model = None
