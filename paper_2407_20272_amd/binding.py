"""ctypes binding of libee_decode.so: the same entry points as include/ee_decode.h, argument marshalling only.

Every step of the decode path runs in the library's HIP kernels; torch is used here for device memory and for
the current HIP stream.  There is no CPU fallback: if the library is missing or no GPU is present the calls raise.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Dict, List, Optional

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libee_decode.so")

EE_OK = 0
EE_ERR_INVALID_ARG, EE_ERR_SHAPE, EE_ERR_UNSUPPORTED, EE_ERR_WORKSPACE, EE_ERR_HIP = -1, -2, -3, -4, -5
EE_FP32, EE_BF16 = 0, 1
EE_PACK_PLAIN, EE_PACK_QKV, EE_PACK_GATE_UP = 0, 1, 2
EXPORTS = ["ee_last_error", "ee_packed_weight_bytes", "ee_pack_weight", "ee_workspace_bytes", "ee_decode_iteration",
           "ee_exit_check", "ee_kv_fill", "ee_paged_attention_decode", "ee_profile_enable", "ee_profile_read", "ee_calibration_copy",
           "ee_noalloc_init", "ee_exit_check_noalloc_bytes", "ee_exit_check_noalloc", "ee_calibration_read", "ee_calibration_mfma",
           "ee_calibration_mfma_tile", "ee_calibration_intake"]
EE_NOALLOC_SCRATCH_BYTES = 8 << 20
KERNEL_CLASSES = ["norm", "qkv", "attention", "o_proj", "gate_up", "down", "head", "combine", "kv_fill", "other"]


class ee_model_desc(C.Structure):
    _fields_ = [("n_layers", C.c_int32), ("d_model", C.c_int32), ("n_heads", C.c_int32), ("head_dim", C.c_int32),
                ("d_ffn", C.c_int32), ("vocab", C.c_int32), ("dtype", C.c_int32), ("rms_eps", C.c_float),
                ("rope_theta", C.c_float), ("exit_every", C.c_int32), ("logit_scale", C.c_float),
                ("conf_mode", C.c_int32)]


class ee_layer_weights(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("g_attn", "w_qkv", "w_o", "g_ffn", "w_gate_up", "w_down")]


class ee_model(C.Structure):
    _fields_ = [("desc", ee_model_desc), ("embed", C.c_void_p), ("g_final", C.c_void_p), ("w_lm", C.c_void_p),
                ("layers", C.POINTER(ee_layer_weights)), ("w_cls", C.c_void_p), ("b_cls", C.c_void_p)]


class ee_kv_cache(C.Structure):
    _fields_ = [("k_pool", C.c_void_p), ("v_pool", C.c_void_p), ("num_blocks", C.c_int32), ("block_size", C.c_int32)]


class ee_batch(C.Structure):
    _fields_ = [("batch", C.c_int32), ("tokens", C.c_void_p), ("context_lens", C.c_void_p),
                ("block_tables", C.c_void_p), ("max_blocks", C.c_int32), ("max_context", C.c_int32),
                ("row_table", C.c_void_p)]


class EEError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"ee_decode error {code}: {msg}")
        self.code = code


_lib = None


def lib() -> C.CDLL:
    """Loads the native library (once).  Raises if it has not been built: there is no fallback path."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_2407_20272_amd.build`")
        L = C.CDLL(LIB_PATH)
        L.ee_last_error.restype = C.c_char_p
        L.ee_packed_weight_bytes.restype = C.c_size_t
        L.ee_packed_weight_bytes.argtypes = [C.c_int32, C.c_int32]
        L.ee_pack_weight.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p]
        L.ee_workspace_bytes.restype = C.c_size_t
        L.ee_workspace_bytes.argtypes = [C.POINTER(ee_model_desc), C.c_int32, C.c_int32]
        L.ee_decode_iteration.argtypes = [C.POINTER(ee_model), C.POINTER(ee_kv_cache), C.POINTER(ee_batch),
                                          C.POINTER(C.c_float), C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p,
                                          C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
        L.ee_exit_check.argtypes = [C.POINTER(ee_model), C.c_int32, C.c_void_p, C.c_int32, C.c_float, C.c_void_p,
                                    C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                    C.c_void_p, C.c_size_t, C.c_void_p]
        L.ee_exit_check_noalloc.argtypes = L.ee_exit_check.argtypes[:13] + [C.c_void_p]
        L.ee_exit_check_noalloc_bytes.restype = C.c_size_t
        L.ee_exit_check_noalloc_bytes.argtypes = [C.POINTER(ee_model_desc), C.c_int32]
        L.ee_noalloc_init.argtypes = []
        L.ee_kv_fill.argtypes = [C.POINTER(ee_model), C.POINTER(ee_kv_cache), C.POINTER(ee_batch), C.c_void_p,
                                 C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
        L.ee_paged_attention_decode.argtypes = [C.POINTER(ee_model_desc), C.POINTER(ee_kv_cache), C.c_int32, C.c_void_p,
                                                C.POINTER(ee_batch), C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
        L.ee_calibration_copy.argtypes = [C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
        L.ee_calibration_copy.restype = C.c_int
        L.ee_calibration_read.argtypes = [C.c_void_p, C.c_size_t, C.c_void_p, C.c_int32, C.c_void_p]
        L.ee_calibration_read.restype = C.c_int
        L.ee_calibration_mfma.argtypes = [C.c_int32, C.c_int32, C.c_void_p, C.c_void_p]
        L.ee_calibration_mfma.restype = C.c_int
        L.ee_calibration_mfma_tile.argtypes = [C.c_int32, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p]
        L.ee_calibration_mfma_tile.restype = C.c_int
        L.ee_calibration_intake.argtypes = [C.c_void_p, C.c_size_t, C.c_void_p, C.c_size_t, C.c_int32, C.c_int32, C.c_int32,
                                            C.c_void_p, C.c_void_p]
        L.ee_calibration_intake.restype = C.c_int
        L.ee_profile_enable.argtypes = [C.c_int32]
        L.ee_profile_read.argtypes = [C.POINTER(C.c_int32), C.POINTER(C.c_int32), C.POINTER(C.c_float), C.c_int32]
        L.ee_profile_enable.restype = C.c_int
        L.ee_profile_read.restype = C.c_int
        for name in ("ee_pack_weight", "ee_decode_iteration", "ee_exit_check", "ee_kv_fill", "ee_paged_attention_decode",
                     "ee_exit_check_noalloc", "ee_noalloc_init"):
            getattr(L, name).restype = C.c_int
        _lib = L
    return _lib


def _check(rc: int):
    if rc != EE_OK:
        raise EEError(rc, lib().ee_last_error().decode())


def _ptr(t: Optional[torch.Tensor]) -> Optional[int]:
    if t is None:
        return None
    assert t.is_cuda and t.is_contiguous(), "device pointer arguments must be contiguous CUDA tensors"
    return t.data_ptr()


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def _i32(t: torch.Tensor) -> torch.Tensor:
    assert t.dtype == torch.int32
    return t


# ------------------------------------------------------------------------------------------------------
# plain wrappers (same names as the C entry points)
# ------------------------------------------------------------------------------------------------------
def make_desc(cfg) -> ee_model_desc:
    return ee_model_desc(cfg.n_layers, cfg.d_model, cfg.n_heads, cfg.head_dim, cfg.d_ffn, cfg.vocab,
                         EE_FP32 if cfg.dtype == "fp32" else EE_BF16, cfg.rms_eps, cfg.rope_theta, cfg.exit_every,
                         cfg.logit_scale, cfg.conf_mode)


def ee_last_error() -> str:
    return lib().ee_last_error().decode()


def ee_packed_weight_bytes(n_out: int, n_in: int) -> int:
    return lib().ee_packed_weight_bytes(n_out, n_in)


def ee_pack_weight(w: torch.Tensor, order: int, pair_stride: int = 0) -> torch.Tensor:
    """Returns the MFMA tile-order image of a plain bf16 [n_out][n_in] matrix (a new device tensor)."""
    assert w.dtype == torch.bfloat16 and w.dim() == 2
    n_out, n_in = w.shape
    out = torch.empty(ee_packed_weight_bytes(n_out, n_in) // 2, dtype=torch.bfloat16, device=w.device)
    _check(lib().ee_pack_weight(_ptr(w.contiguous()), n_out, n_in, order, pair_stride, _ptr(out), _stream()))
    return out


def ee_workspace_bytes(desc: ee_model_desc, max_batch: int, max_context: int) -> int:
    return lib().ee_workspace_bytes(C.byref(desc), max_batch, max_context)


class DeviceModel:
    """Device-resident weights in the layouts the library takes, plus the host-side ee_model record."""

    def __init__(self, cfg, weights: Dict, device="cuda"):
        self.cfg = cfg
        self.desc = make_desc(cfg)
        bf = cfg.dtype == "bf16"
        self._keep: List[torch.Tensor] = []

        def dev(t):
            t = t.to(device).contiguous()
            self._keep.append(t)
            return t

        def mat(t, order=EE_PACK_PLAIN, stride=0):
            t = t.to(device).contiguous()
            if bf:
                t = ee_pack_weight(t, order, stride)
            self._keep.append(t)
            return t

        self.embed = dev(weights["embed"])
        self.g_final = dev(weights["g_final"])
        self.w_lm = mat(weights["w_lm"])
        self.layers = (ee_layer_weights * cfg.n_layers)()
        for i, lw in enumerate(weights["layers"]):
            qkv = torch.cat([lw["w_q"].to(device), lw["w_k"].to(device), lw["w_v"].to(device)], 0)
            gu = torch.cat([lw["w_gate"].to(device), lw["w_up"].to(device)], 0)
            L = self.layers[i]
            L.g_attn = dev(lw["g_attn"]).data_ptr()
            L.w_qkv = mat(qkv, EE_PACK_QKV, cfg.head_dim // 2).data_ptr()
            L.w_o = mat(lw["w_o"]).data_ptr()
            L.g_ffn = dev(lw["g_ffn"]).data_ptr()
            L.w_gate_up = mat(gu, EE_PACK_GATE_UP, cfg.d_ffn).data_ptr()
            L.w_down = mat(lw["w_down"]).data_ptr()
            del qkv, gu
        # dedicated-classifier rows and biases (float32 in every dtype), if the weight set has them
        self.w_cls = dev(weights["w_cls"].float()) if "w_cls" in weights else None
        self.b_cls = dev(weights["b_cls"].float()) if "b_cls" in weights else None
        self.c = ee_model(self.desc, self.embed.data_ptr(), self.g_final.data_ptr(), self.w_lm.data_ptr(), self.layers,
                          self.w_cls.data_ptr() if self.w_cls is not None else None,
                          self.b_cls.data_ptr() if self.b_cls is not None else None)
        torch.cuda.synchronize()

    def with_conf_mode(self, conf_mode: int) -> "DeviceModel":
        """The same device weights under another confidence measure (a second host-side record, nothing copied)."""
        import copy
        v = copy.copy(self)
        v.cfg = self.cfg.with_(conf_mode=conf_mode)
        v.desc = make_desc(v.cfg)
        v.c = ee_model(v.desc, self.c.embed, self.c.g_final, self.c.w_lm, self.layers, self.c.w_cls, self.c.b_cls)
        return v


class PagedKV:
    """Paged K/V pools [n_layers][num_blocks][H][16][dh] in the model dtype."""

    def __init__(self, cfg, num_blocks: int, device="cuda", fill: float = 0.0):
        self.cfg, self.num_blocks = cfg, num_blocks
        shape = (cfg.n_layers, num_blocks, cfg.n_heads, cfg.block_size, cfg.head_dim)
        self.k = torch.full(shape, fill, dtype=cfg.torch_dtype, device=device)
        self.v = torch.full(shape, fill, dtype=cfg.torch_dtype, device=device)
        self.c = ee_kv_cache(self.k.data_ptr(), self.v.data_ptr(), num_blocks, cfg.block_size)


def make_batch(tokens: Optional[torch.Tensor], context_lens: torch.Tensor, block_tables: torch.Tensor,
               max_context: int, row_table: Optional[torch.Tensor] = None) -> ee_batch:
    B = int(context_lens.shape[0])
    b = ee_batch(B, _ptr(_i32(tokens)) if tokens is not None else None, _ptr(_i32(context_lens)),
                 _ptr(_i32(block_tables)), int(block_tables.shape[1]) if block_tables.dim() == 2 else 0, max_context,
                 _ptr(_i32(row_table)) if row_table is not None else None)
    b._keep = (tokens, context_lens, block_tables, row_table)   # the record only holds raw pointers: keep the tensors alive
    return b


class Workspace:
    def __init__(self, desc: ee_model_desc, max_batch: int, max_context: int, device="cuda"):
        self.bytes = ee_workspace_bytes(desc, max_batch, max_context)
        if self.bytes == 0:
            raise EEError(EE_ERR_INVALID_ARG, ee_last_error())
        self.buf = torch.empty(self.bytes, dtype=torch.uint8, device=device)
        assert self.buf.data_ptr() % 256 == 0


EE_EXIT_NONE, EE_EXIT_BATCH, EE_EXIT_PER_SEQUENCE = 0, 1, 2


def ee_decode_iteration(model: DeviceModel, cache: PagedKV, batch: ee_batch, thresholds, forced_exit_layer,
                        use_exit_heads, out_tokens, out_exit_layer, out_batch_exit_layer, out_conf, out_hidden,
                        ws: Workspace):
    n = model.cfg.n_layers
    th = (C.c_float * n)(*([float(thresholds)] * n if isinstance(thresholds, (int, float)) else list(thresholds)))
    _check(lib().ee_decode_iteration(C.byref(model.c), C.byref(cache.c), C.byref(batch), th,
                                     _ptr(forced_exit_layer), int(use_exit_heads), _ptr(out_tokens),
                                     _ptr(out_exit_layer), _ptr(out_batch_exit_layer), _ptr(out_conf), _ptr(out_hidden),
                                     _ptr(ws.buf), ws.bytes, _stream()))


def ee_exit_check(model: DeviceModel, layer: int, hidden, threshold: float, forced_exit_layer, status, exit_layer,
                  n_exited, done_flag, batch_exit_layer, argmax, conf, ws: Workspace):
    _check(lib().ee_exit_check(C.byref(model.c), layer, _ptr(hidden), int(hidden.shape[0]), float(threshold),
                               _ptr(forced_exit_layer), _ptr(status), _ptr(exit_layer), _ptr(n_exited), _ptr(done_flag),
                               _ptr(batch_exit_layer), _ptr(argmax), _ptr(conf), _ptr(ws.buf), ws.bytes, _stream()))


def ee_noalloc_init():
    _check(lib().ee_noalloc_init())


def ee_exit_check_noalloc_bytes(desc: ee_model_desc, batch: int) -> int:
    return lib().ee_exit_check_noalloc_bytes(C.byref(desc), batch)


def ee_exit_check_noalloc(model: DeviceModel, layer: int, hidden, threshold: float, forced_exit_layer, status, exit_layer,
                          n_exited, done_flag, batch_exit_layer, argmax, conf):
    _check(lib().ee_exit_check_noalloc(C.byref(model.c), layer, _ptr(hidden), int(hidden.shape[0]), float(threshold),
                                       _ptr(forced_exit_layer), _ptr(status), _ptr(exit_layer), _ptr(n_exited),
                                       _ptr(done_flag), _ptr(batch_exit_layer), _ptr(argmax), _ptr(conf), _stream()))


def ee_kv_fill(model: DeviceModel, cache: PagedKV, batch: ee_batch, hidden, fill_from_layer, ws: Workspace):
    _check(lib().ee_kv_fill(C.byref(model.c), C.byref(cache.c), C.byref(batch), _ptr(hidden), _ptr(fill_from_layer),
                            _ptr(ws.buf), ws.bytes, _stream()))


def ee_paged_attention_decode(desc: ee_model_desc, cache: PagedKV, layer: int, q, batch: ee_batch, out,
                              ws: Optional[Workspace] = None):
    _check(lib().ee_paged_attention_decode(C.byref(desc), C.byref(cache.c), layer, _ptr(q), C.byref(batch), _ptr(out),
                                           _ptr(ws.buf) if ws else None, ws.bytes if ws else 0, _stream()))


def ee_profile_enable(on: bool):
    _check(lib().ee_profile_enable(int(bool(on))))


def ee_profile_read(max_records: int = 1 << 20):
    """Returns a list of (class name, layer, milliseconds) for every kernel enqueued since the last read."""
    cls = (C.c_int32 * max_records)()
    lay = (C.c_int32 * max_records)()
    ms = (C.c_float * max_records)()
    n = lib().ee_profile_read(cls, lay, ms, max_records)
    if n < 0:
        raise EEError(n, ee_last_error())
    return [(KERNEL_CLASSES[cls[i]], lay[i], ms[i]) for i in range(n)]


def ee_calibration_copy(src: torch.Tensor, dst: torch.Tensor):
    assert src.dtype == torch.float32 and dst.dtype == torch.float32 and src.numel() == dst.numel()
    _check(lib().ee_calibration_copy(_ptr(src), _ptr(dst), src.numel(), _stream()))


def ee_calibration_read(src: torch.Tensor, sink: torch.Tensor, workgroups: int):
    _check(lib().ee_calibration_read(_ptr(src), src.numel() * src.element_size(), _ptr(sink), workgroups, _stream()))


def ee_calibration_mfma(workgroups: int, iterations: int, sink: torch.Tensor):
    assert sink.dtype == torch.float32 and sink.numel() >= 256
    _check(lib().ee_calibration_mfma(workgroups, iterations, _ptr(sink), _stream()))


def ee_calibration_intake(own: torch.Tensor, common: torch.Tensor, workgroups: int, loads_in_flight: int, pairs: bool,
                          sink: torch.Tensor):
    _check(lib().ee_calibration_intake(_ptr(own), own.numel() * own.element_size(), _ptr(common),
                                       common.numel() * common.element_size(), workgroups, loads_in_flight, int(pairs),
                                       _ptr(sink), _stream()))


def ee_calibration_mfma_tile(workgroups: int, steps: int, lds_fragment_reads: int, sink: torch.Tensor):
    assert sink.dtype == torch.float32 and sink.numel() >= 256
    _check(lib().ee_calibration_mfma_tile(workgroups, steps, lds_fragment_reads, _ptr(sink), _stream()))
