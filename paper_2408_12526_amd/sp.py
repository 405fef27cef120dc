"""Thin binding over libsp_mi355x.so (the C ABI declared in include/sp.h).

Only argument marshalling happens here: torch supplies device memory and the
current stream, every step of the forward runs in the library's HIP kernels.
There is no fallback: importing this module without the built library, or
calling it without a GPU, raises.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libsp_mi355x.so")

SP_DTYPE_FP32, SP_DTYPE_BF16, SP_DTYPE_FP8 = 0, 1, 2
ACT_QUANT_SCALE = 16.0      # fp8 activations hold e4m3(16 * value)
SP_BAD_ID, SP_BAD_CU0, SP_BAD_ORDER, SP_BAD_LENGTH, SP_BAD_TOTAL = 1, 2, 4, 8, 16
PHASES = ("embed", "qkv", "attention", "oproj", "layernorm", "ffn_up", "ffn_down", "head", "last_first")


class sp_config(C.Structure):
    _fields_ = [(n, C.c_int32) for n in
                ("K", "layers", "hidden", "heads", "ffn", "vocab", "max_pos", "classes", "dtype")] + [
        ("ln_eps", C.c_float), ("last_layer_all_tokens", C.c_int32), ("single_stream", C.c_int32)]


class sp_ws_layout(C.Structure):
    _fields_ = [(n, C.c_size_t) for n in ("x", "qkv", "vt", "att", "x1", "g", "z")] + [
        ("rows", C.c_int32), ("act_bytes", C.c_int32), ("first_q", C.c_size_t), ("first_att", C.c_size_t),
        ("first_rows", C.c_int32), ("xq", C.c_size_t), ("x1q", C.c_size_t), ("gq", C.c_size_t), ("attq", C.c_size_t)]


def _load() -> C.CDLL:
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is missing: run `python -m paper_2408_12526_amd.build` (there is no fallback path)")
    lib = C.CDLL(LIB_PATH)
    vp, i32, sz = C.c_void_p, C.c_int32, C.c_size_t
    cfgp = C.POINTER(sp_config)
    lib.sp_blob_floats.restype = sz; lib.sp_blob_floats.argtypes = [cfgp]
    lib.sp_arena_bytes.restype = sz; lib.sp_arena_bytes.argtypes = [cfgp]
    lib.sp_workspace_bytes.restype = sz; lib.sp_workspace_bytes.argtypes = [cfgp, i32, i32]
    lib.sp_load_students.restype = C.c_int
    lib.sp_load_students.argtypes = [cfgp, vp, sz, vp, sz, vp, C.POINTER(vp)]
    lib.sp_forward.restype = C.c_int
    lib.sp_forward.argtypes = [vp, vp, vp, i32, i32, i32, i32, vp, sz, vp, vp]
    lib.sp_forward_static.restype = C.c_int
    lib.sp_forward_static.argtypes = [vp, vp, vp, i32, i32, i32, i32, vp, vp]
    lib.sp_static_scratch_bytes.restype = sz; lib.sp_static_scratch_bytes.argtypes = []
    lib.sp_forward_partial.restype = C.c_int
    lib.sp_forward_partial.argtypes = [vp, vp, vp, i32, i32, i32, i32, i32, vp, sz, vp]
    lib.sp_forward_profiled.restype = C.c_int
    lib.sp_forward_profiled.argtypes = [vp, vp, vp, i32, i32, i32, i32, vp, sz, vp, vp, vp]
    lib.sp_probe_gelu.restype = C.c_int; lib.sp_probe_gelu.argtypes = [vp, vp, C.c_int64, vp]
    lib.sp_probe_gelu_fp8.restype = C.c_int; lib.sp_probe_gelu_fp8.argtypes = [vp, vp, C.c_int64, vp]
    lib.sp_probe_e4m3.restype = C.c_int; lib.sp_probe_e4m3.argtypes = [vp, C.c_int64, vp]
    lib.sp_probe_mfma_rate.restype = C.c_int
    lib.sp_probe_mfma_rate.argtypes = [i32, i32, vp, vp, C.POINTER(C.c_float)]
    lib.sp_free.restype = None; lib.sp_free.argtypes = [vp]
    lib.sp_strerror.restype = C.c_char_p; lib.sp_strerror.argtypes = [C.c_int]
    lib.sp_pack.restype = C.c_int; lib.sp_pack.argtypes = [vp, i32, vp]
    lib.sp_check_inputs.restype = C.c_int
    lib.sp_check_inputs.argtypes = [vp, vp, vp, i32, i32, i32, vp, vp, C.POINTER(C.c_int32)]
    lib.sp_workspace_layout.restype = C.c_int
    lib.sp_workspace_layout.argtypes = [cfgp, i32, i32, C.POINTER(sp_ws_layout)]
    return lib


_lib = _load()


class SpError(RuntimeError):
    def __init__(self, code: int):
        self.code = code
        super().__init__(f"sp error {code}: {_lib.sp_strerror(code).decode()}")


def _check(rc: int) -> None:
    if rc != 0:
        raise SpError(rc)


def make_config(K, layers, hidden, heads, ffn, vocab, max_pos, classes, dtype="bf16", ln_eps=1e-12,
                last_layer_all_tokens=False, single_stream=False) -> sp_config:
    return sp_config(K, layers, hidden, heads, ffn, vocab, max_pos, classes,
                     {"bf16": SP_DTYPE_BF16, "fp8": SP_DTYPE_FP8, "fp32": SP_DTYPE_FP32}[dtype], ln_eps, 1 if last_layer_all_tokens else 0,
                     1 if single_stream else 0)


def config_from_shape(shape, last_layer_all_tokens=False, single_stream=False) -> sp_config:
    """shape: any object with the StudentShape fields (see synth.py)."""
    return make_config(shape.K, shape.layers, shape.hidden, shape.heads, shape.ffn, shape.vocab, shape.max_pos,
                       shape.classes, shape.dtype, shape.ln_eps, last_layer_all_tokens, single_stream)


def sp_blob_floats(cfg: sp_config) -> int:
    return int(_lib.sp_blob_floats(C.byref(cfg)))


def sp_arena_bytes(cfg: sp_config) -> int:
    return int(_lib.sp_arena_bytes(C.byref(cfg)))


def sp_workspace_bytes(cfg: sp_config, max_tokens: int, max_batch: int) -> int:
    return int(_lib.sp_workspace_bytes(C.byref(cfg), max_tokens, max_batch))


def sp_static_scratch_bytes() -> int:
    return int(_lib.sp_static_scratch_bytes())


def sp_probe_gelu(x: torch.Tensor) -> torch.Tensor:
    """The bf16 path's GELU evaluated in fp32 on a float32 device tensor (test aid)."""
    assert x.dtype == torch.float32 and x.is_cuda and x.is_contiguous()
    y = torch.empty_like(x)
    _check(_lib.sp_probe_gelu(x.data_ptr(), y.data_ptr(), x.numel(), _stream_ptr(None)))
    return y


def sp_probe_gelu_fp8(x: torch.Tensor) -> torch.Tensor:
    """The fp8 path's GELU evaluated in fp32 on a float32 device tensor, before scaling and rounding (test aid)."""
    assert x.dtype == torch.float32 and x.is_cuda and x.is_contiguous()
    y = torch.empty_like(x)
    _check(_lib.sp_probe_gelu_fp8(x.data_ptr(), y.data_ptr(), x.numel(), _stream_ptr(None)))
    return y


def sp_probe_e4m3(x: np.ndarray) -> np.ndarray:
    """e4m3 codes (uint8) the fp8 weight loader gives the float32 values x (host only)."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    out = np.empty(x.size, dtype=np.uint8)
    _check(_lib.sp_probe_e4m3(x.ctypes.data, x.size, out.ctypes.data))
    return out.reshape(x.shape)


def sp_probe_mfma_rate(operand_kind: int, milliseconds: int = 200) -> float:
    """Sustained TFLOP/s of a pure bf16 matrix-instruction loop (0: operands in {0, 1}; 1: random mantissas)."""
    scratch = torch.zeros(16, dtype=torch.float32, device="cuda")
    out = C.c_float()
    _check(_lib.sp_probe_mfma_rate(operand_kind, milliseconds, scratch.data_ptr(), _stream_ptr(None), C.byref(out)))
    return float(out.value)


def sp_pack(lengths) -> np.ndarray:
    lengths = np.ascontiguousarray(lengths, dtype=np.int32)
    cu = np.zeros(lengths.size + 1, dtype=np.int32)
    _check(_lib.sp_pack(lengths.ctypes.data, lengths.size, cu.ctypes.data))
    return cu


def sp_workspace_layout(cfg: sp_config, total_tokens: int, batch: int) -> sp_ws_layout:
    out = sp_ws_layout()
    _check(_lib.sp_workspace_layout(C.byref(cfg), total_tokens, batch, C.byref(out)))
    return out


def _stream_ptr(stream) -> int:
    s = stream if stream is not None else torch.cuda.current_stream()
    return int(s.cuda_stream)


class Students:
    """A loaded student group: owns the device arena tensor and the library handle."""

    def __init__(self, cfg: sp_config, blob: np.ndarray, device="cuda:0"):
        if not torch.cuda.is_available():
            raise RuntimeError("sp_load_students needs a GPU: there is no CPU path in this library")
        blob = np.ascontiguousarray(blob, dtype=np.float32)
        self.cfg = cfg
        self.device = torch.device(device)
        self.arena = torch.empty(sp_arena_bytes(cfg), dtype=torch.uint8, device=self.device)
        handle = C.c_void_p()
        with torch.cuda.device(self.device):
            _check(_lib.sp_load_students(C.byref(cfg), blob.ctypes.data, blob.size, self.arena.data_ptr(),
                                         self.arena.numel(), _stream_ptr(None), C.byref(handle)))
        self.handle = handle
        self._ws = None

    def workspace(self, total_tokens: int, batch: int) -> torch.Tensor:
        need = sp_workspace_bytes(self.cfg, total_tokens, batch)
        if self._ws is None or self._ws.numel() < need:
            self._ws = torch.empty(need, dtype=torch.uint8, device=self.device)
        return self._ws

    def release_workspace(self) -> None:
        """Drop the cached workspace tensor (the next call that needs one allocates it again)."""
        self._ws = None

    def sp_forward(self, token_ids: torch.Tensor, cu_seqlens: torch.Tensor, max_seqlen: int, k_active: int,
                   logits_out: torch.Tensor | None = None, workspace: torch.Tensor | None = None, stream=None):
        """token_ids int32 [T], cu_seqlens int32 [B+1] (device).  Returns logits_out (float32 [B, C])."""
        assert token_ids.dtype == torch.int32 and cu_seqlens.dtype == torch.int32
        assert token_ids.is_cuda and cu_seqlens.is_cuda and token_ids.is_contiguous() and cu_seqlens.is_contiguous()
        batch, total = cu_seqlens.numel() - 1, token_ids.numel()
        if logits_out is None:
            logits_out = torch.empty(batch, self.cfg.classes, dtype=torch.float32, device=self.device)
        ws = workspace if workspace is not None else self.workspace(total, batch)
        _check(_lib.sp_forward(self.handle, token_ids.data_ptr(), cu_seqlens.data_ptr(), batch, total, max_seqlen,
                               k_active, ws.data_ptr(), ws.numel(), logits_out.data_ptr(), _stream_ptr(stream)))
        return logits_out

    def sp_forward_static(self, token_ids: torch.Tensor, cu_seqlens: torch.Tensor, max_seqlen: int, k_active: int,
                          logits_out: torch.Tensor, stream=None):
        """sp_forward on the library's static workspace: nothing is allocated (logits_out must be given)."""
        assert token_ids.dtype == torch.int32 and cu_seqlens.dtype == torch.int32
        assert token_ids.is_cuda and cu_seqlens.is_cuda and token_ids.is_contiguous() and cu_seqlens.is_contiguous()
        assert logits_out.dtype == torch.float32 and logits_out.is_cuda and logits_out.is_contiguous()
        batch, total = cu_seqlens.numel() - 1, token_ids.numel()
        _check(_lib.sp_forward_static(self.handle, token_ids.data_ptr(), cu_seqlens.data_ptr(), batch, total, max_seqlen,
                                      k_active, logits_out.data_ptr(), _stream_ptr(stream)))
        return logits_out

    def sp_check_inputs(self, token_ids: torch.Tensor, cu_seqlens: torch.Tensor, max_seqlen: int, stream=None) -> int:
        """Bit set of SP_BAD_* problems found in the device-resident inputs of a forward (0: none).  Blocks."""
        scratch = torch.empty(64, dtype=torch.int32, device=self.device)
        out = C.c_int32()
        _check(_lib.sp_check_inputs(self.handle, token_ids.data_ptr(), cu_seqlens.data_ptr(), cu_seqlens.numel() - 1,
                                    token_ids.numel(), max_seqlen, scratch.data_ptr(), _stream_ptr(stream),
                                    C.byref(out)))
        return out.value

    def sp_forward_profiled(self, token_ids, cu_seqlens, max_seqlen, k_active, logits_out=None, workspace=None,
                            stream=None) -> dict:
        """One forward with per-phase device times (ms), as {phase name: ms}."""
        batch, total = cu_seqlens.numel() - 1, token_ids.numel()
        if logits_out is None:
            logits_out = torch.empty(batch, self.cfg.classes, dtype=torch.float32, device=self.device)
        ws = workspace if workspace is not None else self.workspace(total, batch)
        ms = (C.c_float * len(PHASES))()
        _check(_lib.sp_forward_profiled(self.handle, token_ids.data_ptr(), cu_seqlens.data_ptr(), batch, total,
                                        max_seqlen, k_active, ws.data_ptr(), ws.numel(), logits_out.data_ptr(),
                                        _stream_ptr(stream), C.cast(ms, C.c_void_p)))
        return {n: float(ms[i]) for i, n in enumerate(PHASES)}

    def sp_forward_partial(self, token_ids, cu_seqlens, max_seqlen, k_active, stop_after_layers, workspace=None,
                           stream=None):
        batch, total = cu_seqlens.numel() - 1, token_ids.numel()
        ws = workspace if workspace is not None else self.workspace(total, batch)
        _check(_lib.sp_forward_partial(self.handle, token_ids.data_ptr(), cu_seqlens.data_ptr(), batch, total,
                                       max_seqlen, k_active, stop_after_layers, ws.data_ptr(), ws.numel(),
                                       _stream_ptr(stream)))
        return ws

    def read_activation(self, ws: torch.Tensor, name: str, total_tokens: int, batch: int, k_active: int) -> np.ndarray:
        """Copy one intermediate tensor out of a workspace as float64 [k][T][width] (tests / profiling)."""
        lay = sp_workspace_layout(self.cfg, total_tokens, batch)
        H, F = self.cfg.hidden, self.cfg.ffn
        if name == "z":
            n = self.cfg.K * batch * self.cfg.classes
            z = ws[lay.z:lay.z + 4 * n].view(torch.float32).view(self.cfg.K, batch, self.cfg.classes)
            return z[:k_active].double().cpu().numpy()
        if name in ("first_q", "first_att"):        # compact rows of the first-token last layer: [k][batch][H]
            off, dt = getattr(lay, name), (torch.bfloat16 if lay.act_bytes == 2 else torch.float32)
            n = k_active * lay.first_rows * H
            t = ws[off:off + n * lay.act_bytes].view(dt).view(k_active, lay.first_rows, H)
            return t[:, :batch].double().cpu().numpy()
        if name in ("xq", "x1q", "gq", "attq"):              # fp8 activations: e4m3 codes of 16 * value, [k][rows][width] bytes
            width, off = (F if name == "gq" else H), getattr(lay, name)
            n = k_active * lay.rows * width
            t = ws[off:off + n].view(torch.float8_e4m3fn).view(k_active, lay.rows, width)
            return (t[:, :total_tokens].float().double() / ACT_QUANT_SCALE).cpu().numpy()
        width = {"x": H, "qkv": 3 * H, "att": H, "x1": H, "g": F}[name]
        off = getattr(lay, name)
        dt = torch.bfloat16 if lay.act_bytes == 2 else torch.float32
        n = k_active * lay.rows * width
        t = ws[off:off + n * lay.act_bytes].view(dt).view(k_active, lay.rows, width)
        t = t[:, :total_tokens].double()
        if name == "qkv" and lay.act_bytes == 2:      # bf16 mode keeps the values feature-major in `vt`
            nv = k_active * H * lay.rows
            vt = ws[lay.vt:lay.vt + nv * 2].view(dt).view(k_active, H, lay.rows)
            t = t.clone()
            t[:, :, 2 * H:] = vt[:, :, :total_tokens].double().transpose(1, 2)
        return t.cpu().numpy()

    def close(self):
        if self.handle:
            _lib.sp_free(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def raw_lib() -> C.CDLL:
    """The ctypes handle itself, for tests of the error paths."""
    return _lib
