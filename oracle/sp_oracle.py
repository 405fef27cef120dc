"""ctypes door to the CPU oracle (sp_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, the smoke check and the
benchmark's cpu_baseline leg.  Nothing here touches the HIP path, and the HIP
path never imports this module.

Two builds of the same source are exposed: ``Oracle("f64")`` (double
arithmetic, the reference for parity) and ``Oracle("f32")`` (float arithmetic,
the naive fp32 forward timed as the CPU baseline).
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "sp_oracle.c")
_LIBS = {"f64": os.path.join(_HERE, "libsp_oracle_f64.so"), "f32": os.path.join(_HERE, "libsp_oracle_f32.so")}


def build(force: bool = False) -> None:
    """Compile both oracle builds with gcc (plain C, OpenMP over student x sequence)."""
    for kind, lib in _LIBS.items():
        if not force and os.path.exists(lib) and os.path.getmtime(lib) >= os.path.getmtime(_SRC):
            continue
        cmd = ["gcc", "-O3", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-Wall", "-Wno-maybe-uninitialized", "-o", lib, _SRC, "-lm"]
        if kind == "f32":
            cmd.insert(1, "-DSPO_REAL_FLOAT")
        subprocess.run(cmd, check=True)


class _Cfg(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("K", "layers", "hidden", "heads", "ffn", "vocab", "max_pos", "classes")] + [
        ("ln_eps", C.c_double)
    ]


@dataclass(frozen=True)
class OracleConfig:
    K: int
    layers: int
    hidden: int
    heads: int
    ffn: int
    vocab: int
    max_pos: int
    classes: int
    ln_eps: float = 1e-12

    def c(self) -> _Cfg:
        return _Cfg(self.K, self.layers, self.hidden, self.heads, self.ffn, self.vocab, self.max_pos, self.classes,
                    self.ln_eps)


def _dp(a):
    return a.ctypes.data_as(C.POINTER(C.c_double)) if a is not None else None


def _fp(a):
    return a.ctypes.data_as(C.POINTER(C.c_float))


def _ip(a):
    return a.ctypes.data_as(C.POINTER(C.c_int32))


class Oracle:
    def __init__(self, kind: str = "f64"):
        build()
        self.kind = kind
        self.lib = C.CDLL(_LIBS[kind])
        L = self.lib
        L.spo_blob_floats.restype = C.c_size_t
        L.spo_blob_floats.argtypes = [C.POINTER(_Cfg)]
        L.spo_real_bytes.restype = C.c_int
        L.spo_gelu.restype = C.c_double
        L.spo_gelu.argtypes = [C.c_double]
        L.spo_pack.restype = C.c_int
        L.spo_forward.restype = C.c_int
        L.spo_forward_taps.restype = C.c_int
        assert L.spo_real_bytes() == (8 if kind == "f64" else 4)

    # -- geometry / packing -------------------------------------------------
    def blob_floats(self, cfg: OracleConfig) -> int:
        c = cfg.c()
        return int(self.lib.spo_blob_floats(C.byref(c)))

    def pack(self, lengths) -> np.ndarray:
        lengths = np.ascontiguousarray(lengths, dtype=np.int32)
        cu = np.zeros(len(lengths) + 1, dtype=np.int32)
        rc = self.lib.spo_pack(_ip(lengths), C.c_int32(len(lengths)), _ip(cu))
        if rc:
            raise ValueError("spo_pack rejected the lengths")
        return cu

    # -- whole forward --------------------------------------------------------
    def forward(self, cfg: OracleConfig, blob: np.ndarray, ids, cu, k_active: int, want_terms=False, want_pooled=False):
        blob = np.ascontiguousarray(blob, dtype=np.float32)
        assert blob.size == self.blob_floats(cfg), "blob size does not match the configuration"
        ids = np.ascontiguousarray(ids, dtype=np.int32)
        cu = np.ascontiguousarray(cu, dtype=np.int32)
        B = len(cu) - 1
        assert ids.size == cu[-1]
        logits = np.zeros((B, cfg.classes))
        z = np.zeros((k_active, B, cfg.classes)) if want_terms else None
        pl = np.zeros((k_active, B, cfg.hidden)) if want_pooled else None
        c = cfg.c()
        rc = self.lib.spo_forward(C.byref(c), _fp(blob), _ip(ids), _ip(cu), C.c_int32(B), C.c_int32(k_active),
                                  _dp(logits), _dp(z), _dp(pl))
        if rc:
            raise ValueError(f"spo_forward argument error {rc}")
        out = [logits]
        if want_terms:
            out.append(z)
        if want_pooled:
            out.append(pl)
        return out[0] if len(out) == 1 else tuple(out)

    def taps(self, cfg: OracleConfig, blob: np.ndarray, ids, cu, m: int, b: int) -> dict:
        blob = np.ascontiguousarray(blob, dtype=np.float32)
        ids = np.ascontiguousarray(ids, dtype=np.int32)
        cu = np.ascontiguousarray(cu, dtype=np.int32)
        B = len(cu) - 1
        L = int(cu[b + 1] - cu[b])
        H, F, Ly = cfg.hidden, cfg.ffn, cfg.layers
        t = dict(x0=np.zeros((L, H)), qkv=np.zeros((Ly, L, 3 * H)), att=np.zeros((Ly, L, H)), x1=np.zeros((Ly, L, H)),
                 g=np.zeros((Ly, L, F)), x2=np.zeros((Ly, L, H)), z=np.zeros(cfg.classes))
        c = cfg.c()
        rc = self.lib.spo_forward_taps(C.byref(c), _fp(blob), _ip(ids), _ip(cu), C.c_int32(B), C.c_int32(m),
                                       C.c_int32(b), _dp(t["x0"]), _dp(t["qkv"]), _dp(t["att"]), _dp(t["x1"]),
                                       _dp(t["g"]), _dp(t["x2"]), _dp(t["z"]))
        if rc:
            raise ValueError(f"spo_forward_taps argument error {rc}")
        return t

    # -- elementary pieces (for the pins) -------------------------------------
    def layernorm(self, u, g, b, eps):
        u = np.ascontiguousarray(u, dtype=np.float64)
        g = np.ascontiguousarray(g, dtype=np.float32)
        b = np.ascontiguousarray(b, dtype=np.float32)
        out = np.zeros_like(u)
        self.lib.spo_layernorm(_dp(u), _fp(g), _fp(b), C.c_int(u.size), C.c_double(eps), _dp(out))
        return out

    def gelu(self, u: float) -> float:
        return float(self.lib.spo_gelu(C.c_double(u)))

    def softmax(self, s):
        s = np.array(s, dtype=np.float64)
        self.lib.spo_softmax(_dp(s), C.c_int(s.size))
        return s

    def linear(self, x, W, b):
        x = np.ascontiguousarray(x, dtype=np.float64)
        W = np.ascontiguousarray(W, dtype=np.float32)
        b = np.ascontiguousarray(b, dtype=np.float32)
        L, n_in = x.shape
        n_out = W.shape[1]
        assert W.shape[0] == n_in and b.size == n_out
        y = np.zeros((L, n_out))
        self.lib.spo_linear(_dp(x), C.c_int(L), C.c_int(n_in), C.c_int(n_out), _fp(W), _fp(b), _dp(y))
        return y

    def attention(self, q, k, v, heads: int, want_probs=False):
        q = np.ascontiguousarray(q, dtype=np.float64)
        k = np.ascontiguousarray(k, dtype=np.float64)
        v = np.ascontiguousarray(v, dtype=np.float64)
        L, H = q.shape
        d = H // heads
        o = np.zeros((L, H))
        p = np.zeros((heads, L, L)) if want_probs else None
        self.lib.spo_attention(_dp(q), _dp(k), _dp(v), C.c_int(L), C.c_int(heads), C.c_int(d), _dp(o), _dp(p))
        return (o, p) if want_probs else o

    def encoder_layer(self, x, heads: int, ffn: int, layer_blob, eps: float):
        x = np.ascontiguousarray(x, dtype=np.float64)
        lw = np.ascontiguousarray(layer_blob, dtype=np.float32)
        L, H = x.shape
        out = np.zeros((L, H))
        self.lib.spo_encoder_layer(_dp(x), C.c_int(L), C.c_int(H), C.c_int(heads), C.c_int(ffn), _fp(lw),
                                   C.c_double(eps), _dp(out))
        return out
