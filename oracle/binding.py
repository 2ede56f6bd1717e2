"""ctypes access to the C oracle (oracle/spark_oracle.c).  TEST INFRASTRUCTURE ONLY.

Only tests, the smoke check and the benchmark's CPU-baseline leg import this module.  It takes
model shapes, schedules and weight dictionaries from the shared input generators and marshals
them; all arithmetic happens in the C file.
"""
from __future__ import annotations

import ctypes as C
import pathlib

import numpy as np

HERE = pathlib.Path(__file__).resolve().parent


class OraConfig(C.Structure):
    _fields_ = [(n, C.c_int32) for n in
                ("n_layers", "d_model", "n_q_heads", "n_kv_heads", "head_dim", "d_ffn",
                 "vocab_text", "vocab_speech")] + \
               [("rope_base", C.c_float), ("rms_eps", C.c_float)] + \
               [(n, C.c_int32) for n in
                ("dtype", "exit_layer", "period_k", "phase", "scope", "n_text", "n_speech",
                 "max_seq_len", "kv_round_bf16", "text_period_k", "text_phase")]


WEIGHT_FIELDS = ("embed", "attn_norm", "wq", "wk", "wv", "wo", "mlp_norm", "wg", "wu", "wd",
                 "final_norm", "lm_head", "lens_a", "lens_b", "lens_norm", "lens_head")


class OraWeights(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in WEIGHT_FIELDS]


_libs: dict[str, C.CDLL] = {}


def load(kind: str = "f32") -> C.CDLL:
    if kind in _libs:
        return _libs[kind]
    path = HERE / f"liboracle_{kind}.so"
    if not path.exists():
        from . import build_oracle
        build_oracle.build()
    lib = C.CDLL(str(path))
    P, I = C.c_void_p, C.c_int
    lib.ora_create.restype = P
    lib.ora_create.argtypes = [C.POINTER(OraConfig), C.POINTER(OraWeights)]
    lib.ora_destroy.argtypes = [P]
    lib.ora_seq_open.restype = P
    lib.ora_seq_open.argtypes = [P, I]
    lib.ora_seq_close.argtypes = [P]
    lib.ora_prefill.argtypes = [P, P, I]
    lib.ora_step.argtypes = [P, I, P, P, P]
    lib.ora_step_standard.argtypes = [P, I, P, P, I, P]
    lib.ora_schedule_run.argtypes = [C.POINTER(OraConfig), I, I, P, P]
    lib.ora_schedule_run_budget.argtypes = [C.POINTER(OraConfig), I, I, I, P, P]
    lib.ora_seq_text_budget.argtypes = [P, I]
    lib.ora_seq_set_phase.argtypes = [P, I]
    lib.ora_schedule_run_moves.argtypes = [C.POINTER(OraConfig), I, I, I, I, P, P, P, P]
    lib.ora_seq_j_stream.argtypes = [P]
    lib.ora_layer_saving.restype = C.c_double
    lib.ora_layer_saving.argtypes = [P, I, I]
    for f in ("ora_seq_len", "ora_seq_upper_valid", "ora_seq_pending"):
        getattr(lib, f).argtypes = [P]
    lib.ora_seq_stats.argtypes = [P, P]
    lib.ora_pend_cap.argtypes = [C.POINTER(OraConfig)]
    lib.ora_sample.argtypes = [P, C.c_int, C.c_double, C.c_double, C.c_uint64, C.POINTER(C.c_int32),
                               C.POINTER(C.c_double)]
    lib.ora_get_kv.argtypes = [P, I, I, P, P]
    lib.ora_lens_logits.argtypes = [P, P, P]
    lib.ora_prim_matvec.argtypes = [P, I, I, I, P, P]
    lib.ora_prim_rmsnorm.argtypes = [P, P, I, C.c_double, P]
    lib.ora_prim_rope.argtypes = [P, I, I, C.c_double]
    lib.ora_prim_silu.restype = C.c_double
    lib.ora_prim_silu.argtypes = [C.c_double]
    lib.ora_prim_attend.argtypes = [P, P, P, I, I, P]
    lib.ora_prim_argmax.argtypes = [P, I]
    lib.ora_prim_bf16_round.restype = C.c_double
    lib.ora_prim_bf16_round.argtypes = [C.c_double]
    lib.ora_num_threads.argtypes = []
    _libs[kind] = lib
    return lib


def num_threads(kind: str = "f32") -> int:
    return int(load(kind).ora_num_threads())


def _ptr(a: np.ndarray) -> C.c_void_p:
    return C.c_void_p(a.ctypes.data)


def make_config(shape, sched, max_seq_len: int, kv_round_bf16: bool = False) -> OraConfig:
    return OraConfig(shape.n_layers, shape.d_model, shape.n_q_heads, shape.n_kv_heads,
                     shape.head_dim, shape.d_ffn, shape.vocab_text, shape.vocab_speech,
                     shape.rope_base, shape.rms_eps, shape.dtype, sched.exit_layer,
                     sched.period_k, sched.phase, sched.scope, sched.n_text, sched.n_speech,
                     max_seq_len, int(kv_round_bf16), sched.text_period_k, sched.text_phase)


def sample(logits, temperature: float, top_p: float, omega: int, kind: str = "f32"):
    """(token, nucleus size, gap) of the oracle's nucleus sampler for one vector of logits"""
    lib = load(kind)
    lg = np.ascontiguousarray(logits, dtype=np.float64)
    n, gap = C.c_int32(0), C.c_double(0.0)
    tok = lib.ora_sample(_ptr(lg), len(lg), temperature, top_p, C.c_uint64(omega), C.byref(n), C.byref(gap))
    return tok, n.value, gap.value


def schedule_run(shape, sched, n_steps: int, cycle_offset: int = 0, kind: str = "f32", text_budget: int = 0):
    """(depth[n], is_text[n]) from the oracle's scheduler alone; None if the config is refused."""
    lib = load(kind)
    cfg = make_config(shape, sched, 1)
    depth = np.zeros(n_steps, dtype=np.int32)
    is_text = np.zeros(n_steps, dtype=np.int32)
    rc = lib.ora_schedule_run_budget(C.byref(cfg), cycle_offset, text_budget, n_steps, _ptr(depth), _ptr(is_text))
    if rc != 0:
        return None
    return depth, is_text


def schedule_run_moves(shape, sched, n_steps: int, moves, cycle_offset: int = 0, text_budget: int = 0,
                       kind: str = "f32"):
    """schedule_run with the speech phase moved on the way: moves = [(step, phase), ...], ascending"""
    lib = load(kind)
    cfg = make_config(shape, sched, 1)
    depth = np.zeros(n_steps, dtype=np.int32)
    is_text = np.zeros(n_steps, dtype=np.int32)
    ms = np.array([m[0] for m in moves], dtype=np.int32)
    mp = np.array([m[1] for m in moves], dtype=np.int32)
    rc = lib.ora_schedule_run_moves(C.byref(cfg), cycle_offset, text_budget, n_steps, len(moves), _ptr(ms), _ptr(mp),
                                    _ptr(depth), _ptr(is_text))
    return (depth, is_text) if rc == 0 else None


def layer_saving(depth: np.ndarray, n_layers: int, kind: str = "f32") -> float:
    d = np.ascontiguousarray(depth, dtype=np.int32)
    return float(load(kind).ora_layer_saving(_ptr(d), len(d), n_layers))


class Model:
    """One oracle model: config + borrowed weight arrays (kept alive here)."""

    def __init__(self, shape, sched, weights: dict, max_seq_len: int, kind: str = "f32",
                 kv_round_bf16: bool = False):
        self.lib = load(kind)
        self.shape, self.sched = shape, sched
        self.cfg = make_config(shape, sched, max_seq_len, kv_round_bf16)
        self._keep = {k: np.ascontiguousarray(v) for k, v in weights.items()}
        w = OraWeights(*[_ptr(self._keep[n]) for n in WEIGHT_FIELDS])
        self.handle = self.lib.ora_create(C.byref(self.cfg), C.byref(w))
        if not self.handle:
            raise ValueError("oracle refused the configuration")
        self.vocab = shape.vocab

    def close(self):
        if self.handle:
            self.lib.ora_destroy(self.handle)
            self.handle = None

    def open(self, cycle_offset: int = 0) -> "Seq":
        return Seq(self, cycle_offset)

    def lens_logits(self, h: np.ndarray) -> np.ndarray:
        h = np.ascontiguousarray(h, dtype=np.float64)
        out = np.zeros(self.vocab, dtype=np.float64)
        rc = self.lib.ora_lens_logits(self.handle, _ptr(h), _ptr(out))
        assert rc == 0
        return out


class Seq:
    def __init__(self, model: Model, cycle_offset: int):
        self.m = model
        self.lib = model.lib
        self.handle = self.lib.ora_seq_open(model.handle, cycle_offset)
        if not self.handle:
            raise MemoryError("oracle sequence")

    def set_phase(self, phase: int) -> int:
        """move the sequence's phase on speech positions"""
        return self.lib.ora_seq_set_phase(self.handle, phase)

    @property
    def j_stream(self) -> int:
        return self.lib.ora_seq_j_stream(self.handle)

    def text_budget(self, budget: int) -> int:
        """after `budget` text tokens in all the sequence generates speech only"""
        return self.lib.ora_seq_text_budget(self.handle, budget)

    def close(self):
        if self.handle:
            self.lib.ora_seq_close(self.handle)
            self.handle = None

    def prefill(self, prompt) -> int:
        p = np.ascontiguousarray(prompt, dtype=np.int32)
        return self.lib.ora_prefill(self.handle, _ptr(p), len(p))

    def step(self, forced_next: int = -1, want_logits: bool = True):
        """SPAR-K step -> (rc, token, depth, logits or None)"""
        tok, depth = C.c_int32(-1), C.c_int32(-1)
        logits = np.zeros(self.m.vocab, dtype=np.float64) if want_logits else None
        rc = self.lib.ora_step(self.handle, int(forced_next), C.byref(tok), C.byref(depth),
                               _ptr(logits) if want_logits else None)
        return rc, tok.value, depth.value, logits

    def step_standard(self, forced_next: int = -1, capture_layer: int = 0):
        """standard full-depth step -> (rc, token, logits, h at capture_layer or None)"""
        tok = C.c_int32(-1)
        logits = np.zeros(self.m.vocab, dtype=np.float64)
        hcap = np.zeros(self.m.shape.d_model, dtype=np.float64) if capture_layer else None
        rc = self.lib.ora_step_standard(self.handle, int(forced_next), C.byref(tok), _ptr(logits),
                                        capture_layer, _ptr(hcap) if capture_layer else None)
        return rc, tok.value, logits, hcap

    @property
    def len(self) -> int:
        return self.lib.ora_seq_len(self.handle)

    @property
    def upper_valid(self) -> int:
        return self.lib.ora_seq_upper_valid(self.handle)

    @property
    def pending(self) -> int:
        return self.lib.ora_seq_pending(self.handle)

    def stats(self) -> dict:
        cap = self.lib.ora_pend_cap(C.byref(self.m.cfg))
        out = np.zeros(3 + cap, dtype=np.int64)
        self.lib.ora_seq_stats(self.handle, _ptr(out))
        return {"text": int(out[0]), "speech_full": int(out[1]), "speech_ee": int(out[2]),
                "text_ee": int(out[2 + cap]),
                "flush_hist": {m: int(out[2 + m]) for m in range(1, cap) if out[2 + m]}}

    def kv(self, layer: int, pos: int):
        w = self.m.shape.n_kv_heads * self.m.shape.head_dim
        k, v = np.zeros(w), np.zeros(w)
        rc = self.lib.ora_get_kv(self.handle, layer, pos, _ptr(k), _ptr(v))
        assert rc == 0
        return k, v


# ---------------------------------------------------------------- primitive probes

def prim_matvec(w: np.ndarray, x: np.ndarray, kind="f32") -> np.ndarray:
    lib = load(kind)
    dtype = 1 if w.dtype == np.uint16 else 0
    w = np.ascontiguousarray(w)
    x = np.ascontiguousarray(x, dtype=np.float64)
    y = np.zeros(w.shape[0], dtype=np.float64)
    lib.ora_prim_matvec(_ptr(w), dtype, w.shape[0], w.shape[1], _ptr(x), _ptr(y))
    return y


def prim_rmsnorm(x, gamma, eps, kind="f32") -> np.ndarray:
    lib = load(kind)
    x = np.ascontiguousarray(x, dtype=np.float64)
    g = np.ascontiguousarray(gamma, dtype=np.float32)
    out = np.zeros_like(x)
    lib.ora_prim_rmsnorm(_ptr(x), _ptr(g), len(x), float(eps), _ptr(out))
    return out


def prim_rope(v, pos: int, base: float, kind="f32") -> np.ndarray:
    lib = load(kind)
    v = np.array(v, dtype=np.float64)
    lib.ora_prim_rope(_ptr(v), len(v), pos, float(base))
    return v


def prim_silu(x: float, kind="f32") -> float:
    return float(load(kind).ora_prim_silu(float(x)))


def prim_attend(q, k, v, kind="f32") -> np.ndarray:
    lib = load(kind)
    q = np.ascontiguousarray(q, dtype=np.float64)
    k = np.ascontiguousarray(k, dtype=np.float64)
    v = np.ascontiguousarray(v, dtype=np.float64)
    out = np.zeros(len(q), dtype=np.float64)
    lib.ora_prim_attend(_ptr(q), _ptr(k), _ptr(v), len(q), k.shape[0], _ptr(out))
    return out


def prim_argmax(x, kind="f32") -> int:
    x = np.ascontiguousarray(x, dtype=np.float64)
    return int(load(kind).ora_prim_argmax(_ptr(x), len(x)))


def prim_bf16_round(x: float, kind="f32") -> float:
    return float(load(kind).ora_prim_bf16_round(float(x)))
