"""Thin Python binding of the C ABI in include/spark.h: argument marshalling only.

PyTorch is used for device memory (weights, KV pool, scratch) and for the stream handle; every
step of the decode path runs inside libspark.so.  There is no fallback: if the library is missing
or no GPU is present, construction fails.
"""
from __future__ import annotations

import ctypes as C
import pathlib

import numpy as np

HERE = pathlib.Path(__file__).resolve().parent
LIB_PATH = HERE / "libspark.so"

SPARK_MAX_PERIOD = 16
KC = {"qkv": 0, "attn": 1, "oproj": 2, "gateup": 3, "down": 4, "lens": 5, "head": 6, "sample": 8}

ERRORS = {-1: "SPARK_EINVAL", -2: "SPARK_ENOSEQ", -3: "SPARK_ENOMEM", -4: "SPARK_ESTATE",
          -5: "SPARK_EHIP", -6: "SPARK_ENAN"}

EXPORTS = ("spark_workspace_bytes", "spark_init", "spark_seq_open", "spark_prefill", "spark_step",
           "spark_decode", "spark_get_logits", "spark_get_kv", "spark_seq_state",
           "spark_get_stats", "spark_seq_close", "spark_destroy", "spark_last_error",
           "spark_profile_select", "spark_profile_read", "spark_set_sampling", "spark_decode_sampled",
           "spark_seq_text_budget", "spark_schedule_preview", "spark_seq_set_phase", "spark_align_phases",
           "spark_init_static", "spark_tune", "spark_measure_read")


class SparkConfig(C.Structure):
    _fields_ = [("size", C.c_uint32)] + \
               [(n, C.c_int32) for n in ("n_layers", "d_model", "n_q_heads", "n_kv_heads",
                                         "head_dim", "d_ffn", "vocab_text", "vocab_speech")] + \
               [("rope_base", C.c_float), ("rms_eps", C.c_float)] + \
               [(n, C.c_int32) for n in ("dtype", "exit_layer", "period_k", "phase", "scope",
                                         "n_text", "n_speech", "max_batch", "max_seq_len",
                                         "kv_page_tokens", "text_period_k", "text_phase")]


WEIGHT_FIELDS = ("embed", "attn_norm", "wq", "wk", "wv", "wo", "mlp_norm", "wg", "wu", "wd",
                 "final_norm", "lm_head", "lens_a", "lens_b", "lens_norm", "lens_head")


class SparkWeights(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in WEIGHT_FIELDS]


class SparkStats(C.Structure):
    _fields_ = [("text_steps", C.c_int64), ("speech_full_steps", C.c_int64),
                ("speech_ee_steps", C.c_int64), ("flush_rows", C.c_int64 * (2 * SPARK_MAX_PERIOD)),
                ("mean_text_depth", C.c_double), ("mean_speech_depth", C.c_double),
                ("speech_layer_saving", C.c_double), ("text_ee_steps", C.c_int64)]


class SparkError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"{ERRORS.get(code, code)}: {msg}")
        self.code = code


_lib = None


def load_library() -> C.CDLL:
    """dlopen the in-tree library and declare the signatures; no GPU is touched."""
    global _lib
    if _lib is not None:
        return _lib
    if not LIB_PATH.exists():
        raise FileNotFoundError(f"{LIB_PATH} is not built: run paper_2603_09215_amd/build.py")
    lib = C.CDLL(str(LIB_PATH))
    P, I = C.c_void_p, C.c_int32
    lib.spark_workspace_bytes.argtypes = [C.POINTER(SparkConfig), C.POINTER(C.c_size_t),
                                          C.POINTER(C.c_size_t)]
    lib.spark_init.argtypes = [C.POINTER(SparkConfig), C.POINTER(SparkWeights), P, C.c_size_t, P,
                               C.c_size_t, P, C.POINTER(P)]
    lib.spark_init_static.argtypes = [C.POINTER(SparkConfig), C.POINTER(SparkWeights), P, C.c_size_t, P,
                                      C.POINTER(P)]
    lib.spark_tune.argtypes = [P, C.c_char_p, I]
    lib.spark_measure_read.argtypes = [P, P, C.c_size_t, I, I, C.POINTER(C.c_double), C.POINTER(C.c_uint32)]
    lib.spark_seq_open.argtypes = [P, I, C.POINTER(I)]
    lib.spark_prefill.argtypes = [P, I, P, I]
    lib.spark_step.argtypes = [P, I, P, P, P, P]
    lib.spark_decode.argtypes = [P, I, I, P, P, P, P]
    lib.spark_set_sampling.argtypes = [P, C.c_float, C.c_float]
    lib.spark_seq_text_budget.argtypes = [P, I, I]
    lib.spark_seq_set_phase.argtypes = [P, I, I]
    lib.spark_align_phases.argtypes = [P, I, P]
    lib.spark_schedule_preview.argtypes = [C.POINTER(SparkConfig), I, I, I, P, P]
    lib.spark_decode_sampled.argtypes = [P, I, I, P, P, P, P, P]
    lib.spark_get_logits.argtypes = [P, I, P, C.POINTER(I)]
    lib.spark_get_kv.argtypes = [P, I, I, I, P, P]
    lib.spark_seq_state.argtypes = [P, I, C.POINTER(I), C.POINTER(I), C.POINTER(I)]
    lib.spark_get_stats.argtypes = [P, I, C.POINTER(SparkStats)]
    lib.spark_seq_close.argtypes = [P, I]
    lib.spark_destroy.argtypes = [P]
    lib.spark_destroy.restype = None
    lib.spark_last_error.argtypes = [P]
    lib.spark_last_error.restype = C.c_char_p
    lib.spark_profile_select.argtypes = [P, I]
    lib.spark_profile_read.argtypes = [P, C.POINTER(C.c_int64), C.POINTER(C.c_double), C.POINTER(C.c_double)]
    _lib = lib
    return lib


def make_config(shape, sched, max_batch: int, max_seq_len: int, kv_page_tokens: int = 64) -> SparkConfig:
    return SparkConfig(C.sizeof(SparkConfig), shape.n_layers, shape.d_model, shape.n_q_heads,
                       shape.n_kv_heads, shape.head_dim, shape.d_ffn, shape.vocab_text,
                       shape.vocab_speech, shape.rope_base, shape.rms_eps, shape.dtype,
                       sched.exit_layer, sched.period_k, sched.phase, sched.scope, sched.n_text,
                       sched.n_speech, max_batch, max_seq_len, kv_page_tokens,
                       getattr(sched, "text_period_k", 0), getattr(sched, "text_phase", 0))


def schedule_preview(shape, sched, n_steps: int, cycle_offset: int = 0, text_budget: int = 0):
    """(depth[n], is_text[n]) from the library's own schedule function, on the host; None if the
    configuration is refused"""
    lib = load_library()
    cfg = make_config(shape, sched, 1, 64, 16)
    depth = np.zeros(n_steps, dtype=np.int32)
    is_text = np.zeros(n_steps, dtype=np.int32)
    rc = lib.spark_schedule_preview(C.byref(cfg), cycle_offset, text_budget, n_steps,
                                    C.c_void_p(depth.ctypes.data), C.c_void_p(is_text.ctypes.data))
    return (depth, is_text) if rc == 0 else None


def _iptr(a: np.ndarray):
    return C.c_void_p(a.ctypes.data)


def weights_to_device(weights: dict, device="cuda:0") -> dict:
    """numpy weight dictionary (uint16 = bf16 bit patterns, float32) -> torch device tensors"""
    import torch
    out = {}
    for k in WEIGHT_FIELDS:
        a = weights[k]
        if isinstance(a, np.ndarray):
            if a.dtype == np.uint16:
                t = torch.from_numpy(a.view(np.int16)).to(device).view(torch.bfloat16)
            else:
                t = torch.from_numpy(a).to(device)
        else:
            t = a.to(device)
        out[k] = t.contiguous()
    return out


class Spark:
    """One decoding context on the current CUDA/HIP device."""

    def __init__(self, shape, sched, weights: dict, max_batch: int = 1, max_seq_len: int = 2048,
                 kv_page_tokens: int = 64, device="cuda:0", stream=None, static_scratch: bool = False):
        import torch
        if not torch.cuda.is_available():
            raise RuntimeError("spark needs a GPU: no HIP device is visible")
        self.lib = load_library()
        self.shape, self.sched = shape, sched
        self.vocab = shape.vocab
        self.cfg = make_config(shape, sched, max_batch, max_seq_len, kv_page_tokens)
        self.handle = C.c_void_p()
        kv_b, sc_b = C.c_size_t(), C.c_size_t()
        rc = self.lib.spark_workspace_bytes(C.byref(self.cfg), C.byref(kv_b), C.byref(sc_b))
        if rc:
            raise SparkError(rc, "configuration refused")
        torch.cuda.set_device(device)
        self.dev_weights = weights_to_device(weights, device)
        self.kv_pool = torch.empty(max(kv_b.value, 256), dtype=torch.uint8, device=device)
        self.scratch_bytes = sc_b.value
        self.stream = stream if stream is not None else torch.cuda.current_stream()
        w = SparkWeights(*[self.dev_weights[n].data_ptr() for n in WEIGHT_FIELDS])
        torch.cuda.synchronize()
        if static_scratch:   # spark_init_static: the library's own scratch area, nothing allocated
            self.scratch = None
            rc = self.lib.spark_init_static(C.byref(self.cfg), C.byref(w), self.kv_pool.data_ptr(), kv_b.value,
                                            C.c_void_p(self.stream.cuda_stream), C.byref(self.handle))
        else:
            self.scratch = torch.empty(max(sc_b.value, 256), dtype=torch.uint8, device=device)
            rc = self.lib.spark_init(C.byref(self.cfg), C.byref(w), self.kv_pool.data_ptr(),
                                     kv_b.value, self.scratch.data_ptr(), sc_b.value,
                                     C.c_void_p(self.stream.cuda_stream), C.byref(self.handle))
        if rc:
            self.handle = C.c_void_p()
            raise SparkError(rc, "spark_init_static failed" if static_scratch else "spark_init failed")

    # -- helpers
    def _check(self, rc: int):
        if rc:
            raise SparkError(rc, self.lib.spark_last_error(self.handle).decode())

    def close(self):
        if self.handle:
            self.lib.spark_destroy(self.handle)
            self.handle = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # -- the ABI, one method per entry point
    def seq_open(self, cycle_offset: int = 0) -> int:
        sid = C.c_int32(-1)
        self._check(self.lib.spark_seq_open(self.handle, cycle_offset, C.byref(sid)))
        return sid.value

    def prefill(self, seq_id: int, prompt) -> None:
        p = np.ascontiguousarray(prompt, dtype=np.int32)
        self._check(self.lib.spark_prefill(self.handle, seq_id, _iptr(p), len(p)))

    def step(self, seq_ids, forced_next=None):
        ids = np.ascontiguousarray(seq_ids, dtype=np.int32)
        n = len(ids)
        f = None if forced_next is None else np.ascontiguousarray(forced_next, dtype=np.int32)
        tok = np.empty(n, dtype=np.int32)
        dep = np.empty(n, dtype=np.int32)
        self._check(self.lib.spark_step(self.handle, n, _iptr(ids), _iptr(f) if f is not None else None,
                                        _iptr(tok), _iptr(dep)))
        return tok, dep

    def decode(self, n_steps: int, seq_ids, forced_next=None):
        ids = np.ascontiguousarray(seq_ids, dtype=np.int32)
        n = len(ids)
        f = None
        if forced_next is not None:
            f = np.ascontiguousarray(forced_next, dtype=np.int32).reshape(n_steps, n)
        tok = np.empty((n_steps, n), dtype=np.int32)
        dep = np.empty((n_steps, n), dtype=np.int32)
        self._check(self.lib.spark_decode(self.handle, n_steps, n, _iptr(ids),
                                          _iptr(f) if f is not None else None, _iptr(tok), _iptr(dep)))
        return tok, dep

    def seq_text_budget(self, seq_id: int, n_text_tokens: int) -> None:
        self._check(self.lib.spark_seq_text_budget(self.handle, seq_id, n_text_tokens))

    def seq_set_phase(self, seq_id: int, phase: int) -> None:
        self._check(self.lib.spark_seq_set_phase(self.handle, seq_id, phase))

    def align_phases(self, seq_ids) -> None:
        ids = np.ascontiguousarray(seq_ids, dtype=np.int32)
        self._check(self.lib.spark_align_phases(self.handle, len(ids), _iptr(ids)))

    def set_sampling(self, temperature: float, top_p: float) -> None:
        self._check(self.lib.spark_set_sampling(self.handle, temperature, top_p))

    def decode_sampled(self, n_steps: int, seq_ids, rand_words, forced_next=None):
        ids = np.ascontiguousarray(seq_ids, dtype=np.int32)
        n = len(ids)
        f = None
        if forced_next is not None:
            f = np.ascontiguousarray(forced_next, dtype=np.int32).reshape(n_steps, n)
        rw = np.ascontiguousarray(rand_words, dtype=np.uint64).reshape(n_steps, n)
        tok = np.empty((n_steps, n), dtype=np.int32)
        dep = np.empty((n_steps, n), dtype=np.int32)
        self._check(self.lib.spark_decode_sampled(self.handle, n_steps, n, _iptr(ids),
                                                  _iptr(f) if f is not None else None, _iptr(rw),
                                                  _iptr(tok), _iptr(dep)))
        return tok, dep

    def get_logits(self, seq_id: int):
        out = np.empty(self.vocab, dtype=np.float32)
        head = C.c_int32(0)
        self._check(self.lib.spark_get_logits(self.handle, seq_id, _iptr(out), C.byref(head)))
        return out, head.value

    def get_kv(self, seq_id: int, layer: int, pos: int):
        w = self.shape.n_kv_heads * self.shape.head_dim
        k = np.empty(w, dtype=np.float32)
        v = np.empty(w, dtype=np.float32)
        self._check(self.lib.spark_get_kv(self.handle, seq_id, layer, pos, _iptr(k), _iptr(v)))
        return k, v

    def seq_state(self, seq_id: int):
        a, b, c = C.c_int32(), C.c_int32(), C.c_int32()
        self._check(self.lib.spark_seq_state(self.handle, seq_id, C.byref(a), C.byref(b), C.byref(c)))
        return {"len": a.value, "upper_valid": b.value, "pending": c.value}

    def get_stats(self, seq_id: int) -> dict:
        st = SparkStats()
        self._check(self.lib.spark_get_stats(self.handle, seq_id, C.byref(st)))
        return {"text": st.text_steps, "speech_full": st.speech_full_steps,
                "speech_ee": st.speech_ee_steps, "text_ee": st.text_ee_steps,
                "flush_hist": {m: int(st.flush_rows[m]) for m in range(2 * SPARK_MAX_PERIOD)
                               if st.flush_rows[m]},
                "mean_text_depth": st.mean_text_depth, "mean_speech_depth": st.mean_speech_depth,
                "speech_layer_saving": st.speech_layer_saving}

    def seq_close(self, seq_id: int) -> None:
        self._check(self.lib.spark_seq_close(self.handle, seq_id))

    def profile_select(self, kernel_class) -> None:
        k = KC[kernel_class] if isinstance(kernel_class, str) else int(kernel_class)
        self._check(self.lib.spark_profile_select(self.handle, k))

    def profile_read(self):
        """(bracketed launches, their summed duration in ms, summed duration of as many empty brackets)"""
        n, ms, empty = C.c_int64(), C.c_double(), C.c_double()
        self._check(self.lib.spark_profile_read(self.handle, C.byref(n), C.byref(ms), C.byref(empty)))
        return n.value, ms.value, empty.value

    def tune(self, name: str, value: int) -> None:
        self._check(self.lib.spark_tune(self.handle, name.encode(), int(value)))

    def measure_read(self, tensor, reps: int = 8, nontemporal: bool = True):
        """(GB/s, xor checksum) of a plain streaming read of a torch device tensor"""
        gbps, chk = C.c_double(), C.c_uint32()
        nbytes = tensor.numel() * tensor.element_size() // 16 * 16
        self._check(self.lib.spark_measure_read(self.handle, C.c_void_p(tensor.data_ptr()), nbytes, reps,
                                                int(nontemporal), C.byref(gbps), C.byref(chk)))
        return gbps.value, chk.value
