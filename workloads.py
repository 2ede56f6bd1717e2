"""Seeded synthetic inputs shared by the CPU oracle and the HIP path.

This module holds data recipes only: model shapes, random weight tensors,
random prompts and random teacher-forcing streams.  It contains none of the
method's arithmetic (no schedule, no transformer math), so both sides can draw
identical inputs from it without sharing any computation.

The shapes stand in for the paper's two backbones (Sec. V-A "Models":
Step-Audio-2-mini, 28 layers; GLM-4-Voice, 40 layers) whose checkpoints, trained
layer-specific heads (Sec. IV-B.2) and evaluation responses are not available
here: weights are N(0, 0.02) draws, prompts and streams are uniform ids.
"""
from __future__ import annotations

import dataclasses
from concurrent.futures import ThreadPoolExecutor

import numpy as np

SCOPE_CHUNK = 0   # period counter restarts with every speech chunk (Sec. IV-B.1)
SCOPE_STREAM = 1  # period counter runs over all speech positions of a sequence

DTYPE_FP32 = 0
DTYPE_BF16 = 1


@dataclasses.dataclass(frozen=True)
class ModelShape:
    name: str
    n_layers: int
    d_model: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    d_ffn: int
    vocab_text: int
    vocab_speech: int
    rope_base: float = 10000.0
    rms_eps: float = 1e-6
    dtype: int = DTYPE_BF16

    @property
    def vocab(self) -> int:
        return self.vocab_text + self.vocab_speech

    def replace(self, **kw) -> "ModelShape":
        return dataclasses.replace(self, **kw)


@dataclasses.dataclass(frozen=True)
class Schedule:
    exit_layer: int
    period_k: int
    phase: int
    scope: int
    n_text: int
    n_speech: int
    # the same periodic rule on text positions (Sec. V-C, Table II row G10); K_text <= 1: text
    # always runs full depth
    text_period_k: int = 0
    text_phase: int = 0

    def replace(self, **kw) -> "Schedule":
        return dataclasses.replace(self, **kw)


@dataclasses.dataclass(frozen=True)
class Workload:
    shape: ModelShape
    schedule: Schedule
    prompt_len: int
    decode_len: int
    prompt_ids: str  # "all" = uniform over the whole vocabulary, "speech" = speech range only


TINY = Workload(
    ModelShape("tiny", 4, 256, 4, 2, 64, 1024, 1024, 512, dtype=DTYPE_FP32),
    Schedule(exit_layer=2, period_k=4, phase=3, scope=SCOPE_CHUNK, n_text=2, n_speech=4),
    prompt_len=16, decode_len=64, prompt_ids="all")

STEP_AUDIO_2_MINI = Workload(
    ModelShape("step_audio_2_mini", 28, 3584, 28, 4, 128, 18944, 151936, 6561),
    Schedule(exit_layer=20, period_k=4, phase=3, scope=SCOPE_STREAM, n_text=1, n_speech=2),
    prompt_len=512, decode_len=1024, prompt_ids="speech")

GLM_4_VOICE = Workload(
    ModelShape("glm_4_voice", 40, 4096, 32, 2, 128, 13696, 151552, 16384),
    Schedule(exit_layer=32, period_k=4, phase=3, scope=SCOPE_STREAM, n_text=13, n_speech=26),
    prompt_len=1024, decode_len=2048, prompt_ids="all")

WORKLOADS = {w.shape.name: w for w in (TINY, STEP_AUDIO_2_MINI, GLM_4_VOICE)}


# --------------------------------------------------------------------------- weights

# name -> (shape builder, is_matrix).  Matrices are stored [out][in] row-major and carry the
# model dtype; gains and the lens bias are always fp32.
def tensor_shapes(s: ModelShape) -> dict[str, tuple[int, ...]]:
    L, d, F, V = s.n_layers, s.d_model, s.d_ffn, s.vocab
    q, kv = s.n_q_heads * s.head_dim, s.n_kv_heads * s.head_dim
    return {
        "embed": (V, d),
        "attn_norm": (L, d),
        "wq": (L, q, d), "wk": (L, kv, d), "wv": (L, kv, d), "wo": (L, d, q),
        "mlp_norm": (L, d),
        "wg": (L, F, d), "wu": (L, F, d), "wd": (L, d, F),
        "final_norm": (d,),
        "lm_head": (V, d),
        "lens_a": (d, d), "lens_b": (d,), "lens_norm": (d,), "lens_head": (V, d),
    }


GAIN_TENSORS = ("attn_norm", "mlp_norm", "final_norm", "lens_norm")
FP32_TENSORS = GAIN_TENSORS + ("lens_b",)


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even fp32 -> bf16, returned as uint16 bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    return (r >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


def _fill_normal(out: np.ndarray, seed_key, std: float, bf16: bool, chunk: int = 1 << 24) -> None:
    rng = np.random.Generator(np.random.Philox(np.random.SeedSequence(seed_key)))
    flat = out.reshape(-1)
    n = flat.shape[0]
    for lo in range(0, n, chunk):
        hi = min(n, lo + chunk)
        x = rng.standard_normal(hi - lo, dtype=np.float32)
        x *= np.float32(std)
        if bf16:
            flat[lo:hi] = f32_to_bf16_bits(x)
        else:
            flat[lo:hi] = x


def make_weights(shape: ModelShape, seed: int = 0, std: float = 0.02, gain_std: float = 0.0,
                 threads: int = 8) -> dict[str, np.ndarray]:
    """All tensors of one model.  Matrices are float32 arrays (dtype fp32) or uint16 arrays of
    bf16 bit patterns (dtype bf16), each rounded exactly once here.  Gains are 1 + gain_std*N(0,1)
    (1 exactly when gain_std == 0), fp32."""
    bf16 = shape.dtype == DTYPE_BF16
    shapes = tensor_shapes(shape)
    out: dict[str, np.ndarray] = {}
    jobs = []
    for tid, (name, shp) in enumerate(shapes.items()):
        if name in GAIN_TENSORS:
            g = np.ones(shp, dtype=np.float32)
            if gain_std:
                _fill_normal(g, (seed, tid, 0), gain_std, False)
                g += np.float32(1.0)
            out[name] = g
            continue
        as_bf16 = bf16 and name not in FP32_TENSORS
        arr = np.empty(shp, dtype=np.uint16 if as_bf16 else np.float32)
        out[name] = arr
        if len(shp) == 3:      # per-layer slabs are independent streams
            for l in range(shp[0]):
                jobs.append((arr[l], (seed, tid, l + 1), as_bf16))
        elif arr.size > (1 << 26):  # vocabulary matrices: split rows
            rows = shp[0]
            step = max(1, (1 << 26) // shp[1])
            for k, r0 in enumerate(range(0, rows, step)):
                jobs.append((arr[r0:r0 + step], (seed, tid, 0, k), as_bf16))
        else:
            jobs.append((arr, (seed, tid, 0), as_bf16))
    with ThreadPoolExecutor(max_workers=max(1, threads)) as ex:
        list(ex.map(lambda j: _fill_normal(j[0], j[1], std, j[2]), jobs))
    return out


def weight_bytes(shape: ModelShape) -> int:
    esz = 2 if shape.dtype == DTYPE_BF16 else 4
    tot = 0
    for name, shp in tensor_shapes(shape).items():
        tot += int(np.prod(shp)) * (4 if name in FP32_TENSORS else esz)
    return tot


# --------------------------------------------------------------------------- token streams

def make_prompt(shape: ModelShape, n: int, seed: int = 1, ids: str = "all") -> np.ndarray:
    rng = np.random.Generator(np.random.Philox(np.random.SeedSequence((seed, 101))))
    if ids == "speech":
        return rng.integers(shape.vocab_text, shape.vocab, size=n, dtype=np.int32)
    return rng.integers(0, shape.vocab, size=n, dtype=np.int32)


def make_forced_stream(shape: ModelShape, n: int, n_text: int, n_speech: int, slot_offset: int = 0,
                       seed: int = 2) -> np.ndarray:
    """A fixed stream of n ids to teacher-force: ids at text slots of the repeating
    (n_text text, n_speech speech) pattern are uniform text ids, the others uniform speech ids."""
    rng = np.random.Generator(np.random.Philox(np.random.SeedSequence((seed, 202))))
    t = rng.integers(0, shape.vocab_text, size=n, dtype=np.int32)
    s = rng.integers(shape.vocab_text, shape.vocab, size=n, dtype=np.int32)
    slot = (np.arange(n) + slot_offset) % (n_text + n_speech)
    return np.where(slot < n_text, t, s).astype(np.int32)


def make_prompt_lengths(n_seq: int, lo: int, hi: int, seed: int = 3) -> np.ndarray:
    rng = np.random.Generator(np.random.Philox(np.random.SeedSequence((seed, 303))))
    return rng.integers(lo, hi + 1, size=n_seq, dtype=np.int32)


# --------------------------------------------------------------------------- large models

def make_weights_on_device(shape: ModelShape, seed: int = 0, std: float = 0.02, device="cuda:0") -> dict:
    """The same tensors as make_weights (unit gains), drawn with torch's generator on the GPU:
    billions of parameters in about a second.  Returns torch device tensors."""
    import torch
    g = torch.Generator(device=device)
    g.manual_seed(seed)
    dt = torch.bfloat16 if shape.dtype == DTYPE_BF16 else torch.float32
    out = {}
    for name, shp in tensor_shapes(shape).items():
        if name in GAIN_TENSORS:
            out[name] = torch.ones(shp, dtype=torch.float32, device=device)
        elif name in FP32_TENSORS:
            out[name] = torch.randn(shp, generator=g, dtype=torch.float32, device=device) * std
        else:
            t = torch.empty(shp, dtype=dt, device=device)
            flat = t.view(-1)
            step = 1 << 28          # bounded fp32 temporaries
            for lo in range(0, flat.numel(), step):
                hi = min(flat.numel(), lo + step)
                flat[lo:hi] = (torch.randn(hi - lo, generator=g, dtype=torch.float32, device=device)
                               * std).to(dt)     # rounded to bf16 exactly once, here
            out[name] = t
    return out


def device_weights_to_host(dev_weights: dict) -> dict:
    """torch device tensors -> numpy arrays in make_weights' conventions (bf16 as uint16 bits)"""
    import torch
    out = {}
    for k, t in dev_weights.items():
        c = t.cpu()
        out[k] = c.view(torch.int16).numpy().view(np.uint16) if c.dtype == torch.bfloat16 else c.numpy()
    return out
