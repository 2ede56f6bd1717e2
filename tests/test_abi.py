"""The C-ABI library loads on a machine without a GPU and exports every symbol that
include/spark.h declares; the entry points that need no device behave as documented."""
import ctypes as C
import pathlib
import re

import pytest

import workloads as wl
from paper_2603_09215_amd import binding as sb

HEADER = pathlib.Path(__file__).resolve().parent.parent / "include" / "spark.h"


def declared_functions():
    text = re.sub(r"/\*.*?\*/", "", HEADER.read_text(), flags=re.S)
    return sorted(set(re.findall(r"\b(spark_[a-z_]+)\s*\(", text)))


def test_header_and_binding_list_the_same_entry_points():
    assert declared_functions() == sorted(sb.EXPORTS)


def test_library_exports_every_declared_symbol():
    lib = sb.load_library()
    for name in declared_functions():
        assert hasattr(lib, name), name


def test_config_struct_matches_header_order():
    text = HEADER.read_text()
    body = text[text.index("typedef struct spark_config {"):text.index("} spark_config;")]
    fields = re.findall(r"^\s*(?:uint32_t|int32_t|float)\s+([a-z_]+);", body, flags=re.M)
    assert fields == [f[0] for f in sb.SparkConfig._fields_]
    body = text[text.index("typedef struct spark_weights {"):text.index("} spark_weights;")]
    fields = re.findall(r"^\s*const (?:void|float) \*([a-z_]+);", body, flags=re.M)
    assert fields == list(sb.WEIGHT_FIELDS)


def test_workspace_bytes_and_refusals_need_no_gpu():
    lib = sb.load_library()
    w = wl.STEP_AUDIO_2_MINI
    cfg = sb.make_config(w.shape, w.schedule, 1, 2048, 64)
    kv, sc = C.c_size_t(), C.c_size_t()
    assert lib.spark_workspace_bytes(C.byref(cfg), C.byref(kv), C.byref(sc)) == 0
    # paged bf16 KV: 2 (k,v) * layers * kv heads * head_dim * 2 bytes per token
    assert kv.value == 2048 * 2 * 28 * 4 * 128 * 2
    assert sc.value > 158497 * 4
    bad = [dict(exit_layer=0), dict(exit_layer=29), dict(period_k=0), dict(period_k=17),
           dict(phase=4), dict(scope=3), dict(n_text=0, n_speech=0)]
    for kw in bad:
        cfg = sb.make_config(w.shape, w.schedule.replace(**kw), 1, 2048, 64)
        assert lib.spark_workspace_bytes(C.byref(cfg), None, None) == -1, kw
    for kw in [dict(head_dim=96), dict(d_model=3580), dict(n_q_heads=27)]:
        cfg = sb.make_config(w.shape.replace(**kw), w.schedule, 1, 2048, 64)
        assert lib.spark_workspace_bytes(C.byref(cfg), None, None) == -1, kw
    cfg = sb.make_config(w.shape, w.schedule, 1, 2048, 24)
    assert lib.spark_workspace_bytes(C.byref(cfg), None, None) == -1
    cfg = sb.make_config(w.shape, w.schedule, 1, 2048, 64)
    cfg.size = 4
    assert lib.spark_workspace_bytes(C.byref(cfg), None, None) == -1
    assert lib.spark_last_error(None) == b"null context"


def test_no_gpu_means_loud_failure():
    import torch
    if torch.cuda.is_available():
        pytest.skip("a GPU is present")
    with pytest.raises(RuntimeError):
        sb.Spark(wl.TINY.shape, wl.TINY.schedule, {}, 1, 64)


def test_no_kernel_uses_scratch_memory():
    """The build writes the compiler's per-kernel resource figures next to the objects and refuses
    a kernel with scratch memory or spilled vector registers (an array indexed at run time ends up
    there, a memory round trip per access); this reads the same figures back."""
    import pathlib
    import pytest
    bdir = pathlib.Path(__file__).resolve().parent.parent / "paper_2603_09215_amd" / "_build"
    files = sorted(bdir.glob("*.resources.txt"))
    if not files:
        pytest.skip("the library was not built in this tree")
    n = 0
    for f in files:
        for line in f.read_text().splitlines():
            name, figures = line.split(" ", 1)
            n += 1
            assert "ScratchSize [bytes/lane]=0" in figures, name
            assert "VGPRs Spill=0" in figures, name
    assert n > 100      # every kernel of the library is listed
