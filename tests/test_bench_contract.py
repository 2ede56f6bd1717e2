"""Host-side checks of bench.py that need no GPU: it refuses more than one GPU with a message, and
its byte model (the denominators of the reported bandwidth figures) reproduces the per-step and
per-layer byte counts that follow from the two benchmark shapes: each weight matrix once, the lens
affine and one head for an early-exit step, all layers and the final head for a full-depth step
(the cost model of Sec. IV-B.3)."""
import pathlib
import subprocess
import sys

import workloads as wl

ROOT = pathlib.Path(__file__).resolve().parent.parent
sys.path.insert(0, str(ROOT))


def test_more_than_one_gpu_is_refused_with_a_message():
    p = subprocess.run([sys.executable, str(ROOT / "bench.py"), "--gpus", "2", "--steps", "1", "--warmup", "0"],
                       capture_output=True, text=True, timeout=120)
    assert p.returncode != 0
    assert "one GPU" in p.stderr and p.stdout.strip() == ""


def test_byte_model_matches_the_shapes():
    import bench
    step = wl.WORKLOADS["step_audio_2_mini"]
    ee, full, w_layer = bench.step_bytes(step.shape, step.schedule, 0)
    # 28 layers of 3584 wide, 28 query / 4 KV heads of 128, FFN 18944, 158 497 ids, bf16
    assert w_layer == 2 * (4608 * 3584 + 3584 * 3584 + 2 * 18944 * 3584 + 3584 * 18944) == 466_092_032
    head = 2 * 158_497 * 3584
    assert full == 28 * w_layer + head
    assert ee == 20 * w_layer + 2 * 3584 * 3584 + head
    assert round(full / 1e9, 3) == 14.187 and round(ee / 1e9, 3) == 10.484
    # one cached token costs 2 (K, V) x 4 heads x 128 x 2 bytes per layer that runs
    ee1, full1, _ = bench.step_bytes(step.shape, step.schedule, 1000)
    assert full1 - full == 28 * 1000 * 2048 and ee1 - ee == 20 * 1000 * 2048
    glm = wl.WORKLOADS["glm_4_voice"]
    ee, full, w_layer = bench.step_bytes(glm.shape, glm.schedule, 0)
    assert w_layer == 2 * (4608 * 4096 + 4096 * 4096 + 3 * 13696 * 4096) == 407_896_064
    head = 2 * 167_936 * 4096
    assert full == 40 * w_layer + head and ee == 32 * w_layer + 2 * 4096 * 4096 + head
    assert round(full / 1e9, 3) == 17.692 and round(ee / 1e9, 3) == 14.462
