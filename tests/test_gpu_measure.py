"""Measurement support on the GPU: the plain streaming read (spark_measure_read) reads every word
of the buffer exactly once -- its XOR checksum equals numpy's, for sizes with a ragged end, with
both load flavours -- and reports a plausible rate; the per-class event brackets count launches."""
import numpy as np
import pytest

import workloads as wl

pytestmark = pytest.mark.gpu


def test_streaming_read_checksum_and_rate():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2603_09215_amd import binding as sb
    w = wl.TINY
    sp = sb.Spark(w.shape, w.schedule, wl.make_weights(w.shape, seed=0), max_batch=1, max_seq_len=64, kv_page_tokens=16)
    rng = np.random.default_rng(5)
    for n_words in (4 * 512 * 2048 * 3 + 4 * 777, 4 * 513, 4 * 64, 4):      # whole trips + ragged end, tiny sizes
        host = rng.integers(0, 2 ** 32, size=n_words, dtype=np.uint32)
        dev = torch.from_numpy(host.view(np.int32)).to("cuda:0")
        want = int(np.bitwise_xor.reduce(host))
        for nt in (True, False):
            gbps, chk = sp.measure_read(dev, reps=2, nontemporal=nt)
            assert chk == want, (n_words, nt, hex(chk), hex(want))
            assert gbps > 0
    big = torch.zeros(1 << 28, dtype=torch.int32, device="cuda:0")          # 1 GiB: far beyond the caches
    gbps, chk = sp.measure_read(big, reps=3, nontemporal=True)
    assert chk == 0 and 1000.0 < gbps < 8000.0, gbps
    import ctypes as C
    g = C.c_double()
    rc = sp.lib.spark_measure_read(sp.handle, C.c_void_p(big.data_ptr()), 24, 1, 1, C.byref(g), None)
    assert rc == -1                                 # a size that is not a multiple of 16 is refused
    sp.close()


def test_profile_brackets_count_launches():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2603_09215_amd import binding as sb
    w = wl.TINY
    sp = sb.Spark(w.shape, w.schedule, wl.make_weights(w.shape, seed=0), max_batch=1, max_seq_len=64, kv_page_tokens=16)
    sid = sp.seq_open(0)
    sp.prefill(sid, wl.make_prompt(w.shape, 8, seed=1))
    sp.profile_select("gateup")
    tok, dep = sp.decode(12, [sid])
    n, ms, empty = sp.profile_read()
    layers = sum(int(d) for d in dep[:, 0])        # one gate/up launch per executed layer: e or L per step
    assert n == layers and ms > 0 and 0 <= empty < ms
    sp.profile_select(-1)
    sp.close()
