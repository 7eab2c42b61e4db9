"""The benchmark's measurement aid (bench_aid/) does what its header says, so that the bare-pattern ceilings and
the cold-cache timings bench.py reports mean something.  Not part of the method: no oracle is involved, the
expected values are the copies and sums the header states."""
import sys

import numpy as np
import pytest

pytestmark = pytest.mark.gpu


def _say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


@pytest.mark.parametrize("mix", [(1, 0, 0), (8, 0, 0), (0, 1, 0), (1, 1, 0), (2, 4, 1), (8, 8, 2), (8, 0, 2),
                                 (16, 16, 2), (0, 2, 2), (0, 0, 1)])
def test_stream_probe_moves_what_it_says(mix):
    import torch
    import bench_aid as A
    r, w, x = mix
    n = 5 * 2048
    rng = np.random.default_rng(r * 100 + w * 10 + x)
    host = [[rng.standard_normal(n).astype(np.float32) for _ in range(c)] for c in mix]
    dev = [[torch.from_numpy(a).cuda() for a in group] for group in host]
    _say(f"[probe] mix={mix} n={n}")
    A.stream_probe(*[[t.data_ptr() for t in group] for group in dev], n, int(torch.cuda.current_stream().cuda_stream))
    torch.cuda.synchronize()
    s = np.zeros(n, np.float32)
    for a in host[0]:
        s = s + a                                      # binary32, in array order, as the kernel adds
    for i in range(r):
        assert np.array_equal(dev[0][i].cpu().numpy(), host[0][i]), "inputs must not change"
    for i in range(w):
        want = host[0][i % r] if r else np.ones(n, np.float32)
        assert np.array_equal(dev[1][i].cpu().numpy(), want)
    for j in range(x):
        assert np.array_equal(dev[2][j].cpu().numpy(), host[2][j] + s)


@pytest.mark.parametrize("mix,shape", [((8, 8, 2), (256, 2, 60)), ((3, 2, 1), (128, 1, 20)), ((2, 4, 0), (64, 1, 0)),
                                       ((0, 0, 2), (256, 4, 0)), ((5, 0, 0), (256, 1, 36)), ((1, 1, 0), (128, 2, 8))])
def test_paced_probe_moves_what_it_says(mix, shape):
    import torch
    import bench_aid as A
    r, w, x = mix
    lanes, vecs, kib = shape
    n = 3 * lanes * vecs * 4
    rng = np.random.default_rng(r * 100 + w * 10 + x)
    host = [[rng.standard_normal(n).astype(np.float32) for _ in range(c)] for c in mix]
    dev = [[torch.from_numpy(a).cuda() for a in group] for group in host]
    _say(f"[paced probe] mix={mix} shape={shape} n={n}")
    A.paced_probe(*[[t.data_ptr() for t in group] for group in dev], n, lanes, vecs, kib << 10,
                  int(torch.cuda.current_stream().cuda_stream))
    torch.cuda.synchronize()
    s = np.zeros(n, np.float32)
    for a in host[0]:
        s = s + a                                      # binary32, in array order, as the kernel adds
    for i in range(r):
        assert np.array_equal(dev[0][i].cpu().numpy(), host[0][i]), "inputs must not change"
    for i in range(w):
        want = host[0][i] if i < r else np.ones(n, np.float32)
        assert np.array_equal(dev[1][i].cpu().numpy(), want)
    for j in range(x):
        assert np.array_equal(dev[2][j].cpu().numpy(), host[2][j] + s)
    t = dev[0][0] if r else dev[2][0]
    for bad in ((n + 4, lanes, vecs, 0), (n, 100, vecs, 0), (n, lanes, 3, 0), (n, lanes, vecs, 100 << 10)):
        with pytest.raises(A.BenchAidError):
            A.paced_probe([t.data_ptr()], [], [], *bad)


def test_stream_probe_rejects_what_it_cannot_run():
    import torch
    import bench_aid as A
    t = torch.zeros(4096, dtype=torch.float32, device="cuda")
    for args in (([], [], [], 2048), ([t.data_ptr()] * 3, [], [], 2048), ([t.data_ptr()], [], [], 1000),
                 ([t.data_ptr()], [], [], 0), ([0], [], [], 2048), ([], [], [t.data_ptr()] * 3, 2048)):
        with pytest.raises(A.BenchAidError):
            A.stream_probe(*args)


def test_cache_scrub_copies_first_half_onto_second_and_checks_its_arguments():
    import torch
    import bench_aid as A
    n = 8 * 2048                                           # floats; two halves of 4 tiles each
    _say(f"[scrub] n={n}")
    buf = torch.arange(n, dtype=torch.float32, device="cuda")
    guard = torch.full((64,), 7.0, dtype=torch.float32, device="cuda")
    A.cache_scrub(buf.data_ptr(), n * 4, int(torch.cuda.current_stream().cuda_stream))
    torch.cuda.synchronize()
    got = buf.cpu().numpy()
    assert np.array_equal(got[:n // 2], np.arange(n // 2, dtype=np.float32))
    assert np.array_equal(got[n // 2:], np.arange(n // 2, dtype=np.float32))
    assert bool((guard == 7.0).all())
    for bad in ((0, n * 4), (buf.data_ptr(), 0), (buf.data_ptr(), 5000), (buf.data_ptr() + 4, n * 4)):
        with pytest.raises(A.BenchAidError):
            A.cache_scrub(*bad)
