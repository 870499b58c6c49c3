"""The seeded input generator: torch's wrap-around int64 arithmetic must equal
the big-integer definition, streams must be distinct, moments must be right."""
import numpy as np
import torch

import workloads as wl
from workloads.values import reference_value


def test_torch_fill_equals_bigint_definition():
    key = wl.stream_key(0, "grad", 3, 1, 2)
    t = torch.empty(2000)
    wl.fill_normal_like(t, key, 1e-3, start=12345, chunk=777)
    ref = np.array([reference_value(key, 12345 + i, 1e-3) for i in range(2000)], dtype=np.float32)
    assert np.array_equal(t.numpy(), ref)


def test_streams_differ_and_are_reproducible():
    a, b = torch.empty(4096), torch.empty(4096)
    wl.fill_normal_like(a, wl.stream_key(0, "grad", 0, 0, 0), 1.0)
    wl.fill_normal_like(b, wl.stream_key(0, "grad", 0, 1, 0), 1.0)
    assert not torch.equal(a, b)
    assert abs(float((a * b).mean())) < 0.1
    c = torch.empty(4096)
    wl.fill_normal_like(c, wl.stream_key(0, "grad", 0, 0, 0), 1.0)
    assert torch.equal(a, c)
    # a slice of a stream is the stream at an offset
    d = torch.empty(100)
    wl.fill_normal_like(d, wl.stream_key(0, "grad", 0, 0, 0), 1.0, start=1000)
    assert torch.equal(d, a[1000:1100])


def test_moments():
    t = torch.empty(1 << 20)
    wl.fill_normal_like(t, wl.stream_key(9, "x"), 0.05)
    assert abs(float(t.mean())) < 3 * 0.05 / 1024
    assert abs(float(t.std()) / 0.05 - 1) < 5e-3
    assert float(t.abs().max()) <= 0.05 * 3.4642    # the sum of four uniforms is bounded by 2*sqrt(3) std


def test_packed_wave_draw_is_stable():
    assert [s.W for s in wl.packed_wave_jobs(42)] == [16, 4, 2, 4, 8, 8, 4, 4, 4, 2, 8, 4]
