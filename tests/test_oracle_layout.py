"""Pins for the oracle's integer side: block splitting, arrival order, wave
interleaving (CPU only).  Fixed points: published parameter counts of the
workload architectures, hand-worked small cases, and an independent
sort-by-exact-fraction statement of the interleaving rule."""
from fractions import Fraction as Fr

import numpy as np
import pytest

import workloads as wl

CAP = 1 << 20

# widely published totals for these architectures (torchvision / BERT-base with
# pooler); AWD-LM follows from the shapes listed in workloads/shapes.py
PARAMS = {"mlp": 407_050, "alexnet": 61_100_840, "resnet50": 25_557_032,
          "vgg16": 138_357_544, "bert_base": 109_482_240, "awd_lm": 33_556_078}
TENSORS = {"mlp": 4, "alexnet": 16, "resnet50": 161, "vgg16": 32, "bert_base": 199, "awd_lm": 14}
# ceil(n / 2^20) summed over tensors, counted by hand from the shape lists
BLOCKS = {"mlp": 4, "alexnet": 69, "resnet50": 169, "vgg16": 158, "bert_base": 269, "awd_lm": 43}
FULL = {"alexnet": 55, "resnet50": 14, "vgg16": 128}
SMALL_TENSORS = {"resnet50": (108, 58_216), "bert_base": (124, 123_648), "vgg16": (17, 15_144),
                 "alexnet": (8, 10_344), "awd_lm": (2, 3_200), "mlp": (2, 522)}


@pytest.mark.parametrize("model", list(PARAMS))
def test_model_totals_and_block_counts(orc, model):
    spec = wl.job_config(model)
    assert spec.n_params == PARAMS[model]
    assert len(spec.layer_numel) == TENSORS[model]
    blocks = orc.split_layers(spec.layer_numel, CAP)
    assert len(blocks) == BLOCKS[model]
    assert sum(b[2] for b in blocks) == PARAMS[model]
    if model in FULL:
        assert sum(1 for b in blocks if b[2] == CAP) == FULL[model]
    cnt, tot = SMALL_TENSORS[model]
    small = [n for n in spec.layer_numel if n <= 4096]
    assert (len(small), sum(small)) == (cnt, tot)


def test_split_rule_full_blocks_then_remainder(orc):
    assert orc.split_layers([4096 * 9216], CAP) == [(0, i * CAP, CAP) for i in range(36)]
    b = orc.split_layers([1000 * 4096], CAP)
    assert b == [(0, 0, CAP), (0, CAP, CAP), (0, 2 * CAP, CAP), (0, 3 * CAP, 950_272)]
    assert orc.split_layers([10, 25, 7], 10) == [(0, 0, 10), (1, 0, 10), (1, 10, 10), (1, 20, 5), (2, 0, 7)]
    assert orc.split_layers([1], CAP) == [(0, 0, 1)]
    assert orc.split_layers([], CAP) == []
    with pytest.raises(ValueError):
        orc.split_layers([0], CAP)


def test_split_covers_every_element_once(orc):
    rng = np.random.default_rng(0)
    for _ in range(50):
        layers = [int(x) for x in rng.integers(1, 5000, size=rng.integers(1, 8))]
        cap = int(rng.integers(1, 2000))
        blocks = orc.split_layers(layers, cap)
        seen = [np.zeros(n, dtype=np.int32) for n in layers]
        for l, off, n in blocks:
            assert 1 <= n <= cap
            seen[l][off:off + n] += 1
        assert all((s == 1).all() for s in seen)
        assert [b[0] for b in blocks] == sorted(b[0] for b in blocks)


def test_arrival_is_last_layer_first_offsets_ascending(orc):
    # layers of 1, 3, 2 blocks -> ids 0 | 1 2 3 | 4 5
    assert orc.arrival_order([0, 1, 1, 1, 2, 2]) == [4, 5, 1, 2, 3, 0]
    assert orc.arrival_order([0]) == [0]
    assert orc.arrival_order([]) == []
    assert orc.arrival_order([0, 1, 2, 3]) == [3, 2, 1, 0]
    spec = wl.job_config("vgg16")
    blocks = orc.split_layers(spec.layer_numel, CAP)
    order = orc.arrival_order([b[0] for b in blocks])
    assert sorted(order) == list(range(len(blocks)))
    # last registered tensor (fc16.bias) is first; first conv weight is last
    assert blocks[order[0]][0] == 31 and blocks[order[-1]][0] == 0
    layers_seen = [blocks[b][0] for b in order]
    assert layers_seen == sorted(layers_seen, reverse=True)
    for a, b in zip(order, order[1:]):
        if blocks[a][0] == blocks[b][0]:
            assert blocks[a][1] < blocks[b][1]


def test_interleave_hand_cases(orc):
    # positions (k + 1/2)/n: job0 = 1/4, 3/4 ; job1 = 1/6, 3/6, 5/6
    assert orc.interleave([2, 3]) == [(1, 0), (0, 0), (1, 1), (0, 1), (1, 2)]
    # ties go to the lower job index
    assert orc.interleave([1, 1]) == [(0, 0), (1, 0)]
    assert orc.interleave([1, 3]) == [(1, 0), (0, 0), (1, 1), (1, 2)]
    assert orc.interleave([2, 4]) == [(1, 0), (0, 0), (1, 1), (1, 2), (0, 1), (1, 3)]
    assert orc.interleave([3]) == [(0, 0), (0, 1), (0, 2)]
    assert orc.interleave([]) == []
    assert orc.interleave([0, 2]) == [(1, 0), (1, 1)]


def test_interleave_equals_sort_by_exact_fraction(orc):
    rng = np.random.default_rng(1)
    for _ in range(30):
        ns = [int(x) for x in rng.integers(0, 40, size=rng.integers(1, 7))]
        want = sorted(((Fr(2 * k + 1, 2 * n), j, k) for j, n in enumerate(ns) for k in range(n)))
        assert orc.interleave(ns) == [(j, k) for _, j, k in want]


def test_packed_wave_totals(orc):
    specs = wl.packed_wave_jobs(42)
    assert [s.model for s in specs] == (["resnet50"] * 3 + ["vgg16"] * 3 + ["alexnet"] * 2
                                        + ["bert_base"] * 2 + ["awd_lm"] * 2)
    assert all(s.W in (2, 4, 8, 16) for s in specs)
    jobs = [orc.OracleJob.__new__(orc.OracleJob) for _ in specs]
    for j, s in zip(jobs, specs):          # layout only: skip allocating 7 GB of state
        j.blocks = orc.split_layers(s.layer_numel, CAP)
        j.arrival = lambda j=j: orc.arrival_order([b[0] for b in j.blocks])
    wave = orc.pack_wave(jobs)
    assert len(wave) == 1743
    assert sum(len(s.layer_numel) for s in specs) == 1037
    assert sum(jobs[j].blocks[b][2] for j, b in wave) == 900_022_044
    assert len(set(wave)) == len(wave)
    # each job's own sub-sequence is its arrival order
    for ji, j in enumerate(jobs):
        assert [b for jj, b in wave if jj == ji] == j.arrival()
    # all jobs progress together: after any prefix, done fractions differ by < 1 block each
    done = [0] * len(jobs)
    for t, (ji, _) in enumerate(wave):
        done[ji] += 1
        if t % 97 == 0:
            fr = [done[i] / len(jobs[i].blocks) for i in range(len(jobs))]
            slack = max(1.0 / len(j.blocks) for j in jobs)
            assert max(fr) - min(fr) <= slack + 1e-12
