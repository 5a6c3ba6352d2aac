"""CPU checks of the top-k kernels' arithmetic, without a GPU.

tests/topk_model.cpp re-implements the phases of the argTopK kernels (histogram; pick: k-th bin,
per-slice counts, candidate list in arbitrary order; emit: exact k-th key, slice offsets, compaction,
fallback) as sequential loops; it shares with the kernels only the pure functions of csrc/topk_math.h.  Here it is compared
with the oracle's argTopK (ties to the smaller index, ascending order, -1 padding) on rows built
around the boundaries of that arithmetic: slice edges, misaligned row starts, the candidate list's
capacity, ties at the k-th value.  The bin map is checked for what the kernels rely on: it is
monotone and gives equal keys equal bins."""
import ctypes
import math
import struct

import pytest
import torch

import build_topk_model
from oracle import tidal_oracle as O

SLICE = 4096
BINS = 2048      # kTopkBins of csrc/topk_math.h


@pytest.fixture(scope="module")
def model():
    L = ctypes.CDLL(build_topk_model.build(force=False))
    L.topk_model.argtypes = [ctypes.c_void_p, ctypes.c_int64, ctypes.c_int, ctypes.c_void_p, ctypes.c_int, ctypes.c_int,
                             ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_uint32, ctypes.c_void_p,
                             ctypes.c_void_p]
    L.topk_model.restype = ctypes.c_int
    L.topk_model_bin.argtypes, L.topk_model_bin.restype = [ctypes.c_float] * 3, ctypes.c_int
    L.topk_model_key.argtypes, L.topk_model_key.restype = [ctypes.c_float], ctypes.c_uint32
    L.topk_model_bin_of_scaled.argtypes, L.topk_model_bin_of_scaled.restype = [ctypes.c_float], ctypes.c_int
    L.topk_model_bin_floor.argtypes, L.topk_model_bin_floor.restype = [ctypes.c_int], ctypes.c_float
    L.topk_model_key_to_float.argtypes, L.topk_model_key_to_float.restype = [ctypes.c_uint32], ctypes.c_float
    return L


def run_model(L, scores, lens, rows_per_len, k, first_mis=0, fused=False, cand_max=4096, seed=0):
    scores = scores.contiguous()
    rows, stride = scores.shape
    lens_t = torch.tensor(lens, dtype=torch.int32)
    pos = torch.full((rows, k), -7, dtype=torch.int32)
    paths = torch.zeros(rows, dtype=torch.int32)
    rc = L.topk_model(scores.data_ptr(), stride, rows, lens_t.data_ptr(), rows_per_len, scores.shape[1], k, first_mis,
                      int(fused), cand_max, seed, pos.data_ptr(), paths.data_ptr())
    assert rc == 0
    return pos, paths


def expect(scores, lens, rows_per_len, k):
    return torch.stack([O.topk_row(scores[r, :lens[r // rows_per_len]], k) for r in range(scores.shape[0])])


def f32(x):
    return struct.unpack("f", struct.pack("f", x))[0]


def test_bin_map_is_monotone_and_respects_equal_keys(model):
    g = torch.Generator().manual_seed(11)
    xs = torch.cat([torch.randn(4000, generator=g) * s for s in (1e-6, 1e-2, 1.0, 30.0, 1e4, 1e30)]
                   + [torch.tensor([0.0, -0.0, 2.0 ** -8, -2.0 ** -8, 255.9999, 256.0, -256.0, 3e38, -3e38,
                                    1e-45, -1e-45, 2.0 ** -8 - 1e-10])])
    for center, inv in ((0.0, 1.0), (1.5, 64.0 / 7.0), (-40.0, 0.37), (3e37, 1e-37)):
        order = sorted(xs.tolist())
        bins = [model.topk_model_bin(x, center, inv) for x in order]
        assert all(0 <= b < BINS for b in bins)
        assert all(a <= b for a, b in zip(bins, bins[1:])), (center, inv)
    assert model.topk_model_bin(0.0, 0.0, 1.0) == model.topk_model_bin(-0.0, 0.0, 1.0) == BINS // 2
    assert model.topk_model_key(0.0) == model.topk_model_key(-0.0)
    # the same number of bins per octave on either side of zero, 16 octaves each
    per_octave = BINS // 32
    assert model.topk_model_bin(1.0, 0.0, 1.0) + per_octave == model.topk_model_bin(2.0, 0.0, 1.0)
    assert model.topk_model_bin(-1.0, 0.0, 1.0) - per_octave == model.topk_model_bin(-2.0, 0.0, 1.0)
    assert model.topk_model_bin(f32(1.0 + 1.0 / per_octave), 0.0, 1.0) == model.topk_model_bin(1.0, 0.0, 1.0) + 1
    assert model.topk_model_bin(3e38, 0.0, 1.0) == BINS - 1 and model.topk_model_bin(-3e38, 0.0, 1.0) == 0
    keys = [model.topk_model_key(x) for x in sorted(set(xs.tolist()))]
    assert all(a <= b for a, b in zip(keys, keys[1:]))


def neighbours(x):
    """x and the floats next to it on either side."""
    if math.isnan(x):
        return []
    out = [x]
    for direction in (-math.inf, math.inf):
        y = torch.nextafter(torch.tensor(x, dtype=torch.float32), torch.tensor(direction, dtype=torch.float32)).item()
        out.append(y)
    return out


def test_bin_floor_is_where_the_bin_starts(model):
    """pick and emit compare a scaled score with topk_bin_floor(b) instead of binning it: for every bin b and
    every y (tried: the floor itself, its two neighbours, and random values), y >= floor(b) exactly when bin(y) >= b."""
    g = torch.Generator().manual_seed(5)
    ys = torch.cat([torch.randn(300, generator=g) * s for s in (1e-4, 3e-3, 0.1, 1.0, 20.0, 300.0)]).tolist()
    ys += [0.0, -0.0, math.inf, -math.inf, 2.0 ** -8, -2.0 ** -8, 256.0, -256.0, 1e-45, -1e-45]
    floors = [model.topk_model_bin_floor(b) for b in range(-1, BINS + 2)]
    assert floors[0] == floors[1] == -math.inf and math.isnan(floors[-1]) and math.isnan(floors[-2])
    finite = [f for f in floors[2:-2]]
    assert all(a < b for a, b in zip(finite, finite[1:]))          # strictly increasing: no empty bin
    for b in range(0, BINS + 1):
        fl = model.topk_model_bin_floor(b)
        for y in neighbours(fl) + (ys if b % 97 == 0 else ys[::53]):
            assert (y >= fl) == (model.topk_model_bin_of_scaled(y) >= b), (b, y, fl)
    # a NaN lands in some bin by its bits but compares false with every floor; the kernels bound their writes for that
    assert 0 <= model.topk_model_bin_of_scaled(math.nan) < BINS


def test_key_to_float_inverts_the_key(model):
    g = torch.Generator().manual_seed(6)
    xs = torch.cat([torch.randn(500, generator=g) * s for s in (1e-30, 1e-3, 1.0, 1e20)]).tolist() + [math.inf, -math.inf, f32(1e-45)]
    for x in xs:
        assert model.topk_model_key_to_float(model.topk_model_key(x)) == x
    assert math.copysign(1.0, model.topk_model_key_to_float(model.topk_model_key(-0.0))) == 1.0


LENGTHS = [1, 2, 255, 256, 257, 4093, 4094, 4095, 4096, 4097, 4099, 8191, 8192, 8193, 12289, 20000]


@pytest.mark.parametrize("n", LENGTHS)
@pytest.mark.parametrize("first_mis", [0, 1, 3])
def test_model_matches_oracle_around_slice_boundaries(model, n, first_mis):
    g = torch.Generator().manual_seed(n * 7 + first_mis)
    stride = n + 5           # rows start at every alignment
    scores = torch.randn((4, stride), generator=g) * 2.5
    scores[:, n:] = float("inf")   # beyond the row: must never be picked
    for k in sorted({1, 2, max(1, n // 2), max(1, n - 1), n, n + 3, 255, 256, 257, 4095, 4096, 4097}):
        for fused in (False, True):
            got, _ = run_model(model, scores, [n], 4, k, first_mis=first_mis, fused=fused)
            assert torch.equal(got, expect(scores, [n], 4, k)), (n, k, first_mis, fused)


@pytest.mark.parametrize("cand_max", [1, 7, 255, 256, 257, 4096])
def test_model_candidate_list_capacity_and_ties(model, cand_max):
    g = torch.Generator().manual_seed(cand_max)
    n = 3 * SLICE + 77
    quantised = torch.randint(-3, 4, (n,), generator=g).float()           # 7 distinct values: heavy ties
    constant = torch.full((n,), 2.5)
    zeros = torch.zeros(n)
    zeros[::3] = -0.0
    near = 1.0 + torch.randint(0, 300, (n,), generator=g).float() * 1.1920929e-07   # 300 keys inside one bin
    smooth = torch.randn(n, generator=g)
    scores = torch.stack([quantised, constant, zeros, near, smooth, -quantised])
    want_paths = set()
    for k in (1, 17, 255, 256, 257, 4095, 4096, 4097, n - 1):
        for fused in (False, True):
            got, paths = run_model(model, scores, [n], 6, k, fused=fused, cand_max=cand_max, seed=k)
            assert torch.equal(got, expect(scores, [n], 6, k)), (k, fused, cand_max)
            want_paths |= set(paths.tolist())
    if cand_max <= 257:
        assert 2 in want_paths     # rows of few distinct values overflow a short list: the fallback has run


def test_model_candidate_counts_at_the_list_limit(model):
    """Rows whose k-th bin holds exactly cand_max - 1, cand_max and cand_max + 1 scores."""
    for cand_max in (256, 4096):
        for extra in (-1, 0, 1):
            c = cand_max + extra
            n = 2 * SLICE + 100
            g = torch.Generator().manual_seed(c)
            scores = torch.rand(n, generator=g) * 0.5            # bulk far below
            where = torch.randperm(n, generator=g)[:c + 40]
            scores[where[:c]] = 8.0 + torch.rand(c, generator=g) * 0.05   # inside the bin [8, 8.125)
            scores[where[c:]] = 100.0                            # 40 certain ones above
            k = 40 + c // 2
            for fused in (False, True):
                got, paths = run_model(model, scores[None, :], [n], 1, k, fused=fused, cand_max=cand_max, seed=c)
                assert torch.equal(got, expect(scores[None, :], [n], 1, k)), (cand_max, extra, fused)
                if fused:
                    assert paths[0].item() == (2 if extra > 0 else 1)


def test_model_ragged_rows_many_rows_and_alignments(model):
    g = torch.Generator().manual_seed(3)
    lens = [1, 777, 4097, 64, 9001, 12288, 5000, 4096]
    stride = 12291
    scores = torch.randn((len(lens) * 3, stride), generator=g)
    for b, n in enumerate(lens):
        scores[3 * b:3 * b + 3, n:] = float("inf")
    want = expect(scores, lens, 3, 300)
    for seed in range(8):      # neither the rows' alignment nor the order in which slices run may matter
        got, _ = run_model(model, scores, lens, 3, 300, first_mis=seed % 4, seed=seed)
        assert torch.equal(got, want), seed
