"""GPU parity of the argTopK step on crafted score rows: integer work, compared bit-exactly
with the oracle's argTopK (ties to the smaller index, ascending order, -1 padding)."""
import pytest
import torch

from oracle import tidal_oracle as O
from paper_2410_05076_amd import tidal

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.fixture(scope="module")
def td():
    lens = torch.ones(1, dtype=torch.int32, device=DEV)
    q = torch.zeros((1, 1, 64), dtype=torch.float32, device=DEV)
    K = torch.zeros((1, 1, 8, 64), dtype=torch.float32, device=DEV)
    t = tidal.Tidal(tidal.make_shape(q, K, lens), 1, topk_rows=16, topk_max_len=131072)
    yield t
    t.close()


def run(td, scores, lens, rows_per_len, k):
    s = scores.to(DEV)
    pos = torch.full((s.shape[0], k), -7, dtype=torch.int32, device=DEV)
    td.topk(s, torch.tensor(lens, dtype=torch.int32, device=DEV), rows_per_len, k, pos)
    torch.cuda.synchronize()
    return pos.cpu()


def expect(scores, lens, rows_per_len, k):
    return torch.stack([O.topk_row(scores[r, :lens[r // rows_per_len]], k) for r in range(scores.shape[0])])


@pytest.mark.parametrize("n,k", [(1, 1), (2, 1), (5, 5), (5, 9), (63, 7), (64, 64), (1000, 999),
                                 (4096, 128), (4097, 1), (32768, 2048), (131072, 4096), (131072, 16384),
                                 (70001, 256)])
def test_random_rows(td, n, k):
    g = torch.Generator().manual_seed(n * 31 + k)
    scores = torch.randn((3, n), generator=g) * 3
    assert torch.equal(run(td, scores, [n], 3, k), expect(scores, [n], 3, k))


def test_many_ties_and_special_values(td):
    g = torch.Generator().manual_seed(5)
    n = 9000
    quantised = torch.randint(-3, 4, (n,), generator=g).float()          # 7 distinct values
    constant = torch.full((n,), 2.5)
    zeros = torch.zeros(n)
    zeros[::3] = -0.0                                                     # -0 == +0: ties by index
    wide = torch.randn(n, generator=g) * 1e30
    wide[::7] = -torch.rand(n, generator=g)[::7] * 1e-30
    tiny_gaps = 1.0 + torch.arange(n).float() * 1.1920929e-07             # neighbours 1 ulp apart
    scores = torch.stack([quantised, constant, zeros, wide, tiny_gaps, -quantised])
    for k in (1, 17, 4500, 8999):
        assert torch.equal(run(td, scores, [n], 6, k), expect(scores, [n], 6, k)), k


def test_ragged_rows_and_misaligned_stride(td):
    g = torch.Generator().manual_seed(6)
    lens = [1, 777, 2500, 64, 1301]
    stride = 2501                                                         # rows start off 16-byte boundaries
    buf = torch.randn((5 * 2, stride), generator=g)
    for b, n in enumerate(lens):
        buf[2 * b:2 * b + 2, n:] = float("inf")                          # must never be picked
    k = 256
    got = run(td, buf, lens, 2, k)
    assert torch.equal(got, expect(buf, lens, 2, k))
