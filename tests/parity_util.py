"""Helpers for the GPU parity tests: tolerances and the position-parity rule.

Outputs: max-abs error <= 1e-2 and relative L2 error <= 5e-3 against the fp32
oracle (bf16 inputs, fp32 accumulation, bf16-rounded output).  A bf16 output
element of magnitude 4 or more cannot meet 1e-2 in any implementation: the
correctly rounded value is up to half a unit in the last place, 2^-8 * 4 =
1.56e-2, away from the fp32 result.  For such elements (none in the benchmark
configurations, some in the tests of peaked selections) the bar is 1.25 half
units of the element's own bf16 spacing; below magnitude 4 it is 1e-2 as stated.
Positions: bit-exact against the oracle except inside a band around the
oracle's k-th largest score s*: with tau = 1e-4 * max(|s*|, 1), every token
scoring above s* + tau must be selected, none below s* - tau may be, and the
list must hold exactly min(k, N) distinct in-range tokens in ascending order
followed by -1.  Where the oracle's (k+1)-th largest score lies below s* - tau the band leaves no
freedom, and check_positions then asserts the oracle's positions bit for bit (when they are given).
"""
import torch

MAX_ABS = 1e-2
REL_L2 = 5e-3
BAND = 1e-4


def check_output(gpu_out, oracle_out, what=""):
    g = gpu_out.detach().float().cpu()
    o = oracle_out.float()
    assert g.shape == o.shape, what
    assert torch.isfinite(g).all(), "%s: non-finite output" % what
    err = (g - o).abs()
    max_abs = err.max().item()
    rel = ((g - o).norm() / o.norm().clamp_min(1e-30)).item()
    bar = torch.full_like(o, MAX_ABS)
    if gpu_out.dtype == torch.bfloat16:
        half_ulp = torch.exp2(torch.floor(torch.log2(o.abs().clamp_min(1e-30))) - 8.0)
        bar = torch.maximum(bar, 1.25 * half_ulp)
    worst = (err - bar).max().item()
    assert worst <= 0.0, "%s: max-abs %.3e (%.3e over the bar)" % (what, max_abs, worst)
    assert rel <= REL_L2, "%s: rel-L2 %.3e" % (what, rel)
    return max_abs, rel


def check_positions(gpu_pos, oracle_scores, seq_lens, k, what="", relative_band=False, oracle_pos=None):
    """gpu_pos [B][Hkv][k] int32, oracle_scores [B][Hkv][N_max] fp32 (oracle's group scores).
    oracle_pos (optional, like gpu_pos): rows whose (k+1)-th largest score lies below the band must equal it.
    Returns (rows checked, rows that had to be, and were, identical to the oracle's).

    relative_band: tau = 1e-4 * |s*| without the floor of 1, for scores that are probabilities
    (far below 1, where the floor would make the band wider than the scores themselves)."""
    gp = gpu_pos.detach().cpu()
    B, H, _ = gp.shape
    exact = decided = 0
    for b in range(B):
        n = int(seq_lens[b])
        ke = min(k, n)
        for h in range(H):
            row = gp[b, h]
            sel = row[:ke].long()
            assert (row[ke:] == -1).all(), "%s: tail of (%d,%d) is not -1" % (what, b, h)
            assert sel.min() >= 0 and sel.max() < n, "%s: out of range at (%d,%d)" % (what, b, h)
            assert (sel[1:] > sel[:-1]).all(), "%s: not strictly ascending at (%d,%d)" % (what, b, h)
            r = oracle_scores[b, h, :n]
            top = torch.topk(r, min(ke + 1, n)).values
            kth = top[ke - 1]
            tau = BAND * (abs(kth.item()) if relative_band else max(abs(kth.item()), 1.0))
            chosen = torch.zeros(n, dtype=torch.bool)
            chosen[sel] = True
            must = r > kth + tau
            never = r < kth - tau
            assert chosen[must].all(), "%s: a token above the band is missing at (%d,%d)" % (what, b, h)
            assert not chosen[never].any(), "%s: a token below the band was taken at (%d,%d)" % (what, b, h)
            exact += 1
            if oracle_pos is not None and (ke == n or top[ke] < kth - tau):
                assert torch.equal(row, oracle_pos[b, h].to(row.dtype)), \
                    "%s: (%d,%d) differs from the oracle although its k-th score is clear of the next" % (what, b, h)
                decided += 1
    return exact, decided


def same_positions(a, b):
    return torch.equal(a.detach().cpu().int(), b.detach().cpu().int())
