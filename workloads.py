"""Seeded synthetic inputs for the decode-step attention path.

This module only draws inputs (queries and KV caches shaped like the paper's
models, with planted structure in the keys).  It holds none of the method's
arithmetic and is the one piece of code that the HIP path's callers and the
CPU oracle's callers both use.  The inputs stand in for the paper's model
weights and long-context datasets, which are not available: they take the
paper's shapes (Llama-2-7B MHA 32 x 128, Llama-3-8B GQA 32/8 x 128, 32 layers
with 2 full + 2 selection + 28 sparse layers, Sec. 4.3; budgets and context
lengths of Sec. 4.2) and synthetic value distributions.

Planting: for a KV head g with group queries q_h, u = sum_h q_h / |sum_h q_h|
and a = mean_h (q_h . u) / sqrt(d); K_g[j] += (delta / a) u raises the mean
scaled logit of token j over the group by exactly delta (before rounding to
the cache dtype).
"""
import math
from dataclasses import dataclass, replace

import torch

DENSE, SELECT, SPARSE = 0, 1, 2
BASE_SEED = 20241005


def schedule_for(num_layers, select_layers=(2, 13), num_dense=2):
    """Fig. 2 / Sec. 4.3: full attention first, selection layers, sparse elsewhere (0-based)."""
    sched = []
    for i in range(num_layers):
        if i < num_dense:
            sched.append(DENSE)
        elif i in select_layers:
            sched.append(SELECT)
        else:
            sched.append(SPARSE)
    return tuple(sched)


@dataclass(frozen=True)
class Workload:
    name: str
    index: int              # 1..6, the configuration it is modelled on
    schedule: tuple         # per layer DENSE / SELECT / SPARSE
    batch: int
    num_q_heads: int
    num_kv_heads: int
    head_dim: int
    dtype: str              # "bf16" or "f32"
    k: int                  # token budget
    seq_lens: tuple         # N_b per sequence, includes the current token
    structure: str          # planted16 | cluster | recency | planted_ragged | zipf
    n_heavy: int = 0
    delta: float = 0.0
    tau: float = 4096.0     # recency length scale
    seed: int = BASE_SEED

    @property
    def num_layers(self):
        return len(self.schedule)

    @property
    def max_seq_len(self):
        return max(self.seq_lens)

    @property
    def group(self):
        return self.num_q_heads // self.num_kv_heads

    @property
    def torch_dtype(self):
        return torch.bfloat16 if self.dtype == "bf16" else torch.float32

    @property
    def elem_bytes(self):
        return 2 if self.dtype == "bf16" else 4

    def kv_bytes_per_layer(self):
        return 2 * sum(self.seq_lens) * self.num_kv_heads * self.head_dim * self.elem_bytes

    def sparse_bytes_per_layer(self):
        rows = sum(min(self.k, n) for n in self.seq_lens)
        return 2 * rows * self.num_kv_heads * self.head_dim * self.elem_bytes

    def algorithmic_bytes_per_step(self):
        """Bytes the method itself must move in one decode step: K and V once per
        full/selection layer, the fp32 group scores written and read once per
        selection layer, the selected rows (and their int32 positions) per sparse layer."""
        total = 0
        score_bytes = sum(self.seq_lens) * self.num_kv_heads * 4
        pos_bytes = self.batch * self.num_kv_heads * self.k * 4
        for kind in self.schedule:
            if kind == DENSE:
                total += self.kv_bytes_per_layer()
            elif kind == SELECT:
                total += self.kv_bytes_per_layer() + 2 * score_bytes + pos_bytes
            else:
                total += self.sparse_bytes_per_layer() + pos_bytes
        return total


def _ragged_lens(batch, lo, hi, seed):
    g = torch.Generator().manual_seed(seed)
    return tuple(int(x) for x in torch.randint(lo, hi + 1, (batch,), generator=g))


def workload(name, **over):
    """The benchmark configurations c1..c5 and the 64-layer c6; keyword overrides give scaled-down cases.

    Overrides: context (all sequences), seq_lens, k, batch, schedule, n_heavy, tau,
    num_q_heads, num_kv_heads, head_dim, dtype.
    """
    s32 = schedule_for(32)
    if name == "c1":
        w = Workload("c1", 1, (DENSE, SELECT, SPARSE, SPARSE), 1, 8, 2, 64, "f32", 128, (2048,),
                     "planted16", n_heavy=16, delta=4.0)
    elif name == "c2":
        w = Workload("c2", 2, s32, 1, 32, 8, 128, "bf16", 2048, (32768,), "cluster", n_heavy=256,
                     delta=3.0)
    elif name == "c3":
        w = Workload("c3", 3, s32, 1, 32, 32, 128, "bf16", 4096, (131072,), "recency", delta=4.0,
                     tau=4096.0)
    elif name == "c4":
        w = Workload("c4", 4, s32, 16, 32, 8, 128, "bf16", 2048,
                     _ragged_lens(16, 8192, 65536, BASE_SEED + 4000), "planted_ragged",
                     n_heavy=256, delta=4.0)
    elif name == "c5":
        w = Workload("c5", 5, s32, 4, 32, 8, 128, "bf16", 4096, (131072,) * 4, "zipf")
    elif name == "c6":
        # the 64-layer model of Sec. 4.3 (2 full + 2 selection + 60 sparse layers) with the 70B
        # head shape, 64 query heads on 8 KV heads; re-selection at layer 31 (App. A, 70B table)
        w = Workload("c6", 6, schedule_for(64, select_layers=(2, 31)), 1, 64, 8, 128, "bf16", 2048, (32768,),
                     "cluster", n_heavy=256, delta=3.0)
    else:
        raise ValueError("unknown workload %r" % (name,))
    if "batch" in over and "seq_lens" not in over and "context" not in over:
        b = over["batch"]
        lens = w.seq_lens
        over["seq_lens"] = tuple(lens[i % len(lens)] for i in range(b))
    if "context" in over:
        b = over.get("batch", w.batch)
        over["seq_lens"] = (int(over.pop("context")),) * b
    if "seq_lens" in over:
        over["seq_lens"] = tuple(int(x) for x in over["seq_lens"])
        over["batch"] = len(over["seq_lens"])
    if "schedule" in over:
        over["schedule"] = tuple(over["schedule"])
    return replace(w, **over)


def heavy_positions(w):
    """Planted positions [B][Hkv][n_heavy] (int64, CPU), drawn once and shared by all layers.

    Returns None for structures that touch every token (recency, zipf).
    """
    if w.structure in ("recency", "zipf"):
        return None
    g = torch.Generator().manual_seed(w.seed + 1000 * w.index + 999)
    pos = torch.zeros((w.batch, w.num_kv_heads, w.n_heavy), dtype=torch.int64)
    for b in range(w.batch):
        n = w.seq_lens[b]
        nh = min(w.n_heavy, n)
        for h in range(w.num_kv_heads):
            if w.structure == "cluster":
                start = int(torch.randint(0, n - nh + 1, (1,), generator=g))
                p = torch.arange(start, start + nh)
            else:
                p = torch.randperm(n, generator=g)[:nh]
            pos[b, h, :nh] = p
            if nh < w.n_heavy:          # tiny contexts: repeat a planted position
                pos[b, h, nh:] = p[0]
    return pos


def zipf_ranks(w, device="cpu"):
    """Rank r_j in 1..N per (sequence, KV head): a random permutation (CPU-drawn, seeded)."""
    g = torch.Generator().manual_seed(w.seed + 1000 * w.index + 998)
    n = w.max_seq_len
    r = torch.stack([torch.stack([torch.randperm(n, generator=g) + 1 for _ in range(w.num_kv_heads)])
                     for _ in range(w.batch)])
    return r.to(device)


def make_layer(w, layer, device="cpu", heavy=None, ranks=None):
    """Inputs of one layer: q [B][Hq][d], K and V [B][Hkv][N_max][d] in the cache dtype.

    Rows at or beyond a sequence's length (ragged batches) are filled with NaN so that
    any read outside [0, N_b) shows up in the output.
    """
    dev = torch.device(device)
    gen = torch.Generator(device=dev).manual_seed(w.seed + 1000 * w.index + layer)
    B, Hq, Hkv, d, G, N = w.batch, w.num_q_heads, w.num_kv_heads, w.head_dim, w.group, w.max_seq_len
    q = torch.randn((B, Hq, d), generator=gen, device=dev, dtype=torch.float32).to(w.torch_dtype)
    K = torch.randn((B, Hkv, N, d), generator=gen, device=dev, dtype=torch.float32)
    V = torch.randn((B, Hkv, N, d), generator=gen, device=dev, dtype=torch.float32).to(w.torch_dtype)

    qg = q.float().view(B, Hkv, G, d)
    u = qg.sum(2)
    norm = u.norm(dim=-1, keepdim=True)
    u = u / norm                                         # [B][Hkv][d]
    a = norm.squeeze(-1) / (G * math.sqrt(d))            # mean_h (q_h.u)/sqrt(d) = |sum q_h|/(G sqrt d)

    if w.structure in ("planted16", "cluster", "planted_ragged"):
        pos = (heavy if heavy is not None else heavy_positions(w)).to(dev)
        idx = pos.unsqueeze(-1).expand(-1, -1, -1, d)
        rows = torch.gather(K, 2, idx)
        if w.structure == "cluster":
            rows = rows * 3.0
        rows = rows + (w.delta / a)[..., None, None] * u[:, :, None, :]
        K.scatter_(2, idx, rows)
    elif w.structure == "recency":
        j = torch.arange(N, device=dev, dtype=torch.float32)
        for b in range(B):
            delta = w.delta * torch.exp(-((w.seq_lens[b] - 1) - j).clamp(min=0) / w.tau)
            K[b] += (delta[None, :, None] / a[b][:, None, None]) * u[b][:, None, :]
    elif w.structure == "zipf":
        r = (ranks if ranks is not None else zipf_ranks(w)).to(dev)
        K *= 0.25
        delta = -1.1 * torch.log(r.float())
        K += (delta / a[..., None])[..., None] * u[:, :, None, :]
    else:
        raise ValueError(w.structure)
    K = K.to(w.torch_dtype)
    for b in range(B):
        if w.seq_lens[b] < N:
            K[b, :, w.seq_lens[b]:] = float("nan")
            V[b, :, w.seq_lens[b]:] = float("nan")
    return q, K, V


def page_table(w, page_size, seed=0, spare=0.125, device="cpu"):
    """Block table of a paged cache for workload w: int32 [B][max_pages] and the pool size.

    Every sequence gets ceil(N_b / page_size) pages drawn without order from a pool that is
    `spare` larger than needed (an allocator under churn hands out scattered pages);
    unused table entries are -1."""
    gen = torch.Generator().manual_seed(w.seed + 77 * w.index + 13 * page_size + seed)
    need = [(n + page_size - 1) // page_size for n in w.seq_lens]
    max_pages = (w.max_seq_len + page_size - 1) // page_size
    num_pages = int(sum(need) * (1.0 + spare)) + 1
    perm = torch.randperm(num_pages, generator=gen)
    table = torch.full((w.batch, max_pages), -1, dtype=torch.int32)
    at = 0
    for b, n in enumerate(need):
        table[b, :n] = perm[at:at + n].to(torch.int32)
        at += n
    return table.to(device), num_pages


def paginate(x, table, num_pages, page_size, layout="HND"):
    """Scatters a logical cache x [B][Hkv][N_max][d] into a page pool by `table`.

    Returns (pool, view): pool is the storage, [page][Hkv][slot][d] for layout "HND" or
    [page][slot][Hkv][d] for "NHD"; view is the same memory indexed [page][Hkv][slot][d].
    Pages that no sequence owns and slots never written stay NaN."""
    B, Hkv, N, d = x.shape
    max_pages = table.shape[1]
    pad = max_pages * page_size - N
    if pad:
        x = torch.cat([x, torch.full((B, Hkv, pad, d), float("nan"), dtype=x.dtype, device=x.device)], 2)
    pages = x.view(B, Hkv, max_pages, page_size, d).permute(0, 2, 1, 3, 4)   # [B][page][Hkv][slot][d]
    if layout == "HND":
        pool = torch.full((num_pages, Hkv, page_size, d), float("nan"), dtype=x.dtype, device=x.device)
        view = pool
    elif layout == "NHD":
        pool = torch.full((num_pages, page_size, Hkv, d), float("nan"), dtype=x.dtype, device=x.device)
        view = pool.permute(0, 2, 1, 3)
    else:
        raise ValueError(layout)
    owned = table >= 0
    view[table[owned].long()] = pages[owned]
    return pool, view
