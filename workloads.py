"""Seeded synthetic inputs for paged decode attention.

Serves the oracle-side tests and the HIP-side tests/benchmark alike and holds
none of the method's arithmetic: it draws sequence lengths, deals physical
pages, and fills the caches with random values.  Number-format conversions are
library casts (torch), not code of this repository.

The five workloads mirror the shapes and length mixes of the evaluation the
paper describes (Llama-2-7B-like MHA layers, Sec. 4.1; decode batches of
variable-length requests, Sec. 2.3) and stand in for its request traces, which
are replaced by parametric length distributions.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field

import numpy as np
import torch

PAGE_SIZE = 16
BASE_SEED = 20552


@dataclass(frozen=True)
class Workload:
    ident: int
    name: str
    B: int
    Hq: int
    Hkv: int
    d: int
    lengths: str                  # name of the length distribution
    layers: int = 1               # resident layer caches the benchmark rotates over
    partition_tokens: int = 0     # 0 = single pass
    pool_factor: float = 1.5
    fixed_pool_pages: int = 0     # >0 overrides pool_factor
    page_size: int = PAGE_SIZE

    @property
    def seed(self) -> int:
        return BASE_SEED + self.ident - 1

    @property
    def scale(self) -> float:
        return 1.0 / math.sqrt(self.d)


WORKLOADS = {
    1: Workload(1, "tiny_mha_b4", B=4, Hq=8, Hkv=8, d=64, lengths="uniform_1_512",
                fixed_pool_pages=256),
    2: Workload(2, "llama2_7b_mha_b64", B=64, Hq=32, Hkv=32, d=128,
                lengths="lognormal_1000_16_4096", layers=8, partition_tokens=512),  # the source of the
    # shape does not say whether the pass is split; it is, as in workload 3 (12 % faster than one pass per row)
    3: Workload(3, "llama3_8b_gqa_b256", B=256, Hq=32, Hkv=8, d=128,
                lengths="lognormal_1500_16_8192", layers=32, partition_tokens=512),
    4: Workload(4, "colocated_70b_share_b128", B=128, Hq=64, Hkv=8, d=128,
                lengths="pareto_1.5_256_32768", layers=16, partition_tokens=512),
    5: Workload(5, "length_skew_b512", B=512, Hq=32, Hkv=8, d=128,
                lengths="skew_90_10", layers=1, partition_tokens=512),
}


def draw_lengths(kind: str, B: int, rng: np.random.Generator) -> np.ndarray:
    """Cached tokens per request BEFORE the decode step's append (int32 [B])."""
    if kind == "uniform_1_512":
        L = rng.integers(1, 513, size=B)
    elif kind.startswith("lognormal_"):
        _, median, lo, hi = kind.split("_")
        L = np.rint(np.exp(math.log(float(median)) + 1.0 * rng.standard_normal(B)))
        L = np.clip(L, int(lo), int(hi))
    elif kind.startswith("pareto_"):
        _, alpha, xm, hi = kind.split("_")
        u = rng.random(B)
        L = np.floor(float(xm) * (1.0 - u) ** (-1.0 / float(alpha)))
        L = np.clip(L, int(xm), int(hi))
    elif kind == "skew_90_10":
        n_long = B // 10 if B >= 10 else 1
        short = rng.integers(1, 65, size=B - n_long)
        long_ = rng.integers(32768, 65537, size=n_long)
        L = np.concatenate([short, long_])
        rng.shuffle(L)
    else:
        raise ValueError(kind)
    return L.astype(np.int32)


def deal_pages(capacity_tokens: np.ndarray, page_size: int, rng: np.random.Generator,
               pool_factor: float = 1.5, fixed_pool_pages: int = 0):
    """Give every request enough scattered physical pages for `capacity_tokens`.

    Returns (block_table int32 [B,max_pages], num_pages, spare_page).  Physical
    ids are the head of a random permutation of the pool, dealt round-robin
    over the requests so consecutive logical pages of a request are unrelated
    physical pages.  Table entries past a request's own pages name
    `spare_page`, a page no request owns (callers poison it).
    """
    need = -(-capacity_tokens.astype(np.int64) // page_size)
    total = int(need.sum())
    num_pages = fixed_pool_pages if fixed_pool_pages else int(math.ceil(pool_factor * total)) + 1
    if num_pages <= total:
        raise ValueError("pool too small: need %d pages of %d" % (total + 1, num_pages))
    perm = rng.permutation(num_pages).astype(np.int32)
    spare = int(perm[total])
    B = len(need)
    max_pages = int(need.max()) if B else 0
    bt = np.full((B, max(max_pages, 1)), spare, dtype=np.int32)
    nxt = 0
    for i in range(max_pages):
        rows = np.nonzero(need > i)[0]
        bt[rows, i] = perm[nxt:nxt + len(rows)]
        nxt += len(rows)
    return bt, num_pages, spare


def used_page_mask(block_table: np.ndarray, capacity_tokens: np.ndarray, page_size: int,
                   num_pages: int) -> np.ndarray:
    need = -(-capacity_tokens.astype(np.int64) // page_size)
    mask = np.zeros(num_pages, dtype=bool)
    for b in range(block_table.shape[0]):
        mask[block_table[b, :need[b]]] = True
    return mask


def randn_bf16(shape, seed: int, device="cpu") -> torch.Tensor:
    """N(0,1) values rounded to bf16 (round-to-nearest-even library cast)."""
    g = torch.Generator(device=device)
    g.manual_seed(seed)
    if device == "cpu" or str(device) == "cpu":
        return torch.randn(shape, generator=g, dtype=torch.float32).to(torch.bfloat16)
    return torch.randn(shape, generator=g, dtype=torch.bfloat16, device=device)


def fill_pool_bf16(num_pages, page_size, Hkv, d, used: np.ndarray, seed: int, device="cpu",
                   poison: bool = True) -> torch.Tensor:
    """One cache [num_pages,page_size,Hkv,d] bf16: N(0,1) in used pages, NaN elsewhere."""
    pool = randn_bf16((num_pages, page_size, Hkv, d), seed, device)
    if poison:
        unused = torch.from_numpy(~used).to(pool.device)
        pool[unused] = float("nan")
    return pool


def quantize_pool_fp8(pool_bf16: torch.Tensor, used: np.ndarray):
    """bf16 pool -> (fp8-e4m3 bytes as uint8, fp32 scale [pages,Hkv]).

    scale = amax over (page, kv-head) / 448, floored at 2^-20/448; bytes are
    torch's cast of x/scale to float8_e4m3fn.  Unused pages get NaN bytes and
    NaN scales.
    """
    x = pool_bf16.float()
    x = torch.nan_to_num(x, nan=0.0)
    amax = x.abs().amax(dim=(1, 3)).clamp_min(2.0 ** -20)          # [pages, Hkv]
    scale = (amax / 448.0).float()
    y = (x / scale[:, None, :, None]).clamp(-448.0, 448.0)
    bytes_ = y.to(torch.float8_e4m3fn).view(torch.uint8).clone()
    unused = torch.from_numpy(~used).to(pool_bf16.device)
    bytes_[unused] = 0x7F
    scale[unused] = float("nan")
    return bytes_, scale


def bits(t: torch.Tensor) -> np.ndarray:
    """torch bf16 / uint8 / float32 / int32 tensor -> numpy (bf16 as uint16 bits)."""
    t = t.detach().cpu().contiguous()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).numpy().view(np.uint16)
    return t.numpy()


@dataclass
class Batch:
    """One decode step's inputs (host-side metadata as numpy, tensors as torch)."""
    wl: Workload
    lens_before: np.ndarray       # int32 [B] tokens cached before the append
    block_table: np.ndarray       # int32 [B,max_pages]
    num_pages: int
    spare_page: int
    used: np.ndarray              # bool [num_pages]
    q: torch.Tensor               # bf16 [B,Hq,d]
    k_new: torch.Tensor           # bf16 [B,Hkv,d]
    v_new: torch.Tensor
    k_cache: torch.Tensor         # bf16 [num_pages,ps,Hkv,d]
    v_cache: torch.Tensor
    extra: dict = field(default_factory=dict)

    @property
    def positions(self) -> np.ndarray:
        return self.lens_before.astype(np.int32)

    @property
    def seq_lens(self) -> np.ndarray:
        return (self.lens_before + 1).astype(np.int32)


def make_batch(wl: Workload, device="cpu", headroom_tokens: int = 1, seed_offset: int = 0,
               lens_before: np.ndarray | None = None, with_cache: bool = True) -> Batch:
    """Inputs for workload `wl`: lengths, page table, q/k_new/v_new, one layer's caches.

    Each request gets pages for lens_before + headroom_tokens tokens
    (headroom >= 1 so the append has a slot).
    """
    seed = wl.seed + 1000 * seed_offset
    rng = np.random.default_rng(seed)
    if lens_before is None:
        lens_before = draw_lengths(wl.lengths, wl.B, rng)
    lens_before = np.asarray(lens_before, dtype=np.int32)
    cap = lens_before.astype(np.int64) + headroom_tokens
    bt, num_pages, spare = deal_pages(cap, wl.page_size, rng, wl.pool_factor, wl.fixed_pool_pages)
    used = used_page_mask(bt, cap, wl.page_size, num_pages)
    B = len(lens_before)
    q = randn_bf16((B, wl.Hq, wl.d), seed + 1, device)
    k_new = randn_bf16((B, wl.Hkv, wl.d), seed + 2, device)
    v_new = randn_bf16((B, wl.Hkv, wl.d), seed + 3, device)
    if with_cache:
        kc = fill_pool_bf16(num_pages, wl.page_size, wl.Hkv, wl.d, used, seed + 4, device)
        vc = fill_pool_bf16(num_pages, wl.page_size, wl.Hkv, wl.d, used, seed + 5, device)
    else:
        kc = vc = None
    return Batch(wl, lens_before, bt, num_pages, spare, used, q, k_new, v_new, kc, vc)


def layer_pools(wl: Workload, batch: "Batch", layer: int, device="cpu"):
    """K and V pools of resident layer `layer` (layer 0 is the batch's own pair): same page table and
    poison pattern, values from the layer's own seeds."""
    if layer == 0:
        return batch.k_cache, batch.v_cache
    return (fill_pool_bf16(batch.num_pages, wl.page_size, wl.Hkv, wl.d, batch.used, wl.seed + 100 + 2 * layer, device),
            fill_pool_bf16(batch.num_pages, wl.page_size, wl.Hkv, wl.d, batch.used, wl.seed + 101 + 2 * layer, device))


def describe_lengths(L: np.ndarray) -> dict:
    L = np.asarray(L)
    return {"min": int(L.min()), "median": float(np.median(L)), "mean": float(L.mean()),
            "max": int(L.max()), "total": int(L.sum())}
