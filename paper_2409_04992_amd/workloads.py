"""Seeded synthetic inputs for decode attention (shapes of the paper's 13B workloads).

This module only draws tensors; it contains none of the method's arithmetic and
imports neither the HIP binding nor the oracle, so both sides can be fed the very
same bits.  The paper measures an OPT-13B-shaped model (40 heads of 128, fp16 for
all variables, Sec. VI-A) on text sampled from public datasets; decode attention's
cost depends only on shapes and its result only on the tensors, so seeded
Gaussians of those shapes stand in for that data.

All tensors are torch tensors on `device`:
  q [B, Hq, D] f16; k_new, v_new [B, Hkv, D] f16; seq_lens [B] i32 (length
  INCLUDING the token appended in this step); contiguous caches
  [B, Hkv, capacity, D] f16 or paged pools [num_pages, Hkv, page_size, D] f16 with
  page_table [B, max_pages] i32 (shuffled pool ids, -1 behind the used entries).
"""
from __future__ import annotations

import dataclasses
import math
from typing import Optional

import torch


@dataclasses.dataclass(frozen=True)
class Workload:
    name: str
    batch: int
    num_q_heads: int
    num_kv_heads: int
    head_dim: int
    seq_len: int                 # cached length S before the step (max, if ragged)
    seq_len_min: int = 0         # ragged: S_b ~ U[seq_len_min, seq_len]; 0 = uniform
    paged: bool = False
    page_size: int = 16
    out_dtype: str = "f16"       # "f16" | "f32"
    head_scale: bool = False     # per-KV-head std drawn from U[0.5, 2] for K and V
    layers: int = 1
    seed: int = 0
    kv_adjacent: bool = False    # paged: one pool [num_pages][Hkv][2][page][D], a (page, head)'s K and V blocks adjacent

    @property
    def group(self) -> int:
        return self.num_q_heads // self.num_kv_heads

    @property
    def scale(self) -> float:
        return 1.0 / math.sqrt(self.head_dim)


# The five configurations this build is measured and checked on.
WORKLOADS = {
    "tiny_mha": Workload("tiny_mha", 2, 4, 4, 64, 256, out_dtype="f32", seed=1001),
    "mha13b_4k": Workload("mha13b_4k", 16, 40, 40, 128, 4096, head_scale=True, seed=1002),
    "mha13b_32k": Workload("mha13b_32k", 8, 40, 40, 128, 32768, seed=1003),
    "ragged_paged": Workload("ragged_paged", 64, 40, 40, 128, 16384, seq_len_min=1024,
                             paged=True, page_size=16, seed=1004),
    "gqa70b_16k": Workload("gqa70b_16k", 32, 64, 8, 128, 16384, layers=80, seed=1005),
}


def get_workload(spec: str) -> Workload:
    """A named configuration, or "custom:{json}" with Workload's fields (for sweeps)."""
    if spec.startswith("custom:"):
        import json
        return Workload(**json.loads(spec[7:]))
    return WORKLOADS[spec]


@dataclasses.dataclass
class Case:
    wl: Workload
    q: torch.Tensor
    k_cache: torch.Tensor
    v_cache: torch.Tensor
    k_new: torch.Tensor
    v_new: torch.Tensor
    seq_lens: torch.Tensor
    page_table: Optional[torch.Tensor]
    scale: float
    capacity: int

    def kv_read_bytes(self) -> int:
        """K and V bytes one decode step of this layer must read (every row once)."""
        total = int(self.seq_lens.clamp(min=0).sum().item())
        return total * self.wl.num_kv_heads * self.wl.head_dim * 2 * 2


def _gen(device, seed: int) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(int(seed))
    return g


def _randn_f16(shape, g, device) -> torch.Tensor:
    """N(0,1) drawn in fp32 and rounded once to fp16, in slabs to bound the temporary."""
    out = torch.empty(shape, dtype=torch.float16, device=device)
    flat = out.view(-1)
    slab = 1 << 28
    for lo in range(0, flat.numel(), slab):
        hi = min(lo + slab, flat.numel())
        flat[lo:hi] = torch.randn(hi - lo, dtype=torch.float32, device=device, generator=g)
    return out


def draw_seq_lens(wl: Workload, device="cpu") -> torch.Tensor:
    """Lengths L_b = S_b + 1 (the appended token counted), int32 on `device`."""
    if wl.seq_len_min > 0:
        g = _gen("cpu", wl.seed * 7 + 1)
        s = torch.randint(wl.seq_len_min, wl.seq_len + 1, (wl.batch,), generator=g)
    else:
        s = torch.full((wl.batch,), wl.seq_len, dtype=torch.int64)
    return (s + 1).to(torch.int32).to(device)


def make_case(wl: Workload, device="cpu", layer: int = 0, poison: bool = False,
              capacity: Optional[int] = None, lens=None) -> Case:
    """Draw one layer's inputs.  `poison` fills every cache row at or behind
    position L_b - 1 (stale rows, slack in the last page, spare pages) with NaN so
    that any read outside the valid range shows in the output.  `lens` (a list of
    wl.batch lengths between 0 and wl.seq_len + 1, the appended token counted) takes
    the place of the drawn lengths; page tables and poison follow it."""
    dev = torch.device(device)
    B, Hq, Hkv, D = wl.batch, wl.num_q_heads, wl.num_kv_heads, wl.head_dim
    g = _gen(dev, wl.seed * 1000 + layer)
    if lens is None:
        seq_lens = draw_seq_lens(wl, dev)
    else:
        assert len(lens) == B and all(0 <= int(L) <= wl.seq_len + 1 for L in lens)
        seq_lens = torch.tensor([int(L) for L in lens], dtype=torch.int32, device=dev)
    lens_cpu = seq_lens.cpu()
    q = _randn_f16((B, Hq, D), g, dev)
    k_new = _randn_f16((B, Hkv, D), g, dev)
    v_new = _randn_f16((B, Hkv, D), g, dev)
    sigma = None
    if wl.head_scale:
        gs = _gen("cpu", wl.seed * 7 + 2)
        sigma = (0.5 + 1.5 * torch.rand(Hkv, generator=gs)).to(dev)
        k_new = (k_new.float() * sigma[None, :, None]).half()
        v_new = (v_new.float() * sigma[None, :, None]).half()

    if not wl.paged:
        cap = capacity if capacity is not None else (wl.seq_len + 1 + 15) // 16 * 16
        k_cache = _randn_f16((B, Hkv, cap, D), g, dev)
        v_cache = _randn_f16((B, Hkv, cap, D), g, dev)
        if sigma is not None:
            for t in (k_cache, v_cache):
                for hk in range(Hkv):
                    t[:, hk] = (t[:, hk].float() * sigma[hk]).half()
        if poison:
            for b in range(B):
                k_cache[b, :, max(int(lens_cpu[b]) - 1, 0):, :] = float("nan")
                v_cache[b, :, max(int(lens_cpu[b]) - 1, 0):, :] = float("nan")
        page_table = None
    else:
        ps = wl.page_size
        max_pages = (wl.seq_len + 1 + ps - 1) // ps
        need = [(int(L) + ps - 1) // ps for L in lens_cpu]
        spare = 3
        num_pages = sum(need) + spare
        cap = ps * max_pages
        if wl.kv_adjacent:
            pool = _randn_f16((num_pages, Hkv, 2, ps, D), g, dev)
            k_cache, v_cache = pool[:, :, 0], pool[:, :, 1]     # same strides, bases 4 KB apart
        else:
            k_cache = _randn_f16((num_pages, Hkv, ps, D), g, dev)
            v_cache = _randn_f16((num_pages, Hkv, ps, D), g, dev)
        gp = _gen("cpu", wl.seed * 7 + 3)
        perm = torch.randperm(num_pages, generator=gp).to(torch.int32)
        table = torch.full((B, max_pages), -1, dtype=torch.int32)
        at = 0
        for b in range(B):
            table[b, :need[b]] = perm[at:at + need[b]]
            at += need[b]
        if poison:
            unused = perm[at:].long().to(dev)
            k_cache[unused] = float("nan")
            v_cache[unused] = float("nan")
            for b in range(B):
                L = int(lens_cpu[b])
                if L < 1:
                    continue                                   # no page of its own
                last = int(table[b, (L - 1) // ps])
                k_cache[last, :, (L - 1) % ps:, :] = float("nan")
                v_cache[last, :, (L - 1) % ps:, :] = float("nan")
        page_table = table.to(dev)

    return Case(wl, q, k_cache, v_cache, k_new, v_new, seq_lens, page_table, wl.scale, cap)


def scaled_down(wl: Workload, **changes) -> Workload:
    """Same recipe at a size the CPU oracle finishes in seconds."""
    return dataclasses.replace(wl, **changes)
