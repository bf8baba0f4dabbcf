"""Seeded synthetic decode workloads (inputs only -- no part of the method is computed here).

The five generators mirror the shapes and key statistics of the workloads the
paper evaluates (Section 4: text LLM with 32 query / 8 KV heads of dimension
128 at 32K-128K context; long-form speech), which need datasets and model
weights that are not available here. Everything is drawn from seeded torch
generators; values are drawn in fp32, rounded once to the cache dtype, and the
resulting bit patterns are what both the GPU library and the CPU checker read.

Cache layout: ``k_cache``/``v_cache`` = [num_phys_pages][Hkv][S][D]; ``page_table``
= int32 [B][max_pages_per_seq] (logical -> physical); ``seq_lens`` = int32 [B];
``q`` = [B][H][D]; query head h reads KV head h // (H // Hkv).

Seeds: ``1000 * config + stream`` with stream 0 = q, 1 = K, 2 = V, 3 = page-table
permutation, 4 = lengths, 5 = planted / outlier keys. Small host-side draws
(lengths, permutations, plant positions) always use a CPU generator so they do
not depend on the device; the bulk normal draws use the target device.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field

import numpy as np
import torch


@dataclass
class Workload:
    name: str
    dtype: torch.dtype
    B: int
    H: int
    Hkv: int
    D: int
    S: int
    top_k: int
    lam: float
    q: torch.Tensor
    k_cache: torch.Tensor
    v_cache: torch.Tensor
    page_table: torch.Tensor
    seq_lens: torch.Tensor
    meta: dict = field(default_factory=dict)

    @property
    def G(self) -> int:
        return self.H // self.Hkv

    @property
    def num_phys_pages(self) -> int:
        return int(self.k_cache.shape[0])

    @property
    def max_pages(self) -> int:
        return int(self.page_table.shape[1])

    def num_pages(self, b: int) -> int:
        return (int(self.seq_lens[b]) + self.S - 1) // self.S

    def to(self, device) -> "Workload":
        kw = {k: (v.to(device) if isinstance(v, torch.Tensor) else v) for k, v in self.__dict__.items()}
        return Workload(**kw)

    def host_arrays(self) -> dict:
        """numpy views for a host-side checker: fp32 stays float32, bf16 becomes uint16 bit patterns."""
        def conv(t: torch.Tensor) -> np.ndarray:
            t = t.detach().cpu().contiguous()
            if t.dtype == torch.bfloat16:
                return t.view(torch.int16).numpy().view(np.uint16)
            return t.numpy()
        return dict(q=conv(self.q), k_cache=conv(self.k_cache), v_cache=conv(self.v_cache),
                    page_table=conv(self.page_table), seq_lens=conv(self.seq_lens))


def _gen(seed: int, device="cpu") -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(seed)
    return g


def _ar1(n_tok: int, width: int, rho: float, gen: torch.Generator, device) -> torch.Tensor:
    """Unit-variance AR(1) along time: x_t = rho x_{t-1} + sqrt(1-rho^2) eps_t, x_0 ~ N(0,1). -> [n_tok, width]."""
    L = 512
    idx = torch.arange(L, device=device, dtype=torch.float64)
    T = torch.tril(rho ** (idx[:, None] - idx[None, :]).clamp(min=0)).to(torch.float32)  # T[t,s] = rho^(t-s), s<=t
    carry = (rho ** (idx + 1)).to(torch.float32)[:, None]
    sigma = math.sqrt(1.0 - rho * rho)
    out = torch.empty((n_tok, width), device=device, dtype=torch.float32)
    prev = torch.randn((1, width), generator=gen, device=device, dtype=torch.float32)
    for t0 in range(0, n_tok, L):
        n = min(L, n_tok - t0)
        eps = torch.randn((L, width), generator=gen, device=device, dtype=torch.float32) * sigma
        x = T @ eps + carry * prev
        out[t0:t0 + n] = x[:n]
        prev = x[L - 1:L]
    return out


def build(name: str, cfg: int, *, dtype, B, H, Hkv, D, S, seq_lens, top_k, lam=0.5,
          key_mode="iid", plant_mode="none", permute=False, spare_tokens=0,
          q_seed=None, device="cpu", poison=True) -> Workload:
    """Assemble one workload.

    key_mode: "iid" N(0,1) keys | "shift" N(0,1) + a per-(page, head) mean vector ~ N(0, 0.5^2) per dim
              | "ar1" smooth AR(1) trajectories (rho 0.95, unit variance) along time per (head, dim).
    plant_mode: "none" | "four" (4 pages per KV head each hold one key 4*q_dir + N(0,1))
              | "one_percent" (1% of pages per KV head hold 1-3 such keys), where
              q_dir = q[b, first head of the group] rescaled to RMS 1.
    spare_tokens: capacity reserved past seq_lens[b] for tokens appended later.
    poison: slots that hold no token yet (and unused pool pages) are filled with NaN,
            so anything that reads them shows up in the results.
    """
    base = 1000 * cfg
    G = H // Hkv
    seq_lens = [int(n) for n in seq_lens]
    assert len(seq_lens) == B and all(n >= 1 for n in seq_lens)
    cap_pages = [(n + spare_tokens + S - 1) // S for n in seq_lens]
    max_pages = max(cap_pages)
    pool = sum(cap_pages)

    q = torch.randn((B, H, D), generator=_gen(base if q_seed is None else q_seed, device), device=device,
                    dtype=torch.float32).to(dtype)

    ids = torch.randperm(pool, generator=_gen(base + 3)) if permute else torch.arange(pool)
    page_table = torch.zeros((B, max_pages), dtype=torch.int32)
    off = 0
    for b in range(B):
        page_table[b, :cap_pages[b]] = ids[off:off + cap_pages[b]].to(torch.int32)
        off += cap_pages[b]

    fill = float("nan") if poison else 0.0
    k_cache = torch.full((pool, Hkv, S, D), fill, device=device, dtype=dtype)
    v_cache = torch.full((pool, Hkv, S, D), fill, device=device, dtype=dtype)

    gk, gv, gp = _gen(base + 1, device), _gen(base + 2, device), _gen(base + 5)
    for b in range(B):
        N = seq_lens[b]
        P = (N + S - 1) // S
        if key_mode == "ar1":
            k = _ar1(P * S, Hkv * D, 0.95, gk, device).view(P, S, Hkv, D).permute(0, 2, 1, 3).contiguous()
        else:
            k = torch.randn((P, Hkv, S, D), generator=gk, device=device, dtype=torch.float32)
            if key_mode == "shift":
                k += 0.5 * torch.randn((P, Hkv, 1, D), generator=gk, device=device, dtype=torch.float32)
        v = torch.randn((P, Hkv, S, D), generator=gv, device=device, dtype=torch.float32)

        if plant_mode != "none":
            qf = q[b].to(torch.float32).view(Hkv, G, D)[:, 0, :]
            q_dir = qf / qf.norm(dim=-1, keepdim=True) * math.sqrt(D)  # [Hkv, D], RMS 1
            for h in range(Hkv):
                n_pl = 4 if plant_mode == "four" else max(1, round(0.01 * P))
                pages = torch.randperm(P, generator=gp)[:min(n_pl, P)].tolist()
                for p in pages:
                    n_valid = min(S, N - p * S)
                    n_keys = 1 if plant_mode == "four" else int(torch.randint(1, 4, (1,), generator=gp))
                    slots = torch.randperm(n_valid, generator=gp)[:min(n_keys, n_valid)].tolist()
                    for j in slots:
                        noise = torch.randn((D,), generator=gp, dtype=torch.float32).to(device)
                        k[p, h, j, :] = 4.0 * q_dir[h] + noise

        k = k.to(dtype)
        v = v.to(dtype)
        tail = N - (P - 1) * S
        if tail < S:  # slots past the last token hold no data yet
            k[P - 1, :, tail:, :] = fill
            v[P - 1, :, tail:, :] = fill
        phys = page_table[b, :P].to(torch.int64).to(device)
        k_cache[phys] = k
        v_cache[phys] = v
        del k, v

    return Workload(name=name, dtype=dtype, B=B, H=H, Hkv=Hkv, D=D, S=S, top_k=top_k, lam=lam, q=q,
                    k_cache=k_cache, v_cache=v_cache, page_table=page_table.to(device),
                    seq_lens=torch.tensor(seq_lens, dtype=torch.int32, device=device),
                    meta=dict(cfg=cfg, key_mode=key_mode, plant_mode=plant_mode, permute=permute,
                              spare_tokens=spare_tokens, cap_pages=cap_pages))


# ---- the five benchmark configurations (and scaled-down variants through the keyword overrides) ----

def config1(device="cpu", *, context=2048, top_k=16, poison=True) -> Workload:
    """Tiny fp32: B=1, 8 q / 2 KV heads, D=64, 2048 tokens in 128 pages of 16, k=16; iid keys,
    four planted keys per KV head; the query uses seed 0."""
    return build("c1_tiny_fp32", 1, dtype=torch.float32, B=1, H=8, Hkv=2, D=64, S=16, seq_lens=[context],
                 top_k=top_k, key_mode="iid", plant_mode="four", q_seed=0, device=device, poison=poison)


def config2(device="cpu", *, context=32768, top_k=128, poison=True) -> Workload:
    """Llama-3-8B-shaped bf16 decode: B=1, 32 q / 8 KV heads, D=128, 32768 tokens, S=16, k=128."""
    return build("c2_llama8b_bf16_32k", 2, dtype=torch.bfloat16, B=1, H=32, Hkv=8, D=128, S=16,
                 seq_lens=[context], top_k=top_k, key_mode="shift", plant_mode="one_percent",
                 device=device, poison=poison)


def config3(device="cpu", *, batch=16, context=131072, top_k=256, poison=True) -> Workload:
    """Batched bf16 decode: B=16 x 131072 tokens, S=16, k=256, page table = random permutation of one pool."""
    return build("c3_batched_bf16_128k", 3, dtype=torch.bfloat16, B=batch, H=32, Hkv=8, D=128, S=16,
                 seq_lens=[context] * batch, top_k=top_k, key_mode="shift", plant_mode="one_percent",
                 permute=True, device=device, poison=poison)


def config4(device="cpu", *, batch=32, min_context=4096, max_context=131072, top_k=64,
            spare_tokens=128, poison=True) -> Workload:
    """Ragged bf16 batch: lengths log-uniform in [4K, 128K], S=32, k=64, room for appended tokens."""
    u = torch.rand((batch,), generator=_gen(4000 + 4), dtype=torch.float64)
    lens = torch.exp(math.log(min_context) + u * (math.log(max_context) - math.log(min_context)))
    lens = lens.round().clamp(min_context, max_context).to(torch.int64).tolist()
    return build("c4_ragged_bf16", 4, dtype=torch.bfloat16, B=batch, H=32, Hkv=8, D=128, S=32, seq_lens=lens,
                 top_k=top_k, key_mode="shift", plant_mode="one_percent", permute=True,
                 spare_tokens=spare_tokens, device=device, poison=poison)


def config5(device="cpu", *, batch=4, context=262144, top_k=256, poison=True) -> Workload:
    """Speech-shaped bf16 decode: B=4, 16 q / 4 KV heads, D=128, 262144 tokens of AR(1) keys, S=16;
    top_k is swept over {64, 256, 1024} by the caller. Values are iid N(0,1)."""
    return build("c5_speech_bf16_256k", 5, dtype=torch.bfloat16, B=batch, H=16, Hkv=4, D=128, S=16,
                 seq_lens=[context] * batch, top_k=top_k, key_mode="ar1", plant_mode="none",
                 device=device, poison=poison)


CONFIGS = {1: config1, 2: config2, 3: config3, 4: config4, 5: config5}


def interleave_kv(wl: Workload) -> Workload:
    """The same cache contents with the K and V tiles of every (page, head) side by side in one buffer
    [num_phys_pages][Hkv][2][S][D]; k_cache / v_cache become strided views into it (same bits, other layout)."""
    kv = torch.stack([wl.k_cache, wl.v_cache], dim=2).contiguous()
    kw = dict(wl.__dict__)
    kw["k_cache"], kw["v_cache"] = kv[:, :, 0], kv[:, :, 1]
    kw["meta"] = dict(wl.meta, interleaved_kv=True)
    return Workload(**kw)


def append_tokens(wl: Workload, step: int) -> None:
    """Write one new (k, v) token per sequence into its next free slot and bump seq_lens (config 4's
    decode loop). Draws are seeded by (config, step); this is the serving engine's cache write."""
    dev = wl.k_cache.device
    g = _gen(1000 * wl.meta.get("cfg", 0) + 100 + step, dev)
    newk = torch.randn((wl.B, wl.Hkv, wl.D), generator=g, device=dev, dtype=torch.float32).to(wl.dtype)
    newv = torch.randn((wl.B, wl.Hkv, wl.D), generator=g, device=dev, dtype=torch.float32).to(wl.dtype)
    n = wl.seq_lens.to(torch.int64)
    cap = torch.tensor(wl.meta["cap_pages"], device=dev, dtype=torch.int64)
    assert bool(((n // wl.S) < cap).all()), "no capacity left for another token"
    phys = wl.page_table.to(torch.int64)[torch.arange(wl.B, device=dev), n // wl.S]
    slot = n % wl.S
    wl.k_cache[phys, :, slot, :] = newk
    wl.v_cache[phys, :, slot, :] = newv
    wl.seq_lens += 1
