"""Seeded synthetic decode-step workloads shaped like the paper's models.

The paper measures on LongBench / PG-19 prompts through LongChat-7B, OPT-6.7B
and Yarn-Llama-2-13B (Sec. 6.1).  Neither those datasets nor the weights are
used here.  What is kept is the attention *shape* of those models and the
qualitative structure the paper reports: a small share of tokens carries most
of the attention mass (Sec. 3.3, Fig. 3), unimportant tokens come in long
contiguous runs ("attention deserts", Sec. 3.5, Fig. 7) and the first layers
are flatter than deep ones (Sec. 3.5, Fig. 8).

Everything here is input generation.  There is no abstract, score, selection
or attention arithmetic in this module: the oracle and the HIP library both
receive exactly the tensors built here and share nothing else.

Random streams: small structural draws (ranks, chunk sizes, planted positions)
come from numpy Philox keyed by (seed, config, layer, sequence); the bulk
Gaussian noise comes from a torch.Generator on the requested device seeded with
the same key, so big caches can be generated directly in HBM.  CPU and GPU
streams differ; a parity test always hands the same tensors to both sides.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import Dict, List, Optional, Sequence

import numpy as np
import torch

BASE_SEED = 250620187

# name -> recipe.  "sizes" is a set of allowed chunk sizes, "size_range" an
# inclusive integer range; exactly one of them is given.
CONFIGS: Dict[str, dict] = {
    # Tiny fp32 step: 128 fixed chunks of 32, pick the top 16 chunks.
    "c0": dict(layers=1, batch=1, hq=8, hkv=8, d=128, n_ctx=4096, dtype="f32",
               sizes=(32,), max_chunks=16, token_budget=0, recipe="planted16"),
    # Llama-2-7B-shaped MHA, fp16, 32K, four outlier key channels.
    "c1": dict(layers=32, batch=1, hq=32, hkv=32, d=128, n_ctx=32768, dtype="f16",
               sizes=(16, 32, 64, 128), max_chunks=0, token_budget=2048,
               recipe="zipf", zipf=(1.1, 1.1), outlier_channels=4, outlier_scale=8.0),
    # Llama-3-8B-shaped GQA, bf16, 128K.
    "c2": dict(layers=32, batch=1, hq=32, hkv=8, d=128, n_ctx=131072, dtype="bf16",
               sizes=(16, 32, 64, 128, 256), max_chunks=0, token_budget=4096,
               recipe="zipf", zipf=(0.6, 1.3)),
    # Batched long-context decode: c2 shape, 16 independent sequences.
    "c3": dict(layers=32, batch=16, hq=32, hkv=8, d=128, n_ctx=131072, dtype="bf16",
               size_range=(16, 256), max_chunks=0, token_budget=4096,
               recipe="zipf", zipf=(0.6, 1.3)),
    # Compressed-KV stress: 512K context (values generated in bf16, quantised
    # by the caller of the quantised store).
    "c4": dict(layers=32, batch=1, hq=32, hkv=8, d=128, n_ctx=524288, dtype="bf16",
               size_range=(32, 512), max_chunks=0, token_budget=8192,
               recipe="zipf", zipf=(0.6, 1.3)),
}

_TORCH_DTYPE = {"f32": torch.float32, "f16": torch.float16, "bf16": torch.bfloat16}


@dataclass
class Case:
    """One layer of one decode step for `batch` sequences."""
    name: str
    layer: int
    dtype: str                      # "f32" | "f16" | "bf16"
    batch: int
    hq: int
    hkv: int
    d: int
    n_ctx: int
    K: torch.Tensor                 # [B, Hkv, N, D]
    V: torch.Tensor                 # [B, Hkv, N, D]
    q: torch.Tensor                 # [B, Hq, D]
    chunk_off: torch.Tensor         # int32 [B, c_max + 1], rows padded with N
    n_chunks: torch.Tensor          # int32 [B]
    c_max: int
    max_chunks: int                 # <= 0: unlimited
    token_budget: int               # <= 0: unlimited
    k_max: int                      # row stride for selected-index lists
    planted: Optional[np.ndarray] = None   # c0: planted token positions
    extra: dict = field(default_factory=dict)

    @property
    def g(self) -> int:
        return self.hq // self.hkv


def _key(seed: int, cfg: str, layer: int, seq: int, stream: int) -> List[int]:
    return [seed & 0xFFFFFFFF, int(cfg[1:]) if cfg[1:].isdigit() else 99, layer, seq * 8 + stream]


def _np_rng(seed, cfg, layer, seq, stream=0) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(key=np.random.SeedSequence(_key(seed, cfg, layer, seq, stream)).generate_state(2, dtype=np.uint64)))


def _torch_gen(device, seed, cfg, layer, seq) -> torch.Generator:
    g = torch.Generator(device=device)
    s = int(np.random.SeedSequence(_key(seed, cfg, layer, seq, 7)).generate_state(1, dtype=np.uint64)[0] >> 1)
    g.manual_seed(s)
    return g


# --------------------------------------------------------------------------
# chunk boundaries
# --------------------------------------------------------------------------

def uniform_boundaries(n_ctx: int, size: int) -> np.ndarray:
    """Boundaries of fixed-size chunks; the last chunk takes the ragged tail."""
    off = list(range(0, n_ctx, size)) + [n_ctx]
    return np.asarray(off, dtype=np.int32)


def make_boundaries(n_ctx: int, rng: np.random.Generator, *, sizes: Optional[Sequence[int]] = None,
                    size_range: Optional[Sequence[int]] = None, heavy: Optional[np.ndarray] = None,
                    depth: float = 0.5) -> np.ndarray:
    """Variable chunk boundaries that tile [0, n_ctx) exactly.

    The context is cut into aligned blocks of the largest allowed size; each
    block is filled with chunks whose size is drawn with a tilt: blocks that
    hold heavy tokens and shallow layers (depth -> 0) prefer small chunks,
    desert blocks in deep layers (depth -> 1) prefer large ones.
    `heavy[t]` is a bool per token; None means no locality.
    """
    if (sizes is None) == (size_range is None):
        raise ValueError("give exactly one of sizes / size_range")
    if sizes is not None:
        lo, hi = min(sizes), max(sizes)
        cand = np.asarray(sorted(sizes), dtype=np.int64)
    else:
        lo, hi = int(size_range[0]), int(size_range[1])
        cand = None
    block = hi
    off = [0]
    n_blocks = (n_ctx + block - 1) // block
    for blk in range(n_blocks):
        b0 = blk * block
        b1 = min(n_ctx, b0 + block)
        is_heavy = bool(heavy[b0:b1].any()) if heavy is not None else False
        tilt = 1.5 if is_heavy else (1.0 - 2.5 * depth)
        if depth < 0.05:
            tilt = 2.0
        if cand is not None:
            w = np.exp(-tilt * np.arange(len(cand)))
            s = int(rng.choice(cand, p=w / w.sum()))
            pos = b0
            while pos < b1:
                pos = min(b1, pos + s)
                off.append(pos)
        else:
            # target size log-uniform in [lo, hi] with the same tilt, then a
            # random partition of the block around that target
            u = rng.random()
            frac = u ** math.exp(tilt * 0.6)          # tilt > 0 pushes toward lo
            target = math.exp(math.log(lo) + frac * (math.log(hi) - math.log(lo)))
            pos = b0
            while pos < b1:
                s_lo = max(lo, int(target * 0.6))
                s_hi = min(hi, max(s_lo, int(target * 1.6)))
                s = int(rng.integers(s_lo, s_hi + 1))
                rem = b1 - pos
                if rem - s < lo:          # do not leave a fragment below lo
                    s = rem
                pos += s
                off.append(pos)
    out = np.asarray(off, dtype=np.int32)
    assert out[0] == 0 and out[-1] == n_ctx and np.all(np.diff(out) > 0)
    return out


def pack_boundaries(offs: Sequence[np.ndarray], n_ctx: int, c_max: Optional[int] = None):
    """Stack per-sequence boundary lists into [B, c_max+1] padded with n_ctx."""
    counts = np.asarray([len(o) - 1 for o in offs], dtype=np.int32)
    cm = int(counts.max()) if c_max is None else int(c_max)
    if cm < counts.max():
        raise ValueError("c_max too small")
    packed = np.full((len(offs), cm + 1), n_ctx, dtype=np.int32)
    for b, o in enumerate(offs):
        packed[b, : len(o)] = o
    return packed, counts, cm


# --------------------------------------------------------------------------
# values
# --------------------------------------------------------------------------

def _zipf_ranks(n_ctx: int, rng: np.random.Generator, seg: int = 64) -> np.ndarray:
    """Rank 1..N per token, assigned segment-wise so that heavy tokens (small
    ranks) sit in contiguous runs of `seg` tokens."""
    n_seg = (n_ctx + seg - 1) // seg
    seg_rank = rng.permutation(n_seg).astype(np.int64)
    within = np.argsort(rng.random((n_seg, seg)), axis=1).astype(np.int64)
    ranks = (seg_rank[:, None] * seg + within).reshape(-1)[:n_ctx]
    # compress to a permutation of 1..N (the trim may leave gaps)
    order = np.argsort(ranks, kind="stable")
    out = np.empty(n_ctx, dtype=np.int64)
    out[order] = np.arange(1, n_ctx + 1)
    return out


def _gen_sequence(cfg_name: str, cfg: dict, layer: int, seq: int, n_ctx: int, device, seed: int,
                  K_out: torch.Tensor, V_out: torch.Tensor, q_out: torch.Tensor):
    """Fill K_out/V_out [Hkv,N,D] and q_out [Hq,D] in place; return (chunk_off, planted)."""
    hq, hkv, d = cfg["hq"], cfg["hkv"], cfg["d"]
    g = hq // hkv
    rng = _np_rng(seed, cfg_name, layer, seq)
    tg = _torch_gen(device, seed, cfg_name, layer, seq)
    layers = max(1, cfg["layers"])
    depth = layer / (layers - 1) if layers > 1 else 0.5

    # queries: one shared direction per kv head plus per-head noise (GQA)
    shared = torch.randn(hkv, d, generator=tg, device=device, dtype=torch.float32)
    if g > 1:
        noise = 0.5 * torch.randn(hkv, g, d, generator=tg, device=device, dtype=torch.float32)
        q = (shared[:, None, :] + noise).reshape(hq, d)
    else:
        q = shared.clone()
    q_out.copy_(q.to(q_out.dtype))

    planted = None
    heavy = None
    # noise, generated per kv head to bound the fp32 staging footprint
    if cfg["recipe"] == "planted16":
        size = cfg["sizes"][0]
        n_chunks = (n_ctx + size - 1) // size
        n_plant = min(16, n_chunks)
        chunks = np.sort(rng.choice(n_chunks, size=n_plant, replace=False))
        planted = np.asarray([min(n_ctx - 1, c * size + int(rng.integers(0, size))) for c in chunks], dtype=np.int64)
        add = None
    else:
        s_lo, s_hi = cfg["zipf"]
        s_exp = s_lo + (s_hi - s_lo) * depth
        ranks = _zipf_ranks(n_ctx, rng)
        a = -s_exp * np.log(ranks.astype(np.float64))
        a = a - a.mean()
        heavy = ranks <= max(1, int(0.2 * n_ctx))
        add = torch.from_numpy(a.astype(np.float32)).to(device)          # [N]

    for h in range(hkv):
        kn = torch.randn(n_ctx, d, generator=tg, device=device, dtype=torch.float32)
        if cfg.get("outlier_channels"):
            ch_rng = _np_rng(seed, cfg_name, layer, 0, stream=3)         # fixed per layer
            ch = ch_rng.choice(d, size=cfg["outlier_channels"], replace=False)
            kn[:, torch.from_numpy(ch).to(device)] *= cfg["outlier_scale"]
        if add is not None:
            u = shared[h]
            # raising the scaled logit q.k/sqrt(d) of token t by a_t
            kn += (add * math.sqrt(d))[:, None] * (u / (u * u).sum())[None, :]
        K_out[h].copy_(kn.to(K_out.dtype))
        del kn
        V_out[h].copy_(torch.randn(n_ctx, d, generator=tg, device=device, dtype=torch.float32).to(V_out.dtype))
    if planted is not None:
        pt = torch.from_numpy(planted).to(device)
        # the stored query (already rounded to the cache dtype) times four
        qh = q_out.to(torch.float32).reshape(hkv, g, d)[:, 0, :]
        K_out[:, pt, :] = (4.0 * qh)[:, None, :].to(K_out.dtype).expand(hkv, len(planted), d)

    if cfg.get("sizes") is not None and len(cfg["sizes"]) == 1:
        off = uniform_boundaries(n_ctx, cfg["sizes"][0])
    else:
        off = make_boundaries(n_ctx, _np_rng(seed, cfg_name, layer, seq, stream=1), sizes=cfg.get("sizes"),
                              size_range=cfg.get("size_range"), heavy=heavy, depth=depth)
    return off, planted, heavy


def make_case(config: str, layer: int = 0, *, device="cpu", seed: int = BASE_SEED, batch: Optional[int] = None,
              n_ctx: Optional[int] = None, hq: Optional[int] = None, hkv: Optional[int] = None,
              dtype: Optional[str] = None, token_budget: Optional[int] = None,
              max_chunks: Optional[int] = None, first_seq: int = 0) -> Case:
    """Build one layer of config `config` ("c0".."c4"), optionally reduced
    (n_ctx, batch, heads) or re-typed for small parity cases.  The recipe is
    unchanged by the overrides."""
    cfg = dict(CONFIGS[config])
    for k, v in (("batch", batch), ("n_ctx", n_ctx), ("hq", hq), ("hkv", hkv), ("dtype", dtype),
                 ("token_budget", token_budget), ("max_chunks", max_chunks)):
        if v is not None:
            cfg[k] = v
    B, Hq, Hkv, D, N = cfg["batch"], cfg["hq"], cfg["hkv"], cfg["d"], cfg["n_ctx"]
    if Hq % Hkv:
        raise ValueError("hq must be a multiple of hkv")
    tdt = _TORCH_DTYPE[cfg["dtype"]]
    K = torch.empty(B, Hkv, N, D, dtype=tdt, device=device)
    V = torch.empty(B, Hkv, N, D, dtype=tdt, device=device)
    q = torch.empty(B, Hq, D, dtype=tdt, device=device)
    offs, planted, heavy = [], None, []
    for b in range(B):
        off, pl, hv = _gen_sequence(config, cfg, layer, first_seq + b, N, device, seed, K[b], V[b], q[b])
        offs.append(off)
        heavy.append(hv if hv is not None else np.zeros(N, dtype=bool))
        planted = pl if pl is not None else planted
    # the chunk capacity is rounded up to a multiple of 32: the abstracts of every (sequence, kv head)
    # then start at the same offset inside 16 KiB (what the score kernel's 16 KiB groups like best)
    most = max(len(o) - 1 for o in offs)
    packed, counts, c_max = pack_boundaries(offs, N, c_max=(most + 31) // 32 * 32)
    smallest = min(int(np.diff(o).min()) for o in offs)
    if cfg["max_chunks"] > 0:
        k_max = min(c_max, cfg["max_chunks"])
    elif cfg["token_budget"] > 0:
        k_max = min(c_max, cfg["token_budget"] // max(1, smallest))
    else:
        k_max = c_max
    k_max = max(1, k_max)
    return Case(name=config, layer=layer, dtype=cfg["dtype"], batch=B, hq=Hq, hkv=Hkv, d=D, n_ctx=N,
                K=K, V=V, q=q,
                chunk_off=torch.from_numpy(packed).to(device), n_chunks=torch.from_numpy(counts).to(device),
                c_max=c_max, max_chunks=cfg["max_chunks"], token_budget=cfg["token_budget"], k_max=k_max,
                planted=planted, extra={"heavy": np.stack(heavy)})


def make_desert_keys(batch: int, hkv: int, g: int, n_ctx: int, *, clusters: int = 24, cluster_len=(8, 64),
                     dtype: str = "bf16", device="cpu", seed: int = BASE_SEED):
    """Keys and queries with the structure Sec. 3.5 reports for deep layers: a few short runs of
    tokens that the query attends to, separated by long "attention deserts".

    Per (sequence, kv head): keys 0.1 * N(0,1); `clusters` runs of cluster_len[0]..cluster_len[1]
    tokens at distinct random places get +6 * q_dir added, q_dir being the unit direction shared by the
    group's query heads (query head j = that direction * 4 + N(0, 0.05)).  Returns (K [B,Hkv,N,128],
    q [B,Hkv*g,128], hot bool numpy [B,Hkv,N] marking the planted tokens)."""
    tdt = _TORCH_DTYPE[dtype]
    D = 128
    K = torch.empty(batch, hkv, n_ctx, D, dtype=tdt, device=device)
    q = torch.empty(batch, hkv * g, D, dtype=tdt, device=device)
    hot = np.zeros((batch, hkv, n_ctx), dtype=bool)
    for b in range(batch):
        for h in range(hkv):
            rng = _np_rng(seed, "desert", h, b)
            gen_t = _torch_gen(device, seed, "desert", h, b)
            direction = torch.randn(D, generator=gen_t, device=device)
            direction = direction / direction.norm()
            keys = 0.1 * torch.randn(n_ctx, D, generator=gen_t, device=device)
            slot = n_ctx // clusters
            for c in range(clusters):
                length = int(rng.integers(cluster_len[0], cluster_len[1] + 1))
                start = c * slot + int(rng.integers(0, max(1, slot - length)))
                hot[b, h, start:start + length] = True
            mask = torch.from_numpy(hot[b, h]).to(device)
            keys[mask] += 6.0 * direction
            K[b, h] = keys.to(tdt)
            qs = 4.0 * direction[None, :] + 0.05 * torch.randn(g, D, generator=gen_t, device=device)
            q[b, h * g:(h + 1) * g] = qs.to(tdt)
    return K, q, hot
