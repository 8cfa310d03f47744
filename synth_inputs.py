"""Seeded synthetic decode workloads (inputs only: none of the method's arithmetic).

Serves both the HIP path and the CPU oracle; neither of them is imported here.
Shapes follow Llama-3-8B attention (32 query heads over 8 KV heads, head_dim 128).

Recipe, per (config id, layer):
  keys    fp16(N(0,1) * m) where m = 8 on 4 outlier channels drawn per (sequence, KV head), else 1
  values  fp16(N(0,1))
  planted tokens: every query head owns `planted` distinct positions of its KV head's
          sequence; all of them carry one key vector u (same distribution as the keys);
          the query of that head is fp16(u + 0.3 * N(0,1))
  seed    1000*config + 10*layer + tensor id (0 keys, 1 values, 2 outlier channels,
          3 planted positions, 4 planted vectors, 5 query noise, 6.. appended tokens)

Correlated variant (make_correlated_layer): what a real key cache looks like to a sampler that reads whole
code blocks - neighbouring tokens resemble each other.  The sequence is cut into runs whose lengths are
2^e, e uniform in 0..log2(run_max); every run has one direction vector c ~ N(0,1) (outlier channels x 8) and
its tokens are fp16(c + noise * N(0,1)); the query of every head is fp16(N(0,1)) with the outlier scaling.
Seeds: tensor ids 7 (run lengths), 8 (run vectors), 9 (noise and queries) of the same scheme.
"""
from dataclasses import dataclass

import torch


@dataclass(frozen=True)
class Workload:
    name: str
    config: int          # id used in the seed
    batch: int
    n_q_heads: int
    n_kv_heads: int
    n: int               # context tokens resident at the start
    bits: int
    group: int
    k: int               # top-k per KV head
    planted: int = 16    # planted tokens per query head
    head_dim: int = 128
    layers: int = 1
    evict_keep: int = 0  # M (0: no eviction)
    evict_every: int = 0
    steps: int = 1

    @property
    def gqa(self):
        return self.n_q_heads // self.n_kv_heads


CONFIGS = {
    1: Workload("cfg1-tiny-4k", 1, 1, 1, 1, 4096, 4, 32, 256, evict_keep=3072, evict_every=1),
    2: Workload("cfg2-llama3-8b-32k", 2, 1, 32, 8, 32 * 1024, 4, 32, 1024),
    3: Workload("cfg3-llama3-8b-128k-b4", 3, 4, 32, 8, 128 * 1024, 4, 32, 2048,
                evict_keep=128 * 1024, evict_every=16, steps=64),
    4: Workload("cfg4-llama3-8b-1m-32layers", 4, 1, 32, 8, 1 << 20, 4, 32, 4096, layers=32),
    5: Workload("cfg5-llama3-8b-4m-32layers-2bit", 5, 1, 32, 8, 1 << 22, 2, 64, 8192, layers=32,
                evict_keep=1 << 21, evict_every=1),
}


def _gen(device, seed):
    g = torch.Generator(device=device)
    g.manual_seed(int(seed))
    return g


def _randn(shape, device, seed, chunk_rows=1 << 18):
    """fp16 N(0,1) of `shape`, generated in row chunks so that the fp32 intermediate stays small."""
    g = _gen(device, seed)
    out = torch.empty(shape, dtype=torch.float16, device=device)
    flat = out.view(-1, shape[-1])
    for r0 in range(0, flat.shape[0], chunk_rows):
        r1 = min(flat.shape[0], r0 + chunk_rows)
        flat[r0:r1] = torch.randn((r1 - r0, shape[-1]), generator=g, device=device,
                                  dtype=torch.float32).to(torch.float16)
    return out


def outlier_scale(w: Workload, layer=0, device="cpu"):
    """fp32 [B, Hkv, D]: 8.0 on the 4 outlier channels of each (sequence, KV head), else 1.0."""
    g = _gen("cpu", 1000 * w.config + 10 * layer + 2)
    m = torch.ones(w.batch, w.n_kv_heads, w.head_dim)
    for b in range(w.batch):
        for h in range(w.n_kv_heads):
            ch = torch.randperm(w.head_dim, generator=g)[:4]
            m[b, h, ch] = 8.0
    return m.to(device)


def make_layer(w: Workload, layer=0, device="cpu", want_values=True):
    """Returns dict with
       keys   fp16 [B, Hkv, n, D]      values fp16 [B, Hkv, n, D] (or None)
       q      fp16 [B, Hq, D]          planted int64 [B, Hq, planted] (positions)"""
    base = 1000 * w.config + 10 * layer
    B, Hq, Hkv, D, n, G = w.batch, w.n_q_heads, w.n_kv_heads, w.head_dim, w.n, w.gqa
    m = outlier_scale(w, layer, device)                                   # [B,Hkv,D]
    keys = _randn((B, Hkv, n, D), device, base + 0)
    # apply outliers in chunks (in place, fp16 <- fp32 product rounded once)
    for b in range(B):
        for h in range(Hkv):
            ch = torch.nonzero(m[b, h] > 1.0).flatten()
            keys[b, h][:, ch] = (keys[b, h][:, ch].float() * 8.0).to(torch.float16)
    values = _randn((B, Hkv, n, D), device, base + 1) if want_values else None

    gp = _gen("cpu", base + 3)
    planted = torch.empty(B, Hq, w.planted, dtype=torch.int64)
    for b in range(B):
        for h in range(Hkv):
            p = torch.randperm(n, generator=gp)[: w.planted * G].view(G, w.planted)
            planted[b, h * G:(h + 1) * G] = p
    gu = _gen("cpu", base + 4)
    u = torch.randn(B, Hq, D, generator=gu)                               # planted vectors
    u = (u * m.cpu().repeat_interleave(G, dim=1)).to(torch.float16)
    ge = _gen("cpu", base + 5)
    q = (u.float() + 0.3 * torch.randn(B, Hq, D, generator=ge)).to(torch.float16)
    u_dev = u.to(device)
    for b in range(B):
        for hq in range(Hq):
            keys[b, hq // G, planted[b, hq].to(device)] = u_dev[b, hq]
    return {"keys": keys, "values": values, "q": q.to(device), "planted": planted}


def make_correlated_layer(w: Workload, layer=0, device="cpu", run_max=4096, noise=0.3):
    """Keys whose scores are strongly correlated inside runs of up to `run_max` neighbouring slots (see the
    module text).  Returns dict with keys fp16 [B, Hkv, n, D], q fp16 [B, Hq, D], runs int64 [B, Hkv] (count)."""
    base = 1000 * w.config + 10 * layer
    B, Hq, Hkv, D, n, G = w.batch, w.n_q_heads, w.n_kv_heads, w.head_dim, w.n, w.gqa
    m = outlier_scale(w, layer, device)
    gl, gv, gn = _gen("cpu", base + 7), _gen(device, base + 8), _gen(device, base + 9)
    e_max = max(0, int(run_max).bit_length() - 1)
    keys = torch.empty(B, Hkv, n, D, dtype=torch.float16, device=device)
    runs = torch.zeros(B, Hkv, dtype=torch.int64)
    for b in range(B):
        for h in range(Hkv):
            ends = torch.zeros(0, dtype=torch.int64)
            while ends.numel() == 0 or int(ends[-1]) < n:            # run lengths 2^e until the row is covered
                more = torch.cumsum(2 ** torch.randint(0, e_max + 1, (4096,), generator=gl), 0)
                ends = torch.cat([ends, more + (int(ends[-1]) if ends.numel() else 0)])
            ends = ends[: int(torch.searchsorted(ends, n)) + 1]
            runs[b, h] = ends.numel()
            c = torch.randn(ends.numel(), D, generator=gv, device=device) * m[b, h]
            run_of = torch.searchsorted(ends.to(device), torch.arange(n, device=device), right=True)
            for r0 in range(0, n, 1 << 18):
                r1 = min(n, r0 + (1 << 18))
                e = torch.randn(r1 - r0, D, generator=gn, device=device)
                keys[b, h, r0:r1] = (c[run_of[r0:r1]] + noise * e).to(torch.float16)
    q = (torch.randn(B, Hq, D, generator=gn, device=device) * m.repeat_interleave(G, dim=1)).to(torch.float16)
    return {"keys": keys, "q": q, "runs": runs}


def make_step(w: Workload, layer, step, device="cpu"):
    """One appended token per (sequence, KV head) and a fresh query for decode step `step`:
       k_new fp16 [B,Hkv,1,D], v_new fp16 [B,Hkv,1,D], q fp16 [B,Hq,D]."""
    base = 1000 * w.config + 10 * layer + 6
    g = _gen("cpu", base * 100003 + step)
    B, Hq, Hkv, D = w.batch, w.n_q_heads, w.n_kv_heads, w.head_dim
    m = outlier_scale(w, layer, "cpu")
    k_new = (torch.randn(B, Hkv, 1, D, generator=g) * m[:, :, None, :]).to(torch.float16)
    v_new = torch.randn(B, Hkv, 1, D, generator=g).to(torch.float16)
    q = (torch.randn(B, Hq, D, generator=g) * m.repeat_interleave(w.gqa, dim=1)).to(torch.float16)
    return k_new.to(device), v_new.to(device), q.to(device)
