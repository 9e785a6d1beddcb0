"""Seeded synthetic inputs shaped like the paper's workloads.

Serves both the CPU oracle's tests and the GPU path: every tensor is generated
once, materialised in the kernel dtype, and the same buffers go to both sides.
Nothing here is part of the method: only random draws, the cluster structure
of image tokens, and the Q/K/V projections that turn hidden states into
attention operands.  Datasets and model weights of the paper's evaluation are
not available; these stand in for them (shapes and value distributions only).
"""
from __future__ import annotations

import math

import torch

from .configs import Workload

TORCH_DTYPE = {"bf16": torch.bfloat16, "f32": torch.float32}


def _gen(seed: int, device) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(int(seed) & 0x7FFFFFFFFFFFFFFF)
    return g


def _mix(seed: int, *ids: int) -> int:
    """Substream id from (seed, tensor id, layer, ...): a fixed integer hash."""
    x = (seed + 0x9E3779B97F4A7C15) & 0xFFFFFFFFFFFFFFFF
    for i in ids:
        x ^= (i + 0x9E3779B97F4A7C15 + ((x << 6) & 0xFFFFFFFFFFFFFFFF) + (x >> 2)) & 0xFFFFFFFFFFFFFFFF
        x = (x * 0xBF58476D1CE4E5B9) & 0xFFFFFFFFFFFFFFFF
    return x >> 1


def image_hidden(w: Workload, n_img: int, layer: int, device="cpu") -> torch.Tensor:
    """[B, n_img, C] fp32: cluster centre N(0, I) + noise_sigma * N(0, I) per token."""
    g = _gen(_mix(w.seed, 1, layer), device)
    B, C = w.batch, w.hidden
    if w.cluster_tile:
        n_tiles = (n_img + w.cluster_tile - 1) // w.cluster_tile
        centres = torch.randn(B, n_tiles * w.n_clusters, C, generator=g, device=device)
        local = torch.randint(0, w.n_clusters, (B, n_img), generator=g, device=device)
        tile = (torch.arange(n_img, device=device) // w.cluster_tile)[None, :]
        which = tile * w.n_clusters + local
    else:
        centres = torch.randn(B, w.n_clusters, C, generator=g, device=device)
        which = torch.randint(0, w.n_clusters, (B, n_img), generator=g, device=device)
    rows = torch.gather(centres, 1, which[:, :, None].expand(B, n_img, C))
    rows = rows + w.noise_sigma * torch.randn(B, n_img, C, generator=g, device=device)
    return rows


def layer_inputs(w: Workload, layer: int = 0, n_img: int | None = None, device="cpu",
                 with_v: bool = True) -> dict:
    """Inputs of the token-reduction step at one decoder layer.

    hidden [B,N,C], q [B,T,Hq,d] (instruction rows only), k, v [B,N,Hkv,d],
    pos [B,N,1] int32, all in the workload dtype; N = n_sys + n_img + n_text.
    """
    n_img = w.n_img if n_img is None else n_img
    dt = TORCH_DTYPE[w.dtype]
    B, C, d = w.batch, w.hidden, w.head_dim
    g = _gen(_mix(w.seed, 2, layer), device)
    sys_rows = torch.randn(B, w.n_sys, C, generator=g, device=device)
    txt_rows = torch.randn(B, w.n_text, C, generator=g, device=device)
    hidden = torch.cat([sys_rows, image_hidden(w, n_img, layer, device), txt_rows], dim=1).to(dt)
    std = 1.0 / math.sqrt(C)
    wq = (std * torch.randn(C, w.n_q_heads * d, generator=g, device=device)).to(dt)
    wk = (std * torch.randn(C, w.n_kv_heads * d, generator=g, device=device)).to(dt)
    hf = hidden.float()
    N = hidden.shape[1]
    q = (hf[:, w.n_sys + n_img:] @ wq.float()).view(B, w.n_text, w.n_q_heads, d)
    k = (hf @ wk.float()).view(B, N, w.n_kv_heads, d)
    if w.salient_frac > 0:
        # a shared direction per KV head: instruction queries and the salient image
        # keys both get a * u, which shifts their mean scaled logit by salient_bias
        a = math.sqrt(w.salient_bias * math.sqrt(d))
        u = torch.randn(B, 1, w.n_kv_heads, d, generator=g, device=device)
        u = u / u.norm(dim=-1, keepdim=True)
        n_sal = int(round(w.salient_frac * n_img))
        sal = torch.stack([torch.randperm(n_img, generator=g, device=device)[:n_sal] for _ in range(B)])
        mask = torch.zeros(B, N, 1, 1, device=device)
        mask.scatter_(1, (sal + w.n_sys)[:, :, None, None], 1.0)
        k = k + a * mask * u
        q = q + a * u.repeat_interleave(w.group, dim=2)
    if w.concentration:
        # Attention concentration that grows with depth (the paper's pilot study): every image token j gets a
        # salience z_j (standard normal over the tokens) shared by all heads and all instruction rows.  Per KV head a unit direction u:
        # the instruction queries get their component along u replaced by a = d^(1/4), the image keys get
        # a * sigma(layer) * z_j * u added, so every (row, head) logit of token j is shifted by sigma * z_j and the
        # attention the tokens receive is close to log-normal with spread sigma (linear in relative depth).
        s0, s1 = w.concentration
        sigma = s0 + (s1 - s0) * (layer / max(w.layers - 1, 1))
        a = float(d) ** 0.25
        u = torch.randn(B, 1, w.n_kv_heads, d, generator=g, device=device)
        u = u / u.norm(dim=-1, keepdim=True)
        # the saliences are the normal quantiles of an even grid, dealt to the tokens at random -- the same deal at
        # every layer (a token that stands out early stands out later), so that only sigma changes with depth
        gz = _gen(_mix(w.seed, 5, n_img), device)
        grid = (torch.arange(n_img, device=device, dtype=torch.float64) + 0.5) / n_img
        zq = torch.special.ndtri(grid).float()
        z = torch.stack([zq[torch.randperm(n_img, generator=gz, device=device)] for _ in range(B)]).view(B, n_img, 1, 1)
        k[:, w.n_sys:w.n_sys + n_img] = k[:, w.n_sys:w.n_sys + n_img] + a * sigma * z * u
        uq = u.repeat_interleave(w.group, dim=2)
        q = q - (q * uq).sum(dim=-1, keepdim=True) * uq + a * uq
    out = {"hidden": hidden, "q": q.to(dt).contiguous(), "k": k.to(dt).contiguous(),
           "pos": torch.arange(N, dtype=torch.int32, device=device).view(1, N, 1).expand(B, N, 1).contiguous()}
    if with_v:
        wv = (std * torch.randn(C, w.n_kv_heads * d, generator=g, device=device)).to(dt)
        out["v"] = (hf @ wv.float()).view(B, N, w.n_kv_heads, d).to(dt).contiguous()
    return out


def cache_state(w: Workload, length: int, l_max: int, layer: int = 0, device="cpu",
                n_protected: int | None = None, ragged: bool = False) -> dict:
    """A per-head KV cache as it stands after prefill compression.

    k, v [B,Hkv,Lmax,d] N(0,1); score f32 (skewed positive: a few dominant
    entries); kind u8 (first n_protected slots protected text, the rest image);
    orig_pos i32; len [B,Hkv] (all equal to `length`, or ragged below it).
    """
    dt = TORCH_DTYPE[w.dtype]
    B, H, d = w.batch, w.n_kv_heads, w.head_dim
    g = _gen(_mix(w.seed, 3, layer), device)
    n_protected = (w.n_sys + w.n_text) if n_protected is None else n_protected
    n_protected = min(n_protected, length)
    k = torch.randn(B, H, l_max, d, generator=g, device=device).to(dt)
    v = torch.randn(B, H, l_max, d, generator=g, device=device).to(dt)
    score = torch.rand(B, H, l_max, generator=g, device=device).pow(6.0) * 0.5
    kind = torch.ones(B, H, l_max, dtype=torch.uint8, device=device)
    kind[:, :, :n_protected] = 0
    pos = torch.arange(l_max, dtype=torch.int32, device=device).view(1, 1, l_max).expand(B, H, l_max).contiguous()
    if ragged:
        lens = torch.randint(max(1, length // 2), length + 1, (B, H), generator=g, device=device).to(torch.int32)
        lens[0, 0] = length
    else:
        lens = torch.full((B, H), length, dtype=torch.int32, device=device)
    return {"k": k, "v": v, "score": score, "kind": kind, "pos": pos, "len": lens}


class DecodeStream:
    """q_t, k_t, v_t of successive decode steps at one layer.

    Per (batch, KV head) a mean m_t follows a random walk with step
    drift_sigma; q_t = m_t + N(0,I) for each query head of the group,
    k_t = m_t + N(0,I), v_t = N(0,I).
    """

    def __init__(self, w: Workload, layer: int = 0, device="cpu"):
        self.w, self.device = w, device
        self.g = _gen(_mix(w.seed, 4, layer), device)
        self.mean = torch.zeros(w.batch, w.n_kv_heads, w.head_dim, device=device)

    def next(self):
        w, dt = self.w, TORCH_DTYPE[self.w.dtype]
        B, H, d, G = w.batch, w.n_kv_heads, w.head_dim, w.group
        if w.drift_sigma > 0:
            self.mean = self.mean + w.drift_sigma * torch.randn(B, H, d, generator=self.g, device=self.device)
        q = self.mean.repeat_interleave(G, dim=1) + torch.randn(B, H * G, d, generator=self.g, device=self.device)
        k = self.mean + torch.randn(B, H, d, generator=self.g, device=self.device)
        v = torch.randn(B, H, d, generator=self.g, device=self.device)
        return q.to(dt), k.to(dt), v.to(dt)

    def many(self, n: int):
        """n consecutive steps drawn in one go: q [n,B,Hq,d], k, v [n,B,Hkv,d].  The same law as n calls of
        next() and the running mean carries on, but the draws come in another order, so the values are not
        those n calls would give."""
        w, dt = self.w, TORCH_DTYPE[self.w.dtype]
        B, H, d, G = w.batch, w.n_kv_heads, w.head_dim, w.group
        mean = self.mean[None].expand(n, B, H, d)
        if w.drift_sigma > 0:
            walk = torch.cumsum(w.drift_sigma * torch.randn(n, B, H, d, generator=self.g, device=self.device), dim=0)
            mean = mean + walk
            self.mean = mean[-1].clone()
        q = mean.repeat_interleave(G, dim=2) + torch.randn(n, B, H * G, d, generator=self.g, device=self.device)
        k = mean + torch.randn(n, B, H, d, generator=self.g, device=self.device)
        v = torch.randn(n, B, H, d, generator=self.g, device=self.device)
        return q.to(dt), k.to(dt), v.to(dt)
