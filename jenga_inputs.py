"""Seeded synthetic Q/K/V for the attention-carving path, and the workload table.

This module serves both the HIP library's callers and the CPU oracle's callers; it holds
none of the method's arithmetic (no curve, no pooling, no selection, no attention).

The tensors stand in for the activations of a video DiT (HunyuanVideo / Wan2.1 in the
paper's experiments), which would need the models' weights.  Recipe, per tensor X in
{Q, K, V}, head g, channel c and vision token (t, h, w):

    X = sum_{s=1..4} A[X,g,s,c] * sin(2*pi*(ft[g,s]*t/T + fh[g,s]*h/H + fw[g,s]*w/W) + phi[X,g,s,c])
        + 0.5 * eps,      eps ~ N(0, 1)

with amplitudes A ~ N(0,1), phases uniform in [0, 2*pi), and spatial frequencies uniform in
[0.5, 3] cycles per axis that Q and K of one head share (so block scores have structure:
local, striped and global heads).  Text tokens are i.i.d. N(0, 1).  Values are computed in
float32 and rounded once to bfloat16; every consumer reads those bits.

Layout: [batch, N_v + N_c, heads, head_dim], vision tokens in (t, h, w) row-major order
(w fastest) followed by the text tokens: what a DiT's QKV projection yields.
"""
import math
import numpy as np
import torch

# name -> grid, text tokens, heads, head_dim, block, top-k ratio, cumulative-probability cut
WORKLOADS = {
    "tiny":        dict(T=4,  H=8,  W=8,  n_text=32,  batch=1, heads=2,  head_dim=64,  block=32,  topk=0.25, p=0.3),
    "small":       dict(T=8,  H=16, W=16, n_text=64,  batch=1, heads=8,  head_dim=128, block=128, topk=0.30, p=0.3),
    "wan480p":     dict(T=21, H=30, W=52, n_text=512, batch=1, heads=40, head_dim=128, block=128, topk=0.30, p=0.3),
    "hy_lowres":   dict(T=33, H=24, W=42, n_text=256, batch=1, heads=24, head_dim=128, block=128, topk=0.30, p=0.3),
    "hy720p":      dict(T=33, H=45, W=80, n_text=256, batch=1, heads=24, head_dim=128, block=128, topk=0.30, p=0.3),
    "hy720p_k10":  dict(T=33, H=45, W=80, n_text=256, batch=1, heads=24, head_dim=128, block=128, topk=0.10, p=0.3),
    "wan480p_p90": dict(T=21, H=30, W=52, n_text=512, batch=1, heads=40, head_dim=128, block=128, topk=0.30, p=0.9),
    "hy720p_k20":  dict(T=33, H=45, W=80, n_text=256, batch=1, heads=24, head_dim=128, block=128, topk=0.20, p=0.3),
    # Wan2.1-1.3B's own latent grid (appendix, detailed parameters) with the cumulative-probability cut the paper
    # uses for Wan; the head count (12 x 128) is an assumption, the paper does not state it
    "wan13b":      dict(T=20, H=30, W=52, n_text=512, batch=1, heads=12, head_dim=128, block=128, topk=0.30, p=0.9),
    # the low-resolution ProRes stage with the text-attention amplifier on (rho = 0.5, 0.75x stage: beta =
    # -0.5 log 0.5625); same tensors as hy_lowres
    "hy_lowres_amp": dict(T=33, H=24, W=42, n_text=256, batch=1, heads=24, head_dim=128, block=128, topk=0.30, p=0.3,
                          text_bias=0.2876820724517809),
    # the headline layer with the time-paced walk of the attention kernel (flag bit 3 of the library)
    "hy720p_paced": dict(T=33, H=45, W=80, n_text=256, batch=1, heads=24, head_dim=128, block=128, topk=0.30, p=0.3,
                         flags=15),
    # the p = 0.9 lists (long, of very uneven length) with the time-paced walk
    "wan13b_paced": dict(T=20, H=30, W=52, n_text=512, batch=1, heads=12, head_dim=128, block=128, topk=0.30, p=0.9,
                         flags=15),
    # the largest block count the library takes (M = 2048): 2032 vision blocks of 32 tokens + 16 text blocks
    "max_blocks": {"T": 8, "H": 64, "W": 127, "n_text": 512, "batch": 1, "heads": 2, "head_dim": 64, "block": 32,
                   "topk": 0.05, "p": 0.3},
}


def make_qkv(w, seed, device="cpu", n_terms=4, noise_std=0.5):
    """Return (q, k, v): bf16 tensors [batch, N_v+N_c, heads, head_dim] on `device`."""
    T, H, W = w["T"], w["H"], w["W"]
    B, G, D, Nc = w["batch"], w["heads"], w["head_dim"], w["n_text"]
    Nv = T * H * W
    rng = np.random.Generator(np.random.PCG64(seed))
    freq = rng.uniform(0.5, 3.0, size=(3, G, n_terms)).astype(np.float32)      # shared by Q and K
    freq_v = rng.uniform(0.5, 3.0, size=(3, G, n_terms)).astype(np.float32)
    amp = rng.standard_normal(size=(3, G, n_terms, D)).astype(np.float32)
    phase = rng.uniform(0.0, 2.0 * math.pi, size=(3, G, n_terms, D)).astype(np.float32)
    dev = torch.device(device)
    gen = torch.Generator(device=dev)
    tt = torch.arange(T, device=dev, dtype=torch.float32).view(T, 1, 1) / T
    hh = torch.arange(H, device=dev, dtype=torch.float32).view(1, H, 1) / H
    ww = torch.arange(W, device=dev, dtype=torch.float32).view(1, 1, W) / W
    out = []
    for x in range(3):
        gen.manual_seed(seed * 8 + x)
        f = freq_v if x == 2 else freq
        res = torch.empty((B, Nv + Nc, G, D), dtype=torch.bfloat16, device=dev)
        for b in range(B):
            for g in range(G):
                acc = noise_std * torch.randn((Nv, D), generator=gen, device=dev, dtype=torch.float32)
                for s in range(n_terms):
                    arg = 2.0 * math.pi * (float(f[0, g, s]) * tt + float(f[1, g, s]) * hh + float(f[2, g, s]) * ww)
                    arg = arg.reshape(Nv, 1)
                    a = torch.from_numpy(amp[x, g, s]).to(dev).view(1, D)
                    ph = torch.from_numpy(phase[x, g, s]).to(dev).view(1, D)
                    acc += a * torch.sin(arg + ph)
                res[b, :Nv, g, :] = acc.to(torch.bfloat16)
                if Nc:
                    res[b, Nv:, g, :] = torch.randn((Nc, D), generator=gen, device=dev,
                                                    dtype=torch.float32).to(torch.bfloat16)
        out.append(res)
    return tuple(out)


def bits(t):
    """bf16 tensor -> numpy uint16 array of its bit patterns (host copy)."""
    return t.detach().cpu().contiguous().view(torch.int16).numpy().view(np.uint16)


# Stage switches (Sec. 3.2, Eq. 4): latent shapes [channels, T, H, W] before patchification.  The last one
# is the 540p -> 720p switch of a HunyuanVideo-like latent (16 channels, 33 latent frames, 8x spatial VAE).
STAGE_SWITCHES = {
    "tiny": {"channels": 3, "in": (3, 5, 7), "out": (4, 8, 10), "sigma": 0.6},
    "ragged": {"channels": 2, "in": (5, 13, 11), "out": (5, 17, 16), "sigma": 0.35},
    "down": {"channels": 2, "in": (4, 9, 10), "out": (2, 4, 7), "sigma": 0.9},
    "down_w16": {"channels": 3, "in": (4, 12, 16), "out": (2, 5, 8), "sigma": 0.45},      # rows of 16: staged in LDS
    "up_w12": {"channels": 2, "in": (3, 8, 12), "out": (4, 11, 18), "sigma": 0.55},         # W_out not a multiple of 4
    "up_wide": {"channels": 1, "in": (2, 5, 1024), "out": (2, 7, 1366), "sigma": 0.2},      # more than 256 quads per row
    "hy540to720": {"channels": 16, "in": (33, 68, 120), "out": (33, 90, 160), "sigma": 0.7},
}


def make_latents(w, seed, device="cpu"):
    """x_t, eps_t [channels, T, H, W] and eps_tilde [channels, T', H', W']: seeded N(0, 1) float32."""
    g = torch.Generator().manual_seed(seed)
    shp_in, shp_out = (w["channels"],) + tuple(w["in"]), (w["channels"],) + tuple(w["out"])
    x_t = torch.randn(shp_in, generator=g, dtype=torch.float32)
    eps_t = torch.randn(shp_in, generator=g, dtype=torch.float32)
    eps_tilde = torch.randn(shp_out, generator=g, dtype=torch.float32)
    return x_t.to(device), eps_t.to(device), eps_tilde.to(device)
