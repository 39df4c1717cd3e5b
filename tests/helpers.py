"""Shared test helpers: independent restatements of the operator used to pin the
oracle (they deliberately do not call it), and small conversion utilities."""
import math

import numpy as np

from paper_2603_06738_amd import workloads as wk


def geometry(oracle, wl: wk.Workload):
    return oracle.Geometry(wl.B, wl.H, wl.W, wl.heads, wl.d, wl.r, wl.M, wl.s,
                           wl.scale_c, wl.scale_p)


def brute_force_fwd(wl, x):
    """Sec. 2.2 / Eq. 6 written over GLOBAL pixel coordinates: two pixels attend
    to each other iff, after undoing the cyclic shift, they fall in the same
    MxM block; the RIB row of a pixel is its row-major position in that block.
    Pure Python loops in float64 -- only for tiny grids."""
    q, k, v, fq, fk = (x[n].astype(np.float64) for n in ("q", "k", "v", "f_q", "f_k"))
    B, H, W, M, s, d = wl.B, wl.H, wl.W, wl.M, wl.s, wl.d
    O = np.zeros((B, H, W, wl.C))

    def block_and_pos(y, xx):
        yy, xs = (y - s) % H, (xx - s) % W
        return (yy // M, xs // M), (yy % M) * M + (xs % M)

    for b in range(B):
        for hd in range(wl.heads):
            ch = slice(hd * d, (hd + 1) * d)
            for y in range(H):
                for xx in range(W):
                    blk, pi = block_and_pos(y, xx)
                    logits, vals = [], []
                    for y2 in range(H):
                        for x2 in range(W):
                            blk2, pj = block_and_pos(y2, x2)
                            if blk2 != blk:
                                continue
                            content = float(np.dot(q[b, y, xx, ch], k[b, y2, x2, ch]))
                            bias = float(np.dot(fq[hd, pi], fk[hd, pj]))
                            logits.append(wl.scale_c * content + wl.scale_p * bias)
                            vals.append(v[b, y2, x2, ch])
                    mx = max(logits)
                    e = [math.exp(t - mx) for t in logits]
                    z = sum(e)
                    acc = np.zeros(d)
                    for w_, vv in zip(e, vals):
                        acc += (w_ / z) * vv
                    O[b, y, xx, ch] = acc
    return O


def partition(a, M, s):
    """[B,H,W,C] numpy grid -> [B*nW, N, C] after rolling by (-s,-s)."""
    B, H, W, C = a.shape
    a = np.roll(a, (-s, -s), axis=(1, 2))
    a = a.reshape(B, H // M, M, W // M, M, C).transpose(0, 1, 3, 2, 4, 5)
    return a.reshape(B * (H // M) * (W // M), M * M, C)


def unpartition(a, B, H, W, M, s):
    C = a.shape[-1]
    a = a.reshape(B, H // M, W // M, M, M, C).transpose(0, 1, 3, 2, 4, 5).reshape(B, H, W, C)
    return np.roll(a, (s, s), axis=(1, 2))


def concat_form_fwd(wl, x, dtype=np.float64):
    """Eq. 5: Q = [scale_c*q || scale_p*f_q], K = [k || f_k], one dot product,
    softmax, PV -- in numpy over explicitly partitioned windows, every operation in
    `dtype` (float64 unless a test asks for single precision)."""
    qs, ks, vs = (partition(x[n].astype(dtype), wl.M, wl.s) for n in ("q", "k", "v"))
    nW, N, d = qs.shape[0], wl.N, wl.d
    O = np.zeros_like(qs)
    lse = np.zeros((nW, wl.heads, N), dtype)
    for hd in range(wl.heads):
        ch = slice(hd * d, (hd + 1) * d)
        fq = np.broadcast_to(x["f_q"][hd].astype(dtype), (nW, N, wl.r))
        fk = np.broadcast_to(x["f_k"][hd].astype(dtype), (nW, N, wl.r))
        Q = np.concatenate([dtype(wl.scale_c) * qs[..., ch], dtype(wl.scale_p) * fq], axis=-1)
        K = np.concatenate([ks[..., ch], fk], axis=-1)
        S = Q @ K.transpose(0, 2, 1)
        mx = S.max(-1, keepdims=True)
        E = np.exp(S - mx)
        Z = E.sum(-1, keepdims=True)
        O[..., ch] = (E / Z) @ vs[..., ch]
        lse[:, hd, :] = (mx + np.log(Z))[..., 0]
    return unpartition(O, wl.B, wl.H, wl.W, wl.M, wl.s), lse


def torch_sdpa_fwd_bwd(wl, x, d_out=None):
    """Library route: torch.roll + view/permute partition, then
    scaled_dot_product_attention with a float additive mask (the RIB bias), in
    float64 on the CPU; gradients by autograd."""
    import torch
    import torch.nn.functional as F
    B, H, W, M, s, h, d = wl.B, wl.H, wl.W, wl.M, wl.s, wl.heads, wl.d
    t = {n: torch.tensor(np.asarray(a), dtype=torch.float64, requires_grad=True)
         for n, a in x.items() if n != "d_out"}

    def part(a):
        a = torch.roll(a, (-s, -s), (1, 2))
        a = a.view(B, H // M, M, W // M, M, h, d).permute(0, 1, 3, 5, 2, 4, 6)
        return a.reshape(-1, h, M * M, d)

    bias = wl.scale_p * t["f_q"] @ t["f_k"].transpose(1, 2)          # [h,N,N]
    o = F.scaled_dot_product_attention(part(t["q"]), part(t["k"]), part(t["v"]),
                                       attn_mask=bias.unsqueeze(0), scale=wl.scale_c)
    o = o.view(B, H // M, W // M, h, M, M, d).permute(0, 1, 4, 2, 5, 3, 6).reshape(B, H, W, h * d)
    o = torch.roll(o, (s, s), (1, 2))
    res = {"O": o.detach().numpy()}
    if d_out is not None:
        o.backward(torch.tensor(np.asarray(d_out), dtype=torch.float64))
        res.update(dQ=t["q"].grad.numpy(), dK=t["k"].grad.numpy(), dV=t["v"].grad.numpy(),
                   dF_q=t["f_q"].grad.numpy(), dF_k=t["f_k"].grad.numpy())
    return res
