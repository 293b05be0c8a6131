"""Independent dense references used to pin the oracle (CPU only, tiny inputs).

Nothing here is shared with the oracle or with the HIP path: K/V are gathered into dense
[L, D] float64 matrices with numpy indexing and the softmax comes from scipy / torch.
"""
import numpy as np
from scipy.special import logsumexp, softmax


def widen_bf16(bits):
    return (np.asarray(bits, dtype=np.uint16).astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def e4m3_to_f64(byts):
    """Decode OCP e4m3 bytes with the library cast of torch.float8_e4m3fn."""
    import torch

    t = torch.from_numpy(np.ascontiguousarray(byts, dtype=np.uint8)).view(torch.float8_e4m3fn)
    return t.to(torch.float64).numpy()


def gather_dense(batch, b, g):
    """Dense float64 K, V of shape [L_b, D] for sequence b and KV head g."""
    L = int(batch.context_lens[b])
    BS = batch.block_size
    t = np.arange(L)
    phys = np.maximum(batch.block_tables[b, t // BS], 0)  # evicted entries (-1): any block, the caller masks them
    slot = t % BS
    kraw = batch.k_cache[phys, g, slot, :]
    vraw = batch.v_cache[phys, g, slot, :]
    if batch.kv_dtype == 0:
        return widen_bf16(kraw), widen_bf16(vraw)
    return (e4m3_to_f64(kraw) * np.float64(batch.k_scale[g]), e4m3_to_f64(vraw) * np.float64(batch.v_scale[g]))


def dense_attention(batch):
    """out [B,Hq,D] float64, lse [B,Hq] via scipy softmax on gathered dense matrices."""
    B, Hq, D = batch.q.shape
    G = Hq // batch.num_kv_heads
    out = np.zeros((B, Hq, D))
    lse = np.full((B, Hq), -np.inf)
    q = widen_bf16(batch.q)
    for b in range(B):
        if batch.context_lens[b] <= 0:
            continue
        for h in range(Hq):
            K, V = gather_dense(batch, b, h // G)
            s = (K @ q[b, h]) * np.float64(batch.scale)
            out[b, h] = softmax(s) @ V
            lse[b, h] = logsumexp(s)
    return out, lse


def torch_sdpa(batch):
    """Same, through torch.nn.functional.scaled_dot_product_attention in float64 on the CPU."""
    import torch
    import torch.nn.functional as F

    B, Hq, D = batch.q.shape
    G = Hq // batch.num_kv_heads
    out = np.zeros((B, Hq, D))
    q = widen_bf16(batch.q)
    for b in range(B):
        if batch.context_lens[b] <= 0:
            continue
        Ks, Vs = zip(*(gather_dense(batch, b, g) for g in range(batch.num_kv_heads)))
        K = torch.from_numpy(np.stack(Ks)).repeat_interleave(G, dim=0)  # [Hq, L, D]
        V = torch.from_numpy(np.stack(Vs)).repeat_interleave(G, dim=0)
        Q = torch.from_numpy(q[b]).unsqueeze(1)  # [Hq, 1, D]
        o = F.scaled_dot_product_attention(Q, K, V, scale=float(batch.scale))
        out[b] = o.squeeze(1).numpy()
    return out


def dense_window_attention(batch, sliding=0):
    """Multi-token window, out [B,Q,Hq,D] float64: torch's scaled_dot_product_attention in float64 with
    an explicit boolean mask.  Query token i of the window may look at logical token t iff
    t <= L - Q + i (the window is the last Q tokens of the context; each sees itself and the past)
    and, with ``sliding`` = W > 0, t > L - Q + i - W (the W most recent of those).  Rows with nothing
    visible are zero.  K/V rows outside every mask may hold anything (they are zeroed first)."""
    import torch
    import torch.nn.functional as F

    B, Q, Hq, D = batch.q.shape
    G = Hq // batch.num_kv_heads
    out = np.zeros((B, Q, Hq, D))
    q = widen_bf16(batch.q)
    for b in range(B):
        L = int(batch.context_lens[b])
        if L <= 0:
            continue
        Ks, Vs = zip(*(gather_dense(batch, b, g) for g in range(batch.num_kv_heads)))
        K = torch.from_numpy(np.stack(Ks)).repeat_interleave(G, dim=0)  # [Hq, L, D]
        V = torch.from_numpy(np.stack(Vs)).repeat_interleave(G, dim=0)
        Qm = torch.from_numpy(q[b]).permute(1, 0, 2)  # [Hq, Q, D]
        key_pos = torch.arange(L)[None, :]
        last_visible = (L - Q + torch.arange(Q))[:, None]
        mask = key_pos <= last_visible  # [Q, L]
        if sliding > 0:
            mask &= key_pos > last_visible - sliding
            unseen = ~mask.any(dim=0)  # evicted / poisoned rows: keep NaN patterns out of the library call
            K = K.clone()
            V = V.clone()
            K[:, unseen] = 0
            V[:, unseen] = 0
        seen = mask.any(dim=1)
        safe = mask.clone()
        safe[~seen, 0] = True  # keep the library away from all-masked rows; they are zeroed below
        o = F.scaled_dot_product_attention(Qm, K, V, attn_mask=safe[None], scale=float(batch.scale))
        o = o.permute(1, 0, 2).numpy().copy()
        o[~seen.numpy()] = 0.0
        out[b] = o
    return out
