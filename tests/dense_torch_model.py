"""Independent full-sequence transformer used only to pin the oracle.

It recomputes the whole sequence in one pass with PyTorch CPU library routines (linear, rms_norm,
scaled_dot_product_attention with an explicit dense boolean mask, silu) in float64 and has no KV
cache, no block logic and no code in common with the oracle.  The rotary embedding is written in
its complex-multiplication form, (x_i + i*x_{i+d/2}) * exp(i*p*theta^(-2i/d)).
"""
import torch
import torch.nn.functional as F


def dense_mask(n_prefix, block, bidir):
    """Literal visibility matrix for [prefix | block]: prefix rows are token-causal; block rows see
    the whole prefix and, inside the block, everything (bidir) or keys j <= i (causal)."""
    T = n_prefix + block
    A = torch.zeros(T, T, dtype=torch.bool)
    for i in range(T):
        for j in range(T):
            if i < n_prefix:
                A[i, j] = j <= i
            elif j < n_prefix:
                A[i, j] = True
            else:
                A[i, j] = True if bidir else (j <= i)
    return A


def rope_complex(x, pos, theta):
    # x [T, heads, d]
    d = x.shape[-1]
    half = d // 2
    freqs = theta ** (-(torch.arange(half, dtype=torch.float64) * 2.0 / d))
    ang = pos.to(torch.float64)[:, None] * freqs[None, :]
    rot = torch.polar(torch.ones_like(ang), ang)[:, None, :]          # e^{i ang}
    z = torch.complex(x[..., :half], x[..., half:]) * rot
    return torch.cat([z.real, z.imag], dim=-1)


def full_forward(shape, weights, x, mask, return_kv=False):
    """x [T, hidden] float64 input embeddings at positions 0..T-1; mask [T,T] bool (True = visible)."""
    W = {k: torch.from_numpy(v).to(torch.float64) for k, v in weights.items() if v.dtype.kind == "f"}
    x = torch.as_tensor(x, dtype=torch.float64)
    T = x.shape[0]
    pos = torch.arange(T)
    G = shape.n_q_heads // shape.n_kv_heads
    kvs = []
    for l in range(shape.n_layers):
        p = f"l{l}."
        h = F.rms_norm(x, (shape.hidden,), W[p + "attn_norm"], shape.rms_eps)
        q = F.linear(h, W[p + "wq"]).view(T, shape.n_q_heads, shape.head_dim)
        k = F.linear(h, W[p + "wk"]).view(T, shape.n_kv_heads, shape.head_dim)
        v = F.linear(h, W[p + "wv"]).view(T, shape.n_kv_heads, shape.head_dim)
        q = rope_complex(q, pos, shape.rope_theta)
        k = rope_complex(k, pos, shape.rope_theta)
        kvs.append((k.clone(), v.clone()))
        kk = k.repeat_interleave(G, dim=1)
        vv = v.repeat_interleave(G, dim=1)
        o = F.scaled_dot_product_attention(q.transpose(0, 1), kk.transpose(0, 1), vv.transpose(0, 1),
                                           attn_mask=mask)
        o = o.transpose(0, 1).reshape(T, -1)
        x = x + F.linear(o, W[p + "wo"])
        h = F.rms_norm(x, (shape.hidden,), W[p + "ffn_norm"], shape.rms_eps)
        x = x + F.linear(F.silu(F.linear(h, W[p + "w_gate"])) * F.linear(h, W[p + "w_up"]), W[p + "w_down"])
    logits = F.linear(F.rms_norm(x, (shape.hidden,), W["final_norm"], shape.rms_eps), W["lm_head"])
    if return_kv:
        return logits, kvs
    return logits


def embed_rows(weights, ids):
    return torch.from_numpy(weights["embed"][ids]).to(torch.float64)
