"""Third opinion used to pin the oracle: the same layer written with PyTorch CPU
library routines in fp64 on CONTIGUOUS sequences (no pages, no cache, no batch
descriptor).  Each request's whole sequence is recomputed from scratch, causal
attention comes from torch's scaled_dot_product_attention.  Test helper only.
"""
import numpy as np
import torch
import torch.nn.functional as F

from paper_2601_11546_amd.workloads import bf16_bits_to_f32


def _t(bits):
    return torch.from_numpy(bf16_bits_to_f32(bits).astype(np.float64))


def rope_complex(v: torch.Tensor, pos: torch.Tensor, base: float) -> torch.Tensor:
    """v: [L, heads, d]; pairs (i, i+d/2) seen as complex numbers times e^{i pos theta_i}."""
    d = v.shape[-1]
    half = d // 2
    theta = torch.tensor(base, dtype=torch.float64) ** (-torch.arange(half, dtype=torch.float64) * 2.0 / d)
    z = torch.complex(v[..., :half], v[..., half:])
    rot = torch.polar(torch.ones_like(theta)[None, :].expand(len(pos), half).contiguous(),
                      pos.to(torch.float64)[:, None] * theta[None, :])
    z = z * rot[:, None, :]
    return torch.cat([z.real, z.imag], dim=-1)


def dense_model_logits(shape, model, token_ids):
    """Whole stack on one request's full token sequence: logits of its last token (fp64)."""
    x_bits = model["embedding"][np.asarray(token_ids)]
    for wts in model["layers"]:
        y = dense_layer(shape, wts, x_bits)["y"]
        x_bits = y.to(torch.float32).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    last = _t(x_bits[-1:])
    h = F.rms_norm(last, (shape.hidden,), _t(model["w_final_norm"]), eps=shape.rms_eps)
    return F.linear(h, _t(model["w_lm_head"]))[0]


def dense_layer(shape, weights, x_bits, round_kv_bf16=True, kv_override=None, quantise=None, code_values=None):
    """x_bits: [L, H] one request's whole sequence.  Returns dict of fp64 tensors.

    kv_override: optional (k, v) fp64 tensors [L, n_kv, d] used instead of the
    recomputed keys/values (lets a test feed the oracle's cached bits back in).
    quantise / code_values: the caller's fp32 -> 8-bit codes and codes -> fp64 conversions (through the library's
    own 8-bit type); then `weights` holds codes w_*, row scales s_* and input scales a_* and every projection is
    (codes of the input) x (codes of the weights) x (input scale x row scale).
    """
    H, d, nh, nkv = shape.hidden, shape.head_dim, shape.n_q_heads, shape.n_kv_heads
    x = _t(x_bits)
    L = x.shape[0]
    if quantise is None:
        w = {k: _t(v) for k, v in weights.items()}

        def proj(a, name, round_bf16=False):
            return F.linear(a, w["w_" + name])
    else:
        w = {k: _t(weights[k]) for k in ("w_in_norm", "w_post_norm")}

        def proj(a, name, round_bf16=False):
            if round_bf16:
                a = a.to(torch.float32).to(torch.bfloat16)
            s_a = float(weights["a_" + name])
            codes = quantise(a.to(torch.float32), s_a)
            out = F.linear(code_values(codes), code_values(weights["w_" + name]))
            return out * torch.from_numpy(weights["s_" + name].astype(np.float64))[None, :] * float(np.float32(s_a))
    h = F.rms_norm(x, (H,), w["w_in_norm"], eps=shape.rms_eps)
    qkv = proj(h, "qkv")
    q = qkv[:, :nh * d].reshape(L, nh, d)
    k = qkv[:, nh * d:(nh + nkv) * d].reshape(L, nkv, d)
    v = qkv[:, (nh + nkv) * d:].reshape(L, nkv, d)
    pos = torch.arange(L)
    q = rope_complex(q, pos, shape.rope_base)
    k = rope_complex(k, pos, shape.rope_base)
    if round_kv_bf16:
        k = k.to(torch.float32).to(torch.bfloat16).to(torch.float64)
        v = v.to(torch.float32).to(torch.bfloat16).to(torch.float64)
    k_own, v_own = k, v
    if kv_override is not None:
        k, v = kv_override
    rep = nh // nkv
    kk = k.repeat_interleave(rep, dim=1)
    vv = v.repeat_interleave(rep, dim=1)
    o = F.scaled_dot_product_attention(q.transpose(0, 1)[None], kk.transpose(0, 1)[None],
                                       vv.transpose(0, 1)[None], is_causal=True)[0]
    o = o.transpose(0, 1).reshape(L, nh * d)
    x1 = x + proj(o, "o", round_bf16=True)
    h2 = F.rms_norm(x1, (H,), w["w_post_norm"], eps=shape.rms_eps)
    gu = proj(h2, "gate_up")
    I = shape.mlp_dim
    act = F.silu(gu[:, :I]) * gu[:, I:]
    y = x1 + proj(act, "down")
    return {"y": y, "x1": x1, "attn_out": o, "k": k_own, "v": v_own, "q": q}
