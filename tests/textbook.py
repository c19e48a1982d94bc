"""Independent pin for the oracle: ordinary causal decoding, one token at a time.

Written with PyTorch library routines in float64 (F.rms_norm, F.linear,
F.scaled_dot_product_attention, F.silu, complex multiplication for the rotary
embedding).  Sequential decoding needs no attention mask at all: each new token
simply attends to everything cached so far.  The paper's correctness claim for
tree verification (Sec. III-B: score order is a topological order, so causal
relations are preserved) is that a node's output equals what this decoder gives
for the node's root-to-node path.
"""
import torch
import torch.nn.functional as F


def _t(a):
    return torch.as_tensor(a, dtype=torch.float64)


def rope_complex(x, pos, theta):
    """x: [..., hd]; pairs (t, t + hd/2) form the complex number x_t + i x_{t+hd/2}."""
    hd = x.shape[-1]
    h = hd // 2
    z = torch.complex(x[..., :h], x[..., h:])
    k = torch.arange(h, dtype=torch.float64)
    ang = float(pos) * torch.pow(torch.tensor(float(theta), dtype=torch.float64), -2.0 * k / hd)
    z = z * torch.polar(torch.ones_like(ang), ang)
    return torch.cat([z.real, z.imag], dim=-1)


class SequentialDecoder:
    """Plain KV-cache decoder over the stage's layers; cache starts as the given prefix."""

    def __init__(self, cfg, layers, prefix):
        self.cfg = cfg
        self.layers = [{k: (None if v is None else _t(v)) for k, v in lw.items()} for lw in layers]
        # prefix[layer]: [2, H_kv, l_glo, hd]
        self.k = [_t(p[0]).clone() for p in prefix]
        self.v = [_t(p[1]).clone() for p in prefix]

    def step(self, x, pos):
        """x: [d] hidden state of the next token, at absolute position pos.  Returns the stage output [d]."""
        c = self.cfg
        x = _t(x)
        G = c.n_q_heads // c.n_kv_heads
        for li, w in enumerate(self.layers):
            n = F.rms_norm(x, (c.d_model,), w["rms_attn"], c.rms_eps)
            q = F.linear(n, w["wq"], w["bq"]).view(c.n_q_heads, c.head_dim)
            k = F.linear(n, w["wk"], w["bk"]).view(c.n_kv_heads, c.head_dim)
            v = F.linear(n, w["wv"], w["bv"]).view(c.n_kv_heads, c.head_dim)
            q = rope_complex(q, pos, c.rope_theta)
            k = rope_complex(k, pos, c.rope_theta)
            self.k[li] = torch.cat([self.k[li], k[:, None, :]], dim=1)
            self.v[li] = torch.cat([self.v[li], v[:, None, :]], dim=1)
            kk = self.k[li].repeat_interleave(G, dim=0)
            vv = self.v[li].repeat_interleave(G, dim=0)
            o = F.scaled_dot_product_attention(q[:, None, :], kk, vv)  # [Hq, 1, hd], default scale 1/sqrt(hd)
            x = x + F.linear(o.reshape(-1), w["wo"])
            n = F.rms_norm(x, (c.d_model,), w["rms_ffn"], c.rms_eps)
            x = x + F.linear(F.silu(F.linear(n, w["w_gate"])) * F.linear(n, w["w_up"]), w["w_down"])
        return x


def decode_path(cfg, layers, prefix, rows, l_glo):
    """Decode the given hidden rows one after another at positions l_glo, l_glo+1, ...; return all outputs."""
    dec = SequentialDecoder(cfg, layers, prefix)
    outs = [dec.step(r, l_glo + t) for t, r in enumerate(rows)]
    return torch.stack(outs).numpy(), dec


def lm_head(cfg, final_norm, lm, hidden):
    n = F.rms_norm(_t(hidden), (cfg.d_model,), _t(final_norm), cfg.rms_eps)
    return F.linear(n, _t(lm)).numpy()


def path_to(parent, i):
    p = []
    while i >= 0:
        p.append(int(i))
        i = int(parent[i])
    return p[::-1]
