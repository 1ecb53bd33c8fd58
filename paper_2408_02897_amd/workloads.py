"""Seeded synthetic inputs with BERT's matrix-multiply shapes.

This module holds no arithmetic of the method itself (no scaling, encoding,
products or metrics): it only draws tensors and names shapes, so both the HIP
path and the CPU oracle can be fed identical bits.  Distribution families
follow what the paper reports for BERT (weights close to normal, upstream
gradients close to log-normal; heavy-tailed Student-t inputs as in its
512 x 512 illustrative example).  Nothing here is taken from a dataset.

All tensors are generated on the host with torch.Generator().manual_seed(seed),
rounded to bfloat16 (RNE) and returned as CPU bfloat16 tensors.
"""
import math
from dataclasses import dataclass

import torch

# role numbers used in the seed schedule  seed = 10000*config + 100*layer + role
ROLE_X, ROLE_WQKV, ROLE_WO, ROLE_WFFN1, ROLE_WFFN2, ROLE_DY, ROLE_Q, ROLE_K, ROLE_V, ROLE_OUTLIER = range(10)


def seed_for(config, layer, role, op=0):
    return 10000 * config + 100 * layer + role + 1000 * op


def _gen(seed):
    g = torch.Generator()
    g.manual_seed(int(seed))
    return g


def normal(shape, std, seed):
    """N(0, std^2), bfloat16."""
    return (torch.randn(shape, generator=_gen(seed), dtype=torch.float32) * std).to(torch.bfloat16)


def student_t(shape, df, seed, scale=1.0):
    """Student-t with integer df as z / sqrt(chi2_df / df), bfloat16."""
    g = _gen(seed)
    z = torch.randn(shape, generator=g, dtype=torch.float32)
    chi2 = torch.zeros(shape, dtype=torch.float32)
    for _ in range(int(df)):
        chi2 += torch.randn(shape, generator=g, dtype=torch.float32) ** 2
    return (scale * z / torch.sqrt(chi2 / df)).to(torch.bfloat16)


def lognormal_signed(shape, mu, sigma, seed):
    """sign * exp(N(mu, sigma^2)) with a fair random sign, bfloat16."""
    g = _gen(seed)
    mag = torch.exp(torch.randn(shape, generator=g, dtype=torch.float32) * sigma + mu)
    sign = (torch.rand(shape, generator=g) < 0.5).to(torch.float32) * 2.0 - 1.0
    return (sign * mag).to(torch.bfloat16)


@dataclass(frozen=True)
class GemmOp:
    """One matrix multiply Y[M,N] = A[M,K] . B[N,K]^T of a BERT layer."""
    name: str
    M: int
    N: int
    K: int

    @property
    def flops(self):
        return 2 * self.M * self.N * self.K


def bert_forward_ops(tokens, hidden, ffn):
    return [GemmOp("qkv", tokens, 3 * hidden, hidden), GemmOp("attn_out", tokens, hidden, hidden),
            GemmOp("ffn1", tokens, ffn, hidden), GemmOp("ffn2", tokens, hidden, ffn)]


BERT_BASE = dict(tokens=4096, hidden=768, ffn=3072)       # batch 32 x seq 128
BERT_LARGE = dict(tokens=16384, hidden=1024, ffn=4096)    # batch 32 x seq 512, 24 layers
_W_ROLE = {"qkv": ROLE_WQKV, "attn_out": ROLE_WO, "ffn1": ROLE_WFFN1, "ffn2": ROLE_WFFN2}


def single_linear(seed=0):
    """X 256x768 ~ N(0,1), W 768x768 ~ N(0, 0.02^2), both from one generator seeded `seed`."""
    g = _gen(seed)
    x = torch.randn((256, 768), generator=g, dtype=torch.float32).to(torch.bfloat16)
    w = (torch.randn((768, 768), generator=g, dtype=torch.float32) * 0.02).to(torch.bfloat16)
    return x, w


def forward_operands(op, config, layer=0):
    """Activations X [M,K] ~ Student-t(4), weights W [N,K] ~ N(0, 0.02^2) for a forward op."""
    i = ["qkv", "attn_out", "ffn1", "ffn2"].index(op.name)
    x = student_t((op.M, op.K), 4, seed_for(config, layer, ROLE_X, i))
    w = normal((op.N, op.K), 0.02, seed_for(config, layer, _W_ROLE[op.name]))
    return x, w


def upstream_gradient(op, config, layer=0):
    """dY [M,N] for a forward op: |dY| ~ log-normal(mu=-8, sigma=2), random sign."""
    i = ["qkv", "attn_out", "ffn1", "ffn2"].index(op.name)
    return lognormal_signed((op.M, op.N), -8.0, 2.0, seed_for(config, layer, ROLE_DY, i))


def attention_operands(batch=32, heads=16, seq=512, dim=64, config=5):
    """Q, K, V [batch*heads, seq, dim] ~ N(0,1) with 1 % of the (head, dim) channels scaled x20
    (same channel set for Q, K and V).  Batch index = example*heads + head."""
    q = normal((batch, heads, seq, dim), 1.0, seed_for(config, 0, ROLE_Q)).float()
    k = normal((batch, heads, seq, dim), 1.0, seed_for(config, 0, ROLE_K)).float()
    v = normal((batch, heads, seq, dim), 1.0, seed_for(config, 0, ROLE_V)).float()
    n_ch = heads * dim
    n_out = max(1, round(0.01 * n_ch))
    perm = torch.randperm(n_ch, generator=_gen(seed_for(config, 0, ROLE_OUTLIER)))[:n_out]
    for ch in perm.tolist():
        h, d = divmod(ch, dim)
        q[:, h, :, d] *= 20.0
        k[:, h, :, d] *= 20.0
        v[:, h, :, d] *= 20.0
    f = lambda t: t.reshape(batch * heads, seq, dim).to(torch.bfloat16)
    return f(q), f(k), f(v)


def softmax_probabilities(scores_ref, dim):
    """P = softmax(S / sqrt(dim)) row-wise from reference scores (harness code, float32 -> bfloat16)."""
    return torch.softmax(scores_ref.float() / math.sqrt(dim), dim=-1).to(torch.bfloat16)


# Degrees of freedom swept in the backward-error example (Eq. 3): heavy tails (1 = Cauchy) to normal (None).
BACKWARD_ERROR_DOFS = (1, 2, 3, 4, 6, 10, 30, None)


def backward_error_operands(dof, n=512):
    """The two n x n operands of the backward-error example: Student-t with `dof` degrees of freedom (None:
    normal), both stored with the contracting axis contiguous (L [M, K], R [N, K]: the product is L R^T)."""
    tag = 0 if dof is None else int(dof)
    if dof is None:
        return normal((n, n), 1.0, 60100 + tag), normal((n, n), 1.0, 60200 + tag)
    return student_t((n, n), dof, 60100 + tag), student_t((n, n), dof, 60200 + tag)
