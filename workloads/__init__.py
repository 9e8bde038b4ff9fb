"""Seeded synthetic inputs shaped like the paper's workloads.

Serves both the CPU oracle's tests and the HIP path's tests/benchmark.  Holds
none of the method's arithmetic: it only draws random tensors, plants outlier
channels, rounds to the bf16 storage type and builds MoE routing lists.

Structure follows the paper's findings: token-persistent outlier channels at
the attention / W_o / W_1,W_3 inputs (Section 2.1, Fig. 2: vertical stripes),
diffuse outliers at W_2 inputs (Section 2.3, low-clustering regions); shapes
follow Qwen3-8B and Qwen3-30B-A3B (Section 4.1).  All bf16 tensors are numpy
uint16 arrays of bit patterns.
"""
import numpy as np

G = 32


def to_bf16_bits(a):
    """float32 array -> bf16 bit patterns (round to nearest even); finite inputs only."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    r = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
    return r.astype(np.uint16)


def from_bf16_bits(b):
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(
        np.float32)


def rng(seed):
    return np.random.Generator(np.random.PCG64(seed))


def planted_table(gen, K, r, group=G):
    """[K/group, max(r,1)] int16 table: r distinct local indices per group (ascending), else -1."""
    Kg = K // group
    table = np.full((Kg, max(r, 1)), -1, np.int16)
    for g in range(Kg):
        if r:
            table[g, :r] = np.sort(gen.choice(group, size=r, replace=False))
    return table


def table_channels(table, group=G):
    """Global channel ids named by a table, ascending (pure index bookkeeping)."""
    out = []
    for g in range(table.shape[0]):
        for j in sorted(int(v) for v in table[g] if v >= 0):
            out.append(g * group + j)
    return np.asarray(out, np.int32)


def gaussian_rows(gen, M, K, chunk=1024):
    x = np.empty((M, K), np.float32)
    for m0 in range(0, M, chunk):
        m1 = min(M, m0 + chunk)
        x[m0:m1] = gen.standard_normal((m1 - m0, K), dtype=np.float32)
    return x


def activations_persistent(seed, M, K, r, factor="loguniform", lo=20.0, hi=100.0, jitter=0.0, group=G):
    """N(0,1) activations with r token-persistent outlier channels per group of `group` channels.

    factor: "loguniform" -> one factor per channel, exp(U(ln lo, ln hi));
            a float      -> that constant.
    jitter: per-(token, channel) relative jitter u*jitter, u ~ U(-1, 1).
    Returns (X bits [M,K], table int16 [K/group, max(r,1)]).
    """
    gen = rng(seed)
    table = planted_table(gen, K, r, group)
    ch = table_channels(table, group)
    x = gaussian_rows(gen, M, K)
    if len(ch):
        if factor == "loguniform":
            f = np.exp(gen.uniform(np.log(lo), np.log(hi), size=len(ch))).astype(np.float32)
        else:
            f = np.full(len(ch), float(factor), np.float32)
        scale = np.broadcast_to(f, (M, len(ch))).copy()
        if jitter:
            scale *= (1.0 + jitter * gen.uniform(-1.0, 1.0, size=(M, len(ch)))).astype(np.float32)
        x[:, ch] *= scale
    return to_bf16_bits(x), table


def activations_diffuse(seed, M, K, p=0.005, factor=50.0):
    """N(0,1) activations; each entry independently x`factor` with probability p."""
    gen = rng(seed)
    x = gaussian_rows(gen, M, K)
    for m0 in range(0, M, 1024):
        m1 = min(M, m0 + 1024)
        mask = gen.random((m1 - m0, K), dtype=np.float32) < p
        x[m0:m1][mask] *= factor
    return to_bf16_bits(x)


def weights(seed, N, K, sigma=0.02):
    gen = rng(seed)
    w = gaussian_rows(gen, N, K)
    w *= np.float32(sigma)
    return to_bf16_bits(w)


def moe_routing(seed, tokens, E, top_k):
    """Top-k routing from seeded N(0,1) logits (softmax is monotone, so top-k by logit).

    Returns (expert_offsets int32[E+1], row_map int32[tokens*top_k]): sorted
    position t reads token row_map[t]; rows of expert e are
    [offsets[e], offsets[e+1]); order inside an expert is by token id.
    """
    gen = rng(seed)
    logits = gen.standard_normal((tokens, E), dtype=np.float32)
    # stable sort on (-logit) keeps the lower expert id first among equal logits
    top = np.argsort(-logits, axis=1, kind="stable")[:, :top_k]
    tok = np.repeat(np.arange(tokens, dtype=np.int32), top_k)
    exp = top.reshape(-1).astype(np.int32)
    order = np.lexsort((tok, exp))
    row_map = tok[order].astype(np.int32)
    counts = np.bincount(exp, minlength=E)
    offsets = np.zeros(E + 1, np.int32)
    offsets[1:] = np.cumsum(counts)
    return offsets, row_map


# ---- the five benchmark configurations ----------------------------------------


def config1_tiny():
    """X[16,256], one outlier channel per group x64 with +-10% per-token jitter; W[256,256]."""
    X, table = activations_persistent(1001, 16, 256, 1, factor=64.0, jitter=0.1)
    W = weights(1002, 256, 256)
    return dict(X=X, table=table, W=W, M=16, K=256, N=256, r=1)


def config2_attn(M, N, seed=2001):
    """Qwen3-8B attention projection input: hidden 4096, 2 persistent outliers per group."""
    X, table = activations_persistent(seed, M, 4096, 2)
    W = weights(seed + 1 + N, N, 4096)
    return dict(X=X, table=table, W=W, M=M, K=4096, N=N, r=2)


def config5_sweep(M, r, N=12288, seed=5001):
    X, table = activations_persistent(seed + r, M, 4096, r, factor=64.0)
    W = weights(seed + 100, N, 4096)
    return dict(X=X, table=table, W=W, M=M, K=4096, N=N, r=r)
