"""CPU oracle for the attention-carving hot path (test infrastructure only).

Plain NumPy, float64 throughout, no blocking or fusion beyond what the paper's
own steps state.  Only tests, the smoke check and the benchmark's cpu_baseline
leg may import this package; the product path never does, and this package
imports nothing from the product.

What each function follows (paper = "Training-Free Efficient Video Generation
via Dynamic Token Carving"):

  Layout / padding        Sec. 3.1 ("padded lengths divisible by m"); partition
                          table in the appendix (112 pad tokens at 720p, m=128)
  permute / unpermute     Eq. 2
  block_pool              Eq. 3, Alg. 3 step 1 (mean pooling per block)
  relevance               Eq. 3 with the 1/sqrt(d_k) of Alg. 3 step 2, softmax step 3
  importance_mask         Sec. 3.1 (top kM blocks, then extend until the
                          accumulated probability exceeds p), Alg. 3 steps 4-8,
                          Eq. 5 of the appendix (minimal set with sum > p)
  condition_mask          Sec. 3.1 item (2), Alg. 3 step 9
  adjacency_mask          Sec. 3.1 item (3); 26-neighbourhood (Sec. 4.1)
  build_mask              Alg. 3 (union), Alg. 2 (text query blocks see all)
  block_sparse_attention  Alg. 4 (visit only selected blocks, sequence-length
                          mask, text bias), Eq. 1 inside the visited set
  dense_attention         Eq. 1, no blocks at all (brute force)

Readings taken where the paper is silent are listed next to the code that
takes them.  Parity status: every function here is pinned by the CPU tests
except equality of the curve with the third-party ordering the paper cites,
which is unpinned (see curve.py).
"""
import math
import numpy as np

from .curve import curve_perm, curve_cells

FLAG_ADJACENCY = 1
FLAG_CONDITION = 2
FLAG_CURVE = 4


class Layout:
    """Derived sizes and index tables of one configuration.

    Sequence layout on the curve side (one reading of Sec. 3.1's "padded
    lengths"): [vision tokens in curve order | pad to M_v*m | text | pad to M_c*m].
    """

    def __init__(self, T, H, W, n_text, block, topk_ratio, flags=7):
        self.T, self.H, self.W = int(T), int(H), int(W)
        self.n_text = int(n_text)
        self.m = int(block)
        self.flags = int(flags)
        self.N_v = self.T * self.H * self.W
        self.M_v = -(-self.N_v // self.m)
        self.M_c = -(-self.n_text // self.m)
        self.M = self.M_v + self.M_c
        self.N_pad = self.M * self.m
        self.pad_v = self.M_v * self.m - self.N_v
        self.pad_c = self.M_c * self.m - self.n_text
        # Alg. 3 step 6 uses k*M_v as a slice bound; rounding is not specified.
        # Reading: floor, with a 1e-6 guard against 0.3*260 = 77.999..., at least 1.
        self.K_top = max(1, int(math.floor(float(topk_ratio) * self.M_v + 1e-6))) if self.M_v > 0 else 0
        self.perm, self.inv = curve_perm(self.T, self.H, self.W, bool(self.flags & FLAG_CURVE))
        # src_of_pos[i]: index into the thw-side sequence (vision then text) or -1 for a pad
        src = np.full(self.N_pad, -1, dtype=np.int64)
        src[: self.N_v] = self.perm
        t0 = self.M_v * self.m
        src[t0: t0 + self.n_text] = self.N_v + np.arange(self.n_text)
        self.src_of_pos = src
        self.valid = src >= 0

    def block_valid_counts(self):
        return self.valid.reshape(self.M, self.m).sum(axis=1)


def bf16_bits_to_f64(bits):
    """Widen bfloat16 bit patterns (uint16/int16 array) to float64, exactly."""
    u = np.asarray(bits).view(np.uint16).astype(np.uint32) << np.uint32(16)
    return u.view(np.float32).astype(np.float64)


def f64_to_bf16_bits(x):
    """Round float64 -> float32 -> bfloat16 (nearest even); used only to build test inputs."""
    f = np.asarray(x, dtype=np.float64).astype(np.float32)
    u = f.view(np.uint32)
    rounded = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
    return rounded.astype(np.uint16)


# --------------------------------------------------------------------------- Eq. 2

def permute(x_thw, lay):
    """x_thw [B, N_v+N_c, heads, d] (thw order, text behind) -> [B, heads, N_pad, d] in curve order.

    Pad rows are zero.
    """
    B, N, Hh, D = x_thw.shape
    assert N == lay.N_v + lay.n_text
    out = np.zeros((B, Hh, lay.N_pad, D), dtype=x_thw.dtype)
    pos = np.nonzero(lay.valid)[0]
    out[:, :, pos, :] = np.transpose(x_thw[:, lay.src_of_pos[pos], :, :], (0, 2, 1, 3))
    return out


def unpermute(y_curve, lay):
    """Inverse of permute on the valid rows: [B, heads, N_pad, d] -> [B, N_v+N_c, heads, d]."""
    B, Hh, Np, D = y_curve.shape
    assert Np == lay.N_pad
    out = np.zeros((B, lay.N_v + lay.n_text, Hh, D), dtype=y_curve.dtype)
    pos = np.nonzero(lay.valid)[0]
    out[:, lay.src_of_pos[pos], :, :] = np.transpose(y_curve[:, :, pos, :], (0, 2, 1, 3))
    return out


# --------------------------------------------------------------------------- Eq. 3 / Alg. 3

def block_pool(x_curve, lay, n_blocks):
    """Mean over the valid tokens of each of the first n_blocks blocks.

    The paper says mean pooling and is silent on partial blocks; reading: divide
    by the number of valid tokens, not by m.
    x_curve [B, heads, N_pad, d] float64 -> [B, heads, n_blocks, d].
    """
    B, Hh, Np, D = x_curve.shape
    m = lay.m
    out = np.zeros((B, Hh, n_blocks, D), dtype=np.float64)
    for j in range(n_blocks):
        rows = np.nonzero(lay.valid[j * m:(j + 1) * m])[0] + j * m
        out[:, :, j, :] = x_curve[:, :, rows, :].sum(axis=2) / float(len(rows))
    return out


def relevance(q_hat, k_hat):
    """R = softmax_j(Q^ K^T / sqrt(d_k)) over all M key blocks (text blocks included)."""
    d = q_hat.shape[-1]
    S = np.einsum("bhid,bhjd->bhij", q_hat, k_hat) / math.sqrt(d)
    S = S - S.max(axis=-1, keepdims=True)
    E = np.exp(S)
    return E / E.sum(axis=-1, keepdims=True)


def importance_row(r, K_top, p):
    """One row of B_top: returns (selected boolean row, N_k).

    Order columns by (R descending, index ascending); C_n = sum of the first n.
    N_k = min(M, max(#{n : C_n <= p} + 1, K_top)); keep the first N_k.
    """
    M = r.shape[0]
    order = np.lexsort((np.arange(M), -r))
    C = np.cumsum(r[order])
    n_star = int((C <= p).sum()) + 1
    N_k = min(M, max(n_star, K_top))
    row = np.zeros(M, dtype=bool)
    row[order[:N_k]] = True
    return row, N_k


def importance_mask(R, K_top, p):
    B, Hh, Mv, M = R.shape
    out = np.zeros((B, Hh, Mv, M), dtype=bool)
    for b in range(B):
        for h in range(Hh):
            for i in range(Mv):
                out[b, h, i], _ = importance_row(R[b, h, i], K_top, p)
    return out


def condition_mask(lay):
    """B_cond over [M_v, M]: every text key column on (text query rows are handled in build_mask)."""
    out = np.zeros((lay.M_v, lay.M), dtype=bool)
    out[:, lay.M_v:] = True
    return out


def adjacency_mask(lay):
    """adja(i, j) for vision blocks: some valid token of i and some valid token of j are
    within Chebyshev distance 1 on the (t, h, w) grid (26-neighbourhood plus the token
    itself, so the diagonal is on); no wrap-around.  [M_v, M_v] bool.
    """
    T, H, W, m = lay.T, lay.H, lay.W, lay.m
    blk = (lay.inv // m).reshape(T, H, W)
    out = np.zeros((lay.M_v, lay.M_v), dtype=bool)
    for dt in (-1, 0, 1):
        for dh in (-1, 0, 1):
            for dw in (-1, 0, 1):
                a = blk[max(0, -dt): T - max(0, dt), max(0, -dh): H - max(0, dh), max(0, -dw): W - max(0, dw)]
                b = blk[max(0, dt): T - max(0, -dt), max(0, dh): H - max(0, -dh), max(0, dw): W - max(0, -dw)]
                out[a.ravel(), b.ravel()] = True
    return out


def build_mask(q_curve, k_curve, lay, p, return_R=False):
    """Full block mask B [B, heads, M, M] (Alg. 3, with Alg. 2's rule that text query
    blocks see every block).  q_curve/k_curve float64 [B, heads, N_pad, d]."""
    B, Hh = q_curve.shape[:2]
    mask = np.zeros((B, Hh, lay.M, lay.M), dtype=bool)
    R = None
    if lay.M_v > 0:
        q_hat = block_pool(q_curve, lay, lay.M_v)
        k_hat = block_pool(k_curve, lay, lay.M)
        R = relevance(q_hat, k_hat)
        top = importance_mask(R, lay.K_top, p)
        fixed = np.zeros((lay.M_v, lay.M), dtype=bool)
        if lay.flags & FLAG_CONDITION:
            fixed |= condition_mask(lay)
        if lay.flags & FLAG_ADJACENCY:
            fixed[:, : lay.M_v] |= adjacency_mask(lay)
        mask[:, :, : lay.M_v, :] = top | fixed[None, None]
    mask[:, :, lay.M_v:, :] = True
    if return_R:
        return mask, R
    return mask


def selection_margins(R, K_top, p):
    """Audit of how far each row's decisions are from flipping.

    Returns (min relative gap between the N_k-th and (N_k+1)-th sorted value,
             min |C_n - p| over all n).
    """
    B, Hh, Mv, M = R.shape
    min_gap, min_c = np.inf, np.inf
    for b in range(B):
        for h in range(Hh):
            for i in range(Mv):
                r = R[b, h, i]
                order = np.lexsort((np.arange(M), -r))
                s = r[order]
                C = np.cumsum(s)
                n_star = int((C <= p).sum()) + 1
                N_k = min(M, max(n_star, K_top))
                if N_k < M:
                    min_gap = min(min_gap, (s[N_k - 1] - s[N_k]) / s[N_k - 1])
                min_c = min(min_c, np.abs(C - p).min())
    return float(min_gap), float(min_c)


# --------------------------------------------------------------------------- Alg. 4 / Eq. 1

def attention_block(q, k, v, mask_row, lay, i, beta=0.0, return_lse=False):
    """Output rows of query block i of one (batch, head).

    q, k, v: float64 [N_pad, d] in curve order.  mask_row: bool [M].
    Keys: the valid tokens of the selected blocks.  Logit = q.k/sqrt(d), plus beta when
    the query block is a vision block and the key block is a text block (added after the
    scaling).  Pad query rows give zeros.  Returns [m, d].

    return_lse: also return [m] with the natural-log sum of exp(logit) over the same keys
    (the normaliser of Eq. 1 restricted to the visited set, Alg. 4's running l and m combined);
    -inf for pad query rows and for rows without any key.
    """
    m, d = lay.m, q.shape[-1]
    out = np.zeros((m, d), dtype=np.float64)
    lse = np.full(m, -np.inf)
    rows = np.nonzero(lay.valid[i * m:(i + 1) * m])[0]
    cols = []
    bias = []
    for j in np.nonzero(mask_row)[0]:
        c = np.nonzero(lay.valid[j * m:(j + 1) * m])[0] + j * m
        cols.append(c)
        is_bias = (i < lay.M_v) and (j >= lay.M_v)
        bias.append(np.full(len(c), beta if is_bias else 0.0))
    if len(rows) > 0 and len(cols) > 0:
        cols = np.concatenate(cols)
        bias = np.concatenate(bias)
        logits = q[rows + i * m] @ k[cols].T / math.sqrt(d) + bias[None, :]
        top = logits.max(axis=1, keepdims=True)
        P = np.exp(logits - top)
        denom = P.sum(axis=1, keepdims=True)
        out[rows] = (P / denom) @ v[cols]
        lse[rows] = top[:, 0] + np.log(denom[:, 0])
    if return_lse:
        return out, lse
    return out


def block_sparse_attention(q, k, v, mask, lay, beta=0.0, only=None, return_lse=False):
    """q, k, v float64 [B, heads, N_pad, d]; mask bool [B, heads, M, M] -> O like q.

    only: optional iterable of (b, h, i) to compute (other rows stay zero).
    return_lse: also return the log-sum-exp of every row, [B, heads, N_pad] (see attention_block).
    """
    B, Hh, Np, D = q.shape
    out = np.zeros_like(q)
    lse = np.full((B, Hh, Np), -np.inf)
    todo = only if only is not None else [(b, h, i) for b in range(B) for h in range(Hh) for i in range(lay.M)]
    m = lay.m
    for (b, h, i) in todo:
        o, l = attention_block(q[b, h], k[b, h], v[b, h], mask[b, h, i], lay, i, beta, return_lse=True)
        out[b, h, i * m:(i + 1) * m] = o
        lse[b, h, i * m:(i + 1) * m] = l
    if return_lse:
        return out, lse
    return out


def dense_attention(q_thw, k_thw, v_thw):
    """Eq. 1 on [B, N, heads, d] float64 tensors in any consistent token order."""
    d = q_thw.shape[-1]
    logits = np.einsum("bnhd,bmhd->bhnm", q_thw, k_thw) / math.sqrt(d)
    logits -= logits.max(axis=-1, keepdims=True)
    P = np.exp(logits)
    P /= P.sum(axis=-1, keepdims=True)
    return np.einsum("bhnm,bmhd->bnhd", P, v_thw)


def mask_to_lists(mask):
    """Ascending index lists and counts from a boolean mask [B, heads, M, M]."""
    B, Hh, M, _ = mask.shape
    count = mask.sum(axis=-1).astype(np.int32)
    index = np.full((B, Hh, M, M), -1, dtype=np.int32)
    for b in range(B):
        for h in range(Hh):
            for i in range(M):
                idx = np.nonzero(mask[b, h, i])[0]
                index[b, h, i, : len(idx)] = idx
    return count, index


def carve_layer(q_thw_bits, k_thw_bits, v_thw_bits, lay, p, beta=0.0):
    """Whole path on bf16 bit patterns [B, N, heads, d]: permute -> mask -> attention -> unpermute.

    Returns (out_thw float64, mask, out_curve).
    """
    q = permute(bf16_bits_to_f64(q_thw_bits), lay)
    k = permute(bf16_bits_to_f64(k_thw_bits), lay)
    v = permute(bf16_bits_to_f64(v_thw_bits), lay)
    mask = build_mask(q, k, lay, p)
    o = block_sparse_attention(q, k, v, mask, lay, beta)
    return unpermute(o, lay), mask, o
