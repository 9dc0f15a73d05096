"""CPU oracle for the E-Sparse hot path.  TEST INFRASTRUCTURE ONLY.

A plain, slow, float64 / exact-integer implementation of what the HIP library
computes, written from the paper (E-Sparse, arXiv 2310.15929) and sharing no code
with the library.  Only tests, the smoke check and the benchmark's CPU-baseline leg
may import it; the product never does.

Notation (the paper overloads its symbols, so this file fixes its own):
  Xc[T, K]  calibration features, T tokens (all sequences pooled) x K input channels
  W[N, K]   weights of one linear layer, N output rows x K input channels
  X[M, K]   inference activations, Y[M, N] = X . W_sparse^T
  n : m     keep n of every m consecutive (re-ordered) input channels of each row
  theta     gather permutation: re-ordered position p holds original channel theta[p]
  B         local-block-shuffle block size (positions), bins = number of histogram bins

Every function names the passage of the paper it follows.  Where the paper leaves a
choice open the choice is stated in the docstring ("Reading: ...").

Pins (tests/test_oracle_pins.py) tie each function to something other than itself:
closed forms, library routines, brute force, invariants.  No numeric worked example
is printed in the paper for any of these steps, so agreement with the authors' own
implementation is NOT pinned: the readings of alpha, of the bin range, of the GNS
dealing pattern and of the greedy search could differ from what the authors ran.
"""
from __future__ import annotations

import itertools
import math

import numpy as np

# --------------------------------------------------------------------------------------
# Section 3.2, eq. (1): information richness (entropy) of every channel
# --------------------------------------------------------------------------------------

def channel_histogram(Xc: np.ndarray, bins: int = 100) -> np.ndarray:
    """Counts n[c, k] of channel c's T calibration values in `bins` equal-width bins.

    Section 3.2: the channel's values are divided into K bins (K = 100 in the paper).
    Reading: the bins span the channel's own range [lo, hi] = [min_t x, max_t x]; the
    top edge is closed, i.e. bin(x) = min(bins-1, floor((x - lo) * bins / (hi - lo)));
    a constant channel (hi == lo) puts everything in bin 0.
    """
    X = np.asarray(Xc, dtype=np.float64)
    T, K = X.shape
    counts = np.zeros((K, bins), dtype=np.int64)
    for c in range(K):
        x = X[:, c]
        lo = x.min()
        hi = x.max()
        if hi == lo:
            counts[c, 0] = T
            continue
        b = np.floor((x - lo) * float(bins) / (hi - lo))
        b = np.minimum(b, float(bins - 1)).astype(np.int64)
        counts[c] = np.bincount(b, minlength=bins)
    return counts


def channel_entropy(Xc: np.ndarray, bins: int = 100) -> np.ndarray:
    """IR_c = - sum_k p_k ln p_k with p_k = n_k / T   (eq. 1).

    Reading: natural logarithm; empty bins contribute 0 (the limit of p ln p); the sum
    runs over k in ascending order in float64 with the C library's log.
    """
    counts = channel_histogram(Xc, bins)
    T = int(np.asarray(Xc).shape[0])
    K = counts.shape[0]
    IR = np.zeros(K, dtype=np.float64)
    for c in range(K):
        acc = 0.0
        for k in range(bins):
            nk = int(counts[c, k])
            if nk > 0:
                p = float(nk) / float(T)
                acc = acc + p * math.log(p)
        IR[c] = -acc
    return IR


# --------------------------------------------------------------------------------------
# Section 3.2, eq. (2): amplitude of every channel
# --------------------------------------------------------------------------------------

def channel_amplitude(Xc: np.ndarray) -> np.ndarray:
    """AM_c = || X_c ||_2 over the T tokens  (eq. 2).

    The squares of 16-bit inputs are exact in float64; their sum is taken exactly and
    rounded once (math.fsum), followed by one correctly rounded square root.
    """
    X = np.asarray(Xc, dtype=np.float64)
    K = X.shape[1]
    AM = np.zeros(K, dtype=np.float64)
    for c in range(K):
        col = X[:, c]
        AM[c] = math.sqrt(math.fsum((col * col).tolist()))
    return AM


# --------------------------------------------------------------------------------------
# Section 3.2, eq. (3): pruning metric
# --------------------------------------------------------------------------------------

def channel_score(Xc: np.ndarray, alpha: float, bins: int = 100,
                  use_entropy: bool = True, use_norm: bool = True) -> np.ndarray:
    """s_c = IR_c + alpha * AM_c, the per-channel factor of eq. (3).

    The two switches reproduce the ablation rows of Table 4 (norm only = the metric of
    Wanda when alpha = 1; norm + entropy = the full metric).
    """
    K = np.asarray(Xc).shape[1]
    s = np.zeros(K, dtype=np.float64)
    if use_entropy:
        s = s + channel_entropy(Xc, bins)
    if use_norm:
        s = s + float(alpha) * channel_amplitude(Xc)
    return s


def metric(W: np.ndarray, s: np.ndarray) -> np.ndarray:
    """xi[j, c] = |w[j, c]| * s_c  (eq. 3); one float64 multiplication per element."""
    return np.abs(np.asarray(W, dtype=np.float64)) * np.asarray(s, dtype=np.float64)[None, :]


# --------------------------------------------------------------------------------------
# Section 3.3: global naive shuffle (Algorithm 1, step 1)
# --------------------------------------------------------------------------------------

def channel_mean_metric(W: np.ndarray, s: np.ndarray) -> np.ndarray:
    """g_c = mean over output rows of xi[:, c].

    Reading: since xi[:, c] = |w[:, c]| * s_c the mean is evaluated as
    (s_c * sum_j |w[j, c]|) / N with the column sum exact (math.fsum), which makes the
    value independent of the order in which rows are visited.
    """
    A = np.abs(np.asarray(W, dtype=np.float64))
    N, K = A.shape
    g = np.zeros(K, dtype=np.float64)
    for c in range(K):
        colsum = math.fsum(A[:, c].tolist())
        g[c] = (float(s[c]) * colsum) / float(N)
    return g


def global_naive_shuffle(W: np.ndarray, s: np.ndarray, m: int) -> np.ndarray:
    """theta0 from the global naive shuffle (Section 3.3, Fig. 3a caption).

    Channels are ranked by g_c in descending order (ties: lower channel index first) and
    then dealt so that channels with close means land in different groups of m.
    Reading (the figure is not available): plain round-robin.  With G = K / m groups, the
    channel of rank r goes to position (r mod G) * m + (r div G).
    """
    g = channel_mean_metric(W, s)
    K = g.shape[0]
    assert K % m == 0
    G = K // m
    order = np.argsort(-g, kind="stable")          # rank r -> channel
    theta0 = np.empty(K, dtype=np.int64)
    for r in range(K):
        p = (r % G) * m + (r // G)
        theta0[p] = order[r]
    return theta0


# --------------------------------------------------------------------------------------
# eq. (5): retained metric of a set of m channels
# --------------------------------------------------------------------------------------

def _top_n_sum_rows(xi_cols: np.ndarray, n: int) -> np.ndarray:
    """Per row: the n largest of the m values, added largest first.  xi_cols[N, m]."""
    srt = -np.sort(-xi_cols, axis=1)               # descending
    t = srt[:, 0].copy()
    for q in range(1, n):
        t = t + srt[:, q]
    return t


def sum_rows(t: np.ndarray, order="sequential") -> float:
    """Sum of the per-row terms t[0..N-1] in float64.

    Reading (eq. 5 does not say in which order its terms are added, and float64 addition is not
    associative): the plain one - rows in ascending order, one running sum.  The other orders exist
    for the pin that shows the search result does not depend on this choice on the workloads:
    ("lanes", L): L interleaved sub-sums (sub-sum l takes rows l, l + L, ...) added in ascending l;
    "exact": the correctly rounded sum (math.fsum).
    """
    if order == "sequential":
        acc = 0.0
        for j in range(t.shape[0]):
            acc = acc + float(t[j])
        return acc
    if order == "exact":
        return math.fsum(t.tolist())
    kind, L = order
    assert kind == "lanes"
    lanes = [0.0] * L
    for j in range(t.shape[0]):
        lanes[j % L] = lanes[j % L] + float(t[j])
    acc = lanes[0]
    for l in range(1, L):
        acc = acc + lanes[l]
    return acc


def group_value(xi_cols: np.ndarray, n: int, order="sequential") -> float:
    """v(g) = sum over the output rows of the row's retained metric in the group: the
    contribution of one group of m channels to eq. (5).  Rows are added in ascending order."""
    t = _top_n_sum_rows(np.asarray(xi_cols, dtype=np.float64), n)
    return sum_rows(t, order)


def retained_metric(W: np.ndarray, s: np.ndarray, theta: np.ndarray, n: int, m: int) -> float:
    """Objective of eq. (5): total metric kept by n:m sparsity under channel order theta."""
    xi = metric(W, s)[:, np.asarray(theta)]
    K = xi.shape[1]
    total = 0.0
    for g in range(K // m):
        total = total + group_value(xi[:, g * m:(g + 1) * m], n)
    return total


# --------------------------------------------------------------------------------------
# Section 3.3: local block shuffle (Algorithm 1, steps 3-14)
# --------------------------------------------------------------------------------------

def _block_swap_search(xi_blk: np.ndarray, n: int, m: int, order="sequential"):
    """One call of the search step of Algorithm 1 on a block whose columns are in the
    block's current order.  Returns (i, j, delta) for the pair of positions in different
    groups whose exchange raises the retained metric most, or None if no exchange raises it.

    Reading: exhaustive over all position pairs i < j in different groups;
    delta(i, j) = (v(a') + v(b')) - (v(a) + v(b)) where a, b are the groups of i, j before
    and a', b' after the exchange; the largest delta wins, ties go to the smallest (i, j);
    only delta > 0 counts.
    """
    Bsz = xi_blk.shape[1]
    G = Bsz // m
    v = [group_value(xi_blk[:, g * m:(g + 1) * m], n, order) for g in range(G)]
    best = None
    for i in range(Bsz):
        a = i // m
        for j in range(i + 1, Bsz):
            b = j // m
            if a == b:
                continue
            cols_a = list(range(a * m, (a + 1) * m))
            cols_b = list(range(b * m, (b + 1) * m))
            cols_a[i - a * m] = j
            cols_b[j - b * m] = i
            va2 = group_value(xi_blk[:, cols_a], n, order)
            vb2 = group_value(xi_blk[:, cols_b], n, order)
            delta = (va2 + vb2) - (v[a] + v[b])
            if delta > 0.0 and (best is None or delta > best[2]):
                best = (i, j, delta)
    return best


def local_block_shuffle(W: np.ndarray, s: np.ndarray, theta0: np.ndarray, n: int, m: int,
                        B: int, max_swaps: int = 0, blocks=None, order="sequential"):
    """Greedy channel exchanges inside blocks of B consecutive positions (Algorithm 1).

    For every block: repeat { find the best exchange; stop if none improves; apply it and
    update theta }.  `max_swaps` > 0 caps the number of exchanges per block (0 = no cap).
    `blocks` restricts the work to the listed block numbers (others keep theta0); `order` is
    the order of the row sums (see sum_rows).  Returns (theta, swaps_per_block).
    """
    theta = np.array(theta0, dtype=np.int64).copy()
    K = theta.shape[0]
    assert K % B == 0 and B % m == 0
    xi_full = metric(W, s)
    nblk = K // B
    swaps = np.zeros(nblk, dtype=np.int64)
    todo = range(nblk) if blocks is None else blocks
    for blk in todo:
        lo = blk * B
        while True:
            if max_swaps > 0 and swaps[blk] >= max_swaps:
                break
            xi_blk = xi_full[:, theta[lo:lo + B]]
            res = _block_swap_search(xi_blk, n, m, order)
            if res is None:
                break
            i, j = res[0], res[1]
            theta[lo + i], theta[lo + j] = theta[lo + j], theta[lo + i]
            swaps[blk] += 1
    return theta, swaps


# --------------------------------------------------------------------------------------
# n:m mask (Sections 1, 3.1, 3.3: keep n of every m consecutive re-ordered channels)
# --------------------------------------------------------------------------------------

def nm_mask(W: np.ndarray, s: np.ndarray, theta: np.ndarray, n: int, m: int) -> np.ndarray:
    """mask'[j, p] in {0, 1}, in RE-ORDERED channel order: inside every group of m
    consecutive positions of every row the n largest xi are kept (ties: lower position)."""
    xi = metric(W, s)[:, np.asarray(theta)]
    N, K = xi.shape
    mask = np.zeros((N, K), dtype=np.uint8)
    for j in range(N):
        for g in range(K // m):
            grp = xi[j, g * m:(g + 1) * m]
            keep = np.argsort(-grp, kind="stable")[:n]
            mask[j, g * m + keep] = 1
    return mask


def mask_to_original_order(mask_reordered: np.ndarray, theta: np.ndarray) -> np.ndarray:
    out = np.zeros_like(mask_reordered)
    out[:, np.asarray(theta)] = mask_reordered
    return out


# --------------------------------------------------------------------------------------
# Section 4, step 1: compressed format (kept values + indices of the kept values)
# --------------------------------------------------------------------------------------

def compress(W: np.ndarray, theta: np.ndarray, mask_reordered: np.ndarray, n: int, m: int):
    """Kept values and their in-group indices.

    values[N, K*n/m] : W[j, theta[p]] of the kept positions p, ascending p, dtype of W.
    2:4  -> meta uint32[N, ceil(K/2 / 16)]: field f (the f-th kept value of the row) holds
            the position of that value inside its group of 4 (2 bits) at bit 2*(f mod 16) of
            word f div 16.
    4:8  -> meta uint8[N, K/8]: occupancy bitmap of each group of 8 (bit i = position i kept).
    Both cost 2 bits per kept value: K/8 bytes per row.
    """
    W = np.asarray(W)
    Wp = W[:, np.asarray(theta)]
    N, K = Wp.shape
    G = K // m
    kept = n * G
    values = np.zeros((N, kept), dtype=W.dtype)
    if m == 4:
        meta = np.zeros((N, (kept + 15) // 16), dtype=np.uint32)
    else:
        meta = np.zeros((N, G), dtype=np.uint8)
    for j in range(N):
        f = 0
        for g in range(G):
            pos = [i for i in range(m) if mask_reordered[j, g * m + i]]
            assert len(pos) == n, "group does not keep exactly n"
            for i in pos:
                values[j, f] = Wp[j, g * m + i]
                if m == 4:
                    meta[j, f // 16] |= np.uint32(i << (2 * (f % 16)))
                else:
                    meta[j, g] |= np.uint8(1 << i)
                f += 1
    return values, meta


def decompress(values: np.ndarray, meta: np.ndarray, K: int, n: int, m: int) -> np.ndarray:
    """Inverse of `compress`: the masked weights in re-ordered channel order."""
    N = values.shape[0]
    out = np.zeros((N, K), dtype=values.dtype)
    G = K // m
    for j in range(N):
        f = 0
        for g in range(G):
            if m == 4:
                for _ in range(n):
                    i = (int(meta[j, f // 16]) >> (2 * (f % 16))) & 3
                    out[j, g * m + i] = values[j, f]
                    f += 1
            else:
                for i in range(m):
                    if (int(meta[j, g]) >> i) & 1:
                        out[j, g * m + i] = values[j, f]
                        f += 1
    return out


def compressed_bytes(N: int, K: int, n: int, m: int, elem_bytes: int = 2):
    """Closed form: (values bytes, metadata bytes).  2 bits per kept value."""
    kept = N * K * n // m
    return kept * elem_bytes, (kept * 2 + 7) // 8


def native_tiling(values: np.ndarray, meta: np.ndarray, N: int, K: int):
    """Re-arrangement of the canonical 2:4 arrays into the order the SpMM kernels stream.

    A pure index map (documented in include/esparse.h).  Rows are padded to a multiple of
    16 and K to a multiple of 256 with zeros.  The unit is (row, 16 re-ordered channels) =
    8 kept values (16 bytes) + their 8 two-bit fields (one uint16).
      values unit order : [row tile rt = row // 16][k-step ks = chunk // 4][ga = chunk % 4][r = row % 16]
      meta   unit order : [rt][ks // 4][ga][r][ks % 4]
    Returns (native_values[Np*Kp/2] of the value dtype, native_meta[Np*Kp/16] uint16).
    """
    Np = -(-N // 16) * 16
    Kp = -(-K // 256) * 256
    nchunk = Kp // 16
    v = np.zeros((Np, nchunk, 8), dtype=values.dtype)
    v.reshape(Np, nchunk * 8)[:N, :K // 2] = values
    m16 = np.zeros((Np, nchunk), dtype=np.uint16)
    meta16 = np.ascontiguousarray(meta).view(np.uint16)      # little-endian halves, 8 fields each
    m16[:N, :meta16.shape[1]] = meta16
    nv = np.zeros((Np // 16, nchunk // 4, 4, 16, 8), dtype=values.dtype)
    nm = np.zeros((Np // 16, nchunk // 16, 4, 16, 4), dtype=np.uint16)
    for row in range(Np):
        rt, r = divmod(row, 16)
        for ch in range(nchunk):
            ks, ga = divmod(ch, 4)
            nv[rt, ks, ga, r, :] = v[row, ch, :]
            nm[rt, ks // 4, ga, r, ks % 4] = m16[row, ch]
    return nv.reshape(-1), nm.reshape(-1)


def native_tiling_4_8(values: np.ndarray, meta: np.ndarray, N: int, K: int):
    """Re-arrangement of the canonical 4:8 arrays into the order the 4:8 product streams.

    A pure index map (documented in include/esparse.h), same size and unit numbering as the
    2:4 one.  The group of row 16 rt + r that covers re-ordered channels 64 ks + 32 h + 8 g ..
    + 8 belongs to lane 16 g + r: its 4 kept values (8 bytes) are the half h of the 16-byte
    value unit (rt * nks + ks) * 64 + lane, its pattern code the byte h of the 16-bit metadata unit
    ordered [rt][ks // 4][g][r][ks % 4].  The pattern code of a group is the index of its occupancy
    bitmap in the ascending list of the 70 bitmaps with four bits set.  Padding (rows to 16, K to
    256) is zero: zero values, code 0.
    Returns (native_values[Np*Kp/2] of the value dtype, native_meta[Np*Kp/8] uint8).
    """
    patterns = [b for b in range(256) if bin(b).count("1") == 4]        # ascending; 70 of them
    code_of = np.zeros(256, dtype=np.uint8)
    for code, b in enumerate(patterns):
        code_of[b] = code
    Np = -(-N // 16) * 16
    Kp = -(-K // 256) * 256
    nks = Kp // 64
    v = np.zeros((Np, Kp // 8, 4), dtype=values.dtype)
    v.reshape(Np, Kp // 2)[:N, :K // 2] = values
    mb = np.zeros((Np, Kp // 8), dtype=np.uint8)
    mb[:N, :K // 8] = code_of[np.asarray(meta, dtype=np.uint8).reshape(N, K // 8)]
    nv = np.zeros((Np // 16, nks, 64, 2, 4), dtype=values.dtype)
    nm = np.zeros((Np // 16, nks // 4, 64, 4, 2), dtype=np.uint8)
    for row in range(Np):
        rt, r = divmod(row, 16)
        for q in range(Kp // 8):
            ks, rem = divmod(q, 8)
            h, g = divmod(rem, 4)
            lane = 16 * g + r
            nv[rt, ks, lane, h, :] = v[row, q, :]
            nm[rt, ks // 4, lane, ks % 4, h] = mb[row, q]
    return nv.reshape(-1), nm.reshape(-1)


# --------------------------------------------------------------------------------------
# Section 4: the products
# --------------------------------------------------------------------------------------

def spmm_ref(X: np.ndarray, W: np.ndarray, theta: np.ndarray, mask_reordered: np.ndarray) -> np.ndarray:
    """Y = X . (W with the pruned weights set to zero)^T in float64, no output rounding."""
    W64 = np.asarray(W, dtype=np.float64)
    keep = mask_to_original_order(np.asarray(mask_reordered), theta).astype(np.float64)
    return np.asarray(X, dtype=np.float64) @ (W64 * keep).T


def dense_ref(X: np.ndarray, W: np.ndarray) -> np.ndarray:
    """Y = X . W^T in float64 (the dense GEMM column of Table 5)."""
    return np.asarray(X, dtype=np.float64) @ np.asarray(W, dtype=np.float64).T


def rowwise_rel_error(Y: np.ndarray, Yref: np.ndarray) -> np.ndarray:
    """|| Y[t,:] - Yref[t,:] ||_2 / || Yref[t,:] ||_2 for every token t."""
    Y = np.asarray(Y, dtype=np.float64)
    num = np.sqrt(((Y - Yref) ** 2).sum(axis=1))
    den = np.sqrt((Yref ** 2).sum(axis=1))
    return num / np.where(den == 0.0, 1.0, den)


# --------------------------------------------------------------------------------------
# eq. (4): output error of a pruned layer (report only)
# --------------------------------------------------------------------------------------

def output_error(X: np.ndarray, W: np.ndarray, theta: np.ndarray, mask_reordered: np.ndarray) -> float:
    """|| X W^T - X W_{n:m}^T ||_F^2 / || X W^T ||_F^2, the relative form of eq. (4)."""
    Yd = dense_ref(X, W)
    Ys = spmm_ref(X, W, theta, mask_reordered)
    return float(((Yd - Ys) ** 2).sum() / (Yd ** 2).sum())


# --------------------------------------------------------------------------------------
# whole offline pipeline (Section 3.1 overview; Table 4 switches)
# --------------------------------------------------------------------------------------

def prune(Xc: np.ndarray, W: np.ndarray, n: int, m: int, B: int, alpha: float, bins: int = 100,
          use_entropy: bool = True, use_norm: bool = True, use_gns: bool = True,
          use_lbs: bool = True, max_swaps: int = 0, fast: bool = True):
    """calibration features + weights -> (theta, mask', s, swaps_per_block)."""
    s = channel_score(Xc, alpha, bins, use_entropy, use_norm)
    K = W.shape[1]
    theta = global_naive_shuffle(W, s, m) if use_gns else np.arange(K, dtype=np.int64)
    swaps = np.zeros(K // B if B else 0, dtype=np.int64)
    if use_lbs:
        lbs = local_block_shuffle_vectorised if fast else local_block_shuffle
        theta, swaps = lbs(W, s, theta, n, m, B, max_swaps)
    mask = nm_mask_vectorised(W, s, theta, n, m) if fast else nm_mask(W, s, theta, n, m)
    return theta, mask, s, swaps


# --------------------------------------------------------------------------------------
# Same definitions as above with the loops over candidates / groups done by numpy, used
# where the loop versions would take hours.  tests/test_oracle_pins.py checks that they
# return bit-identical results to the loop versions on small inputs.
# --------------------------------------------------------------------------------------

def _sum_rows_axis0(t: np.ndarray, order="sequential") -> np.ndarray:
    """`sum_rows` for every column of t at once (axis 0 = rows): the same additions in the same
    order, each a numpy operation over the columns."""
    if order == "sequential":
        acc = np.zeros(t.shape[1:], dtype=np.float64)
        for j in range(t.shape[0]):
            acc = acc + t[j]
        return acc
    if order == "exact":
        flat = t.reshape(t.shape[0], -1)
        out = np.array([math.fsum(flat[:, q].tolist()) for q in range(flat.shape[1])], dtype=np.float64)
        return out.reshape(t.shape[1:])
    kind, L = order
    assert kind == "lanes"
    N = t.shape[0]
    pad = (-N) % L
    if pad:     # +0.0 changes no sum of non-negative terms
        t = np.concatenate([t, np.zeros((pad,) + t.shape[1:], dtype=np.float64)], axis=0)
    r = t.reshape((t.shape[0] // L, L) + t.shape[1:])
    lanes = np.zeros(r.shape[1:], dtype=np.float64)
    for q in range(r.shape[0]):
        lanes = lanes + r[q]
    acc = lanes[0]
    for l in range(1, L):
        acc = acc + lanes[l]
    return acc


def _top_n_sum_lastaxis(x: np.ndarray, n: int) -> np.ndarray:
    srt = -np.sort(-x, axis=-1)
    t = srt[..., 0].copy()
    for q in range(1, n):
        t = t + srt[..., q]
    return t


def _block_swap_search_vectorised(xi_blk: np.ndarray, n: int, m: int, order="sequential"):
    N, Bsz = xi_blk.shape
    G = Bsz // m
    v = _sum_rows_axis0(_top_n_sum_lastaxis(xi_blk.reshape(N, G, m), n), order)       # [G]
    pairs = [(i, j) for i in range(Bsz) for j in range(i + 1, Bsz) if i // m != j // m]
    best = None
    chunk = max(1, (1 << 24) // max(1, N * 2 * m))
    for lo in range(0, len(pairs), chunk):
        pr = pairs[lo:lo + chunk]
        P = len(pr)
        cols = np.empty((P, 2, m), dtype=np.int64)
        for q, (i, j) in enumerate(pr):
            a, b = i // m, j // m
            ca = np.arange(a * m, (a + 1) * m)
            cb = np.arange(b * m, (b + 1) * m)
            ca[i - a * m] = j
            cb[j - b * m] = i
            cols[q, 0] = ca
            cols[q, 1] = cb
        vals = _sum_rows_axis0(_top_n_sum_lastaxis(xi_blk[:, cols], n), order)          # [P, 2]
        for q, (i, j) in enumerate(pr):
            a, b = i // m, j // m
            delta = (float(vals[q, 0]) + float(vals[q, 1])) - (float(v[a]) + float(v[b]))
            if delta > 0.0 and (best is None or delta > best[2]):
                best = (i, j, delta)
    return best


def local_block_shuffle_vectorised(W, s, theta0, n, m, B, max_swaps=0, blocks=None, order="sequential"):
    theta = np.array(theta0, dtype=np.int64).copy()
    K = theta.shape[0]
    assert K % B == 0 and B % m == 0
    A = np.abs(np.asarray(W, dtype=np.float64))
    s = np.asarray(s, dtype=np.float64)
    nblk = K // B
    swaps = np.zeros(nblk, dtype=np.int64)
    todo = range(nblk) if blocks is None else blocks
    for blk in todo:
        lo = blk * B
        while True:
            if max_swaps > 0 and swaps[blk] >= max_swaps:
                break
            ch = theta[lo:lo + B]
            xi_blk = A[:, ch] * s[ch][None, :]
            res = _block_swap_search_vectorised(xi_blk, n, m, order)
            if res is None:
                break
            i, j = res[0], res[1]
            theta[lo + i], theta[lo + j] = theta[lo + j], theta[lo + i]
            swaps[blk] += 1
    return theta, swaps


def nm_mask_vectorised(W, s, theta, n, m, rows=None):
    A = np.abs(np.asarray(W, dtype=np.float64))
    if rows is not None:
        A = A[rows]
    xi = (A * np.asarray(s, dtype=np.float64)[None, :])[:, np.asarray(theta)]
    N, K = xi.shape
    grp = xi.reshape(N, K // m, m)
    order = np.argsort(-grp, axis=2, kind="stable")[:, :, :n]
    mask = np.zeros((N, K // m, m), dtype=np.uint8)
    np.put_along_axis(mask, order, 1, axis=2)
    return mask.reshape(N, K)


def compress_vectorised(W, theta, mask_reordered, n, m):
    W = np.asarray(W)
    Wp = W[:, np.asarray(theta)]
    N, K = Wp.shape
    G = K // m
    mk = np.asarray(mask_reordered).astype(bool)
    assert (mk.reshape(N, G, m).sum(axis=2) == n).all(), "group does not keep exactly n"
    values = Wp[mk].reshape(N, n * G)
    if m == 4:
        pos = np.broadcast_to(np.arange(K) % m, (N, K))[mk].reshape(N, n * G).astype(np.uint32)
        kept = n * G
        pad = (-kept) % 16
        if pad:
            pos = np.concatenate([pos, np.zeros((N, pad), dtype=np.uint32)], axis=1)
        f = pos.reshape(N, -1, 16)
        sh = (2 * np.arange(16, dtype=np.uint32))[None, None, :]
        meta = np.bitwise_or.reduce(f << sh, axis=2).astype(np.uint32)
    else:
        bits = (mk.reshape(N, G, m).astype(np.uint32) << np.arange(m, dtype=np.uint32)[None, None, :])
        meta = bits.sum(axis=2).astype(np.uint8)
    return values, meta


def brute_force_best_partition(xi_blk: np.ndarray, n: int, m: int) -> float:
    """Largest retained metric over ALL ways of splitting the block's channels into groups
    of m (tiny blocks only; 8 channels, m = 4: 35 partitions)."""
    Bsz = xi_blk.shape[1]
    best = -1.0

    def rec(remaining, acc):
        nonlocal best
        if not remaining:
            best = max(best, acc)
            return
        first = remaining[0]
        rest = remaining[1:]
        for comb in itertools.combinations(rest, m - 1):
            cols = [first] + list(comb)
            left = [c for c in rest if c not in comb]
            rec(left, acc + group_value(xi_blk[:, cols], n))

    rec(list(range(Bsz)), 0.0)
    return best
