"""CPU oracle for the weight-side steps: masking, pattern assignment, connectivity selection, canonical packing.

TEST INFRASTRUCTURE ONLY: imported by tests, the smoke check and the bench's cpu_baseline leg; never by the product
path, with which it shares no code.  Plain numpy, float64 arithmetic, no blocking or reordering.

Notation follows the paper: a layer's weights are W[f][c][ky][kx] (F filters, C channels, section 6.1), a pattern is
a binary 3x3 mask M_j of the library Omega = {M_1..M_K} with exactly four ones (section 5.1), the selection variable
z is stored as the index `pid[f][c]` of the chosen mask, and the connectivity score of a kernel is its L2 norm
(gamma, section 6.1).  A mask is a 9-bit integer with bit t = 3*ky + kx set where the weight is kept.
"""
from __future__ import annotations

import numpy as np


def library_bits(lib) -> np.ndarray:
    """[K][9] array of 0/1 from the K 9-bit masks; rejects masks that do not keep exactly four taps."""
    lib = np.asarray(lib, dtype=np.int64)
    bits = (lib[:, None] >> np.arange(9)[None, :]) & 1
    if lib.size == 0 or np.any(lib < 0) or np.any(lib >= 512) or np.any(bits.sum(axis=1) != 4):
        raise ValueError("every library mask must be a 9-bit value with exactly four bits set")
    return bits


def mask_weights(w, pid, mask, lib) -> np.ndarray:
    """Wm = W o M_{pid} for kept kernels, 0 for removed ones (section 4.1: pruning is an element-wise product with
    a binary mask; section 3: a removed kernel is a cut connection).  Same dtype and shape as w."""
    w = np.asarray(w)
    F, C = w.shape[:2]
    bits = library_bits(lib)
    pid = np.asarray(pid).reshape(F, C).astype(np.int64)
    keep = np.asarray(mask).reshape(F, C) != 0
    if np.any(pid[keep] >= bits.shape[0]):
        raise ValueError("pattern id outside the library")
    sel = bits[np.where(keep, pid, 0)].reshape(F, C, 3, 3).astype(bool) & keep[:, :, None, None]
    return np.where(sel, w, np.zeros((), dtype=w.dtype))


def retained_energy(w, lib) -> np.ndarray:
    """[F][C][K] float64: for every kernel and every mask, the sum of squares of the weights the mask keeps, added
    in ascending tap order (each product and each sum rounded once to double)."""
    w = np.asarray(w)
    F, C = w.shape[:2]
    sq = w.reshape(F, C, 9).astype(np.float64)
    sq = sq * sq
    bits = library_bits(lib)
    out = np.zeros((F, C, bits.shape[0]), dtype=np.float64)
    for j in range(bits.shape[0]):
        taps = np.nonzero(bits[j])[0]          # ascending
        acc = sq[:, :, taps[0]].copy()
        for t in taps[1:]:
            acc = acc + sq[:, :, t]
        out[:, :, j] = acc
    return out


def assign_patterns(w, lib) -> np.ndarray:
    """pid[f][c] = the mask that keeps the most of the kernel's squared L2 norm, i.e. the Euclidean projection of
    the kernel onto the library (the hard selection that the argmax of z performs at the end of section 5.1);
    ties go to the lowest index."""
    return np.argmax(retained_energy(w, lib), axis=2).astype(np.uint8)


def select_connectivity(w, lib, pid, keep: float) -> np.ndarray:
    """mask[f][c] = 1 for the k = floor(keep*F*C + 0.5) kernels of the layer with the largest retained squared L2
    norm (gamma of section 6.1, taken on the pattern-pruned kernel and squared: same order), ties by ascending
    linear index f*C + c."""
    w = np.asarray(w)
    F, C = w.shape[:2]
    e = retained_energy(w, lib)
    score = np.take_along_axis(e, np.asarray(pid).reshape(F, C, 1).astype(np.int64), axis=2).reshape(-1)
    k = int(np.floor(float(keep) * float(F * C) + 0.5))
    k = max(0, min(k, F * C))
    order = np.lexsort((np.arange(F * C), -score))   # primary: score descending; secondary: index ascending
    mask = np.zeros(F * C, dtype=np.uint8)
    mask[order[:k]] = 1
    return mask.reshape(F, C)


def pack_canonical(w, pid, mask, lib):
    """Canonical pattern-grouped compressed form (the filter/kernel re-ordering of section 6.2 made concrete):

    filter_order[i]   filters sorted by kept-kernel count, descending, then by filter index, ascending
    grp_ptr[i*K + j]  start, in the entry arrays, of the kept kernels of filter filter_order[i] that use mask j;
                      grp_ptr[F*K] = number of kept kernels
    cin[e]            input channel of entry e; ascending inside each (filter, mask) group
    w4[e][0..3]       the four kept weights, in ascending tap order, copied bit for bit
    """
    w = np.asarray(w)
    F, C = w.shape[:2]
    bits = library_bits(lib)
    K = bits.shape[0]
    pid = np.asarray(pid).reshape(F, C).astype(np.int64)
    kept = np.asarray(mask).reshape(F, C) != 0
    if np.any(pid[kept] >= K):
        raise ValueError("pattern id outside the library")
    counts = kept.sum(axis=1)
    filter_order = np.lexsort((np.arange(F), -counts)).astype(np.uint32)
    taps = np.stack([np.nonzero(bits[j])[0] for j in range(K)])       # [K][4] ascending tap indices
    grp_ptr = np.zeros(F * K + 1, dtype=np.uint32)
    cin_parts, w_parts = [], []
    wf = w.reshape(F, C, 9)
    n = 0
    for i, f in enumerate(filter_order):
        for j in range(K):
            grp_ptr[i * K + j] = n
            cs = np.nonzero(kept[f] & (pid[f] == j))[0]
            if cs.size:
                cin_parts.append(cs.astype(np.uint16))
                w_parts.append(wf[f][cs][:, taps[j]])
                n += cs.size
    grp_ptr[F * K] = n
    cin = np.concatenate(cin_parts) if cin_parts else np.zeros(0, dtype=np.uint16)
    w4 = np.concatenate(w_parts) if w_parts else np.zeros((0, 4), dtype=w.dtype)
    return filter_order, grp_ptr, cin, np.ascontiguousarray(w4)


def unpack_canonical(filter_order, grp_ptr, cin, w4, lib, F: int, C: int) -> np.ndarray:
    """Inverse of pack_canonical: the masked dense tensor [F][C][3][3] with zeros everywhere else."""
    bits = library_bits(lib)
    K = bits.shape[0]
    w4 = np.asarray(w4)
    out = np.zeros((F, C, 9), dtype=w4.dtype)
    for i in range(F):
        f = int(filter_order[i])
        for j in range(K):
            a, b = int(grp_ptr[i * K + j]), int(grp_ptr[i * K + j + 1])
            taps = np.nonzero(bits[j])[0]
            for e in range(a, b):
                out[f, int(cin[e]), taps] = w4[e]
    return out.reshape(F, C, 3, 3)


def filter_similarity_order(mask, group: int) -> np.ndarray:
    """Filter re-ordering by similarity (the grouping of similar filters of section 6.2, made concrete as a greedy
    rule): groups of `group` filters; a group starts with the unplaced filter that keeps the most kernels (lowest
    index among equals) and takes, one at a time, the unplaced filter that adds the fewest channels to the union of the
    group's kept channels, among equals the one sharing the most channels with that union, then the lowest index."""
    keep = np.asarray(mask) != 0
    F = keep.shape[0]
    counts = keep.sum(axis=1).astype(np.int64)
    free = np.ones(F, dtype=bool)
    order = []
    while len(order) < F:
        cand = np.nonzero(free)[0]
        seed = int(cand[np.argmax(counts[cand])])           # argmax returns the first (lowest index) of equals
        free[seed] = False
        order.append(seed)
        union = keep[seed].copy()
        for _ in range(1, group):
            cand = np.nonzero(free)[0]
            if cand.size == 0:
                break
            add = (keep[cand] & ~union).sum(axis=1).astype(np.int64)
            share = (keep[cand] & union).sum(axis=1).astype(np.int64)
            best = int(cand[np.lexsort((cand, -share, add))[0]])
            free[best] = False
            order.append(best)
            union |= keep[best]
    return np.asarray(order, dtype=np.uint32)
