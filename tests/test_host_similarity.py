"""Filter re-ordering by similarity and the channel lists of the matrix-core path, on the CPU: the oracle's greedy rule
pinned by what it must do on planted structure and on a hand example, the library's order bit-equal to the oracle's,
and the number of channel blocks that a packed layer multiplies with and without the re-ordering."""
import numpy as np
import pytest

import oracle
import paper_2001_07710_amd as pc
from workloads import layers as L

RNG = np.random.default_rng(6207710)
LIB8 = np.array([0x01B, 0x036, 0x0D8, 0x1B0, 0x03A, 0x0B8, 0x0B2, 0x09A], dtype=np.uint16)


def planted(F, C, group, density=0.8):
    """Filters in clusters of `group`, scattered over the indices; cluster k keeps channels only inside its own
    disjoint slice of the channels."""
    clusters = F // group
    who = RNG.permutation(F) // group
    width = C // clusters
    mask = np.zeros((F, C), dtype=np.uint8)
    for f in range(F):
        k = who[f]
        mask[f, k * width:(k + 1) * width] = RNG.random(width) < density
        mask[f, k * width] = 1                    # (never empty)
    return mask, who


def test_hand_example_of_the_greedy_rule():
    m = np.array([[1, 1, 0, 0, 0, 0],     # 0
                  [0, 0, 1, 1, 1, 0],     # 1: most kernels -> first seed
                  [1, 1, 0, 0, 0, 1],     # 2
                  [0, 0, 1, 1, 0, 0],     # 3: adds nothing to {2,3,4}
                  [0, 0, 0, 1, 1, 0],     # 4: adds nothing either, shares as much as 3, higher index
                  [1, 0, 0, 0, 0, 0]],    # 5
                 dtype=np.uint8)
    # group 1: seed 1, then 3 (adds 0, shares 2; 4 ties and has the higher index); group 2: seed 2 (3 kernels),
    # then 0 (adds 0, shares 2) before 5 (adds 0, shares 1); group 3: 4, 5
    assert list(oracle.filter_similarity_order(m, 2)) == [1, 3, 2, 0, 4, 5]
    assert list(oracle.filter_similarity_order(m, 1)) == [1, 2, 0, 3, 4, 5]          # by count, then index
    # one group of all: after 1, 3, 4 the union is {2,3,4}; 5 adds one channel, 0 two, 2 three; then 0 adds one, 2 two
    assert list(oracle.filter_similarity_order(m, 6)) == [1, 3, 4, 5, 0, 2]


@pytest.mark.parametrize("shape", [(64, 64, 16), (96, 120, 32), (128, 64, 8)])
def test_planted_clusters_are_recovered(shape):
    F, C, group = shape
    mask, who = planted(F, C, group)
    order = oracle.filter_similarity_order(mask, group)
    assert sorted(order) == list(range(F))
    for g in range(F // group):
        members = order[g * group:(g + 1) * group]
        assert len(set(who[members])) == 1, "a group mixes two planted clusters"
    # the union of a group's channels is what its cluster keeps, not more
    natural = sum(int(mask[g * group:(g + 1) * group].any(axis=0).sum()) for g in range(F // group))
    ordered = sum(int(mask[order[g * group:(g + 1) * group]].any(axis=0).sum()) for g in range(F // group))
    assert ordered <= C and ordered * 2 < natural


@pytest.mark.parametrize("case", [(40, 33, 7, 0.3), (128, 96, 32, 0.1), (5, 9, 8, 0.9), (64, 200, 64, 0.5)])
def test_library_order_equals_the_oracles(case):
    F, C, group, density = case
    mask = (RNG.random((F, C)) < density).astype(np.uint8)
    mask[F // 2] = 0                                   # a filter that keeps nothing
    assert np.array_equal(pc.filter_similarity_order(mask, group), oracle.filter_similarity_order(mask, group))
    pm, _ = planted(64, 64, 16)
    assert np.array_equal(pc.filter_similarity_order(pm, 16), oracle.filter_similarity_order(pm, 16))
    with pytest.raises(pc.PconvError):
        pc.filter_similarity_order(mask, 0)


def test_channel_lists_follow_the_reordering():
    # 256 filters in 4 clusters of 64 over 128 channels, each cluster keeping a third of the channels: in their own
    # order every tile of 64 filters sees every channel; re-ordered, a tile is a cluster
    spec = L.LayerSpec(cfg=40, idx=0, name="clustered", N=1, C=128, F=256, H=8, W=8, dtype="f16", K=8, keep=0.25)
    w, _ = L.gen_clustered_weights(spec, clusters=4, share=1.0 / 3.0)
    lib = spec.library()
    pid = oracle.assign_patterns(w.astype(np.float32), lib)
    mask = oracle.select_connectivity(w.astype(np.float32), lib, pid, spec.keep)
    p = pc.pack(w, lib, pid, mask, pc.PACK_HOST_ONLY)
    listed, dense = pc.packed_mfma_blocks(p, 64)
    assert dense == 4 * 8 and listed >= 24          # (a tile of scattered filters sees the union of all clusters)
    order = pc.filter_similarity_order(mask, 64)
    q = pc.pack(w[order], lib, pid[order], mask[order], pc.PACK_HOST_ONLY)
    listed, dense = pc.packed_mfma_blocks(q, 64)
    assert dense == 32 and listed <= 16, (listed, dense)
    # the canonical form is that of the permuted layer: nothing else about packing changes
    ref = oracle.pack_canonical(w[order], pid[order], mask[order], lib)
    for a, b in zip(pc.packed_export(q), ref):
        assert a.tobytes() == b.tobytes()
    with pytest.raises(pc.PconvError):
        pc.packed_mfma_blocks(q, 32)
    for h in (p, q):
        h.free()
