"""A layer read back with pconv_packed_import from the oracle's canonical arrays runs like the layer packed from the
dense weights: outputs against the oracle, and bit-equal between the two handles, for both storage types and strides."""
import numpy as np
import pytest

import oracle
import paper_2001_07710_amd as pc
from workloads import layers as L

from gpu_util import TOL, rel_err

pytestmark = pytest.mark.gpu

CASES = [  # N, C, F, H, W, stride, pad, dtype
    (1, 48, 40, 17, 23, 1, 1, "f32"),
    (3, 64, 96, 14, 28, 1, 1, "f16"),
    (2, 32, 64, 21, 18, 2, 1, "f16"),
    (1, 20, 24, 15, 15, 2, 0, "f32"),
]


def run(torch, packed, x, bias, spec):
    dx, db = torch.from_numpy(x).cuda(), torch.from_numpy(bias).cuda()
    dy = torch.empty((spec.N, spec.F, spec.Ho, spec.Wo), dtype=dx.dtype, device="cuda")
    pc.conv3x3(dx, dy, packed, db, spec.N, spec.H, spec.W, spec.stride, spec.pad, pc.FLAG_RELU,
               torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    return dy.cpu().numpy()


@pytest.mark.parametrize("case", CASES, ids=[f"n{c[0]}c{c[1]}f{c[2]}h{c[3]}w{c[4]}s{c[5]}p{c[6]}{c[7]}" for c in CASES])
def test_imported_layer_runs_like_the_packed_one(case):
    import torch
    N, C, F, H, W, stride, pad, dtype = case
    print("[case]", case, flush=True)
    spec = L.LayerSpec(cfg=43, idx=CASES.index(case), name="imported", N=N, C=C, F=F, H=H, W=W, stride=stride, pad=pad,
                       dtype=dtype, K=8, keep=0.35)
    w, x, bias, lib = L.gen_weights(spec), L.gen_activations(spec), L.gen_bias(spec), spec.library()
    pid = oracle.assign_patterns(w.astype(np.float32), lib)
    mask = oracle.select_connectivity(w.astype(np.float32), lib, pid, spec.keep)
    canon = oracle.pack_canonical(w, pid, mask, lib)
    imported = pc.packed_import(*canon, F, C, lib)
    packed = pc.pack(w, lib, pid, mask)
    a, b = run(torch, imported, x, bias, spec), run(torch, packed, x, bias, spec)
    assert a.tobytes() == b.tobytes()
    ref = oracle.conv3x3(x, oracle.mask_weights(w, pid, mask, lib), bias, stride, pad, True)
    assert rel_err(a, ref) <= TOL[dtype]
    imported.free()
    packed.free()
