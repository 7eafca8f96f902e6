"""GPU parity of the selection-variable steps (include/pconv_admm.h) with oracle/admm_oracle.py and of the device
pattern assignment with oracle.assign_patterns, through the C ABI, on seeded inputs.  The kernels compute in double
exactly what the oracle computes in double, in the same order, and round once to float: the comparison is exact."""
import numpy as np
import pytest

import oracle
from workloads import rng

pytestmark = pytest.mark.gpu


def gen(seed, n, K, scale):
    return (rng.normal(rng.stream_seed(91, seed, K), n * K).reshape(n, K) * scale).astype(np.float32)


@pytest.mark.parametrize("K", [1, 2, 3, 4, 6, 8, 12, 16, 17, 32])
@pytest.mark.parametrize("n", [1, 255, 1000, 66000])          # one thread, a ragged block, several blocks and a tail
def test_proximal_step_matches_the_oracle(K, n):
    import torch
    import paper_2001_07710_amd as pc
    z, mu, rho = gen(1, n, K, 0.6), gen(2, n, K, 0.2), 0.75
    if n == 1000:
        z[::7] = 1.0 / K                                      # ties between all entries
        z[3::11, 0] = 50.0                                    # a vertex
    u_ref, mu_ref = oracle.proximal_step(z, mu, rho)
    dz, dmu = torch.from_numpy(z).cuda(), torch.from_numpy(mu).cuda()
    du, dm2 = torch.full_like(dz, -7.0), torch.full_like(dz, -7.0)
    pc.admm_proximal(dz, dmu, rho, n, K, du, dm2, torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(du.cpu().numpy(), u_ref.astype(np.float32))
    np.testing.assert_array_equal(dm2.cpu().numpy(), mu_ref.astype(np.float32))
    # properties that hold at any size: on the simplex to float rounding
    s = du.double().sum(dim=1)
    assert float((s - 1.0).abs().max()) < 1e-5 and float(du.min()) >= 0.0


def test_plain_projection_in_place_multipliers_and_unaligned_buffers():
    import torch
    import paper_2001_07710_amd as pc
    n, K = 5000, 8
    z, mu = gen(3, n, K, 1.0), gen(4, n, K, 0.3)
    st = torch.cuda.current_stream().cuda_stream
    dz = torch.from_numpy(z).cuda()
    du = torch.empty_like(dz)
    pc.admm_proximal(dz, None, 1.0, n, K, du, None, st)                       # mu = NULL: projection of z
    torch.cuda.synchronize()
    np.testing.assert_array_equal(du.cpu().numpy(), oracle.simplex_project(z).astype(np.float32))
    dmu = torch.from_numpy(mu).cuda()
    pc.admm_proximal(dz, dmu, 2.0, n, K, None, dmu, st)                       # multipliers updated in place, no u
    torch.cuda.synchronize()
    np.testing.assert_array_equal(dmu.cpu().numpy(), oracle.proximal_step(z, mu, 2.0)[1].astype(np.float32))
    # buffers that start 4 bytes into an allocation (no 128-bit accesses possible)
    big = torch.zeros(n * K + 1, dtype=torch.float32, device="cuda")
    big[1:] = torch.from_numpy(z.reshape(-1)).cuda()
    out = torch.zeros(n * K + 1, dtype=torch.float32, device="cuda")
    pc.admm_proximal(big[1:], None, 1.0, n, K, out[1:], None, st)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(out[1:].cpu().numpy().reshape(n, K), oracle.simplex_project(z).astype(np.float32))
    assert float(out[0]) == 0.0


@pytest.mark.parametrize("K", [1, 5, 8, 126])
def test_binarize_matches_the_oracle(K):
    import torch
    import paper_2001_07710_amd as pc
    n = 33333
    z = gen(5, n, K, 1.0)
    z[::5] = np.round(z[::5] * 2) / 2                          # many exact ties
    dz = torch.from_numpy(z).cuda()
    pid = torch.full((n,), -1, dtype=torch.int32, device="cuda")
    pc.admm_binarize(dz, n, K, pid, torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(pid.cpu().numpy(), oracle.binarize(z))


@pytest.mark.parametrize("dtype", ["f32", "f16"])
@pytest.mark.parametrize("K", [4, 8, 12, 56])
def test_device_pattern_assignment_matches_the_oracle_bit_for_bit(dtype, K):
    import torch
    import paper_2001_07710_amd as pc
    from workloads import layers as L
    F, C = 96, 131                                            # 12576 kernels: several blocks and a ragged tail
    w = rng.normal(rng.stream_seed(92, K), F * C * 9).reshape(F, C, 3, 3)
    w = w.astype(np.float16 if dtype == "f16" else np.float32)
    w[0, :8] = 0                                              # all patterns tie: lowest id
    w[1, :8] = 1.0                                            # equal weights: ties again
    lib = np.array(L.centre_masks()[:K], dtype=np.uint16)
    ref = oracle.assign_patterns(w, lib)
    dw = torch.from_numpy(w).cuda()
    pid = torch.full((F * C,), -1, dtype=torch.int32, device="cuda")
    pc.assign_patterns_device(dw, pc.F16 if dtype == "f16" else pc.F32, F * C, lib, pid,
                              torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    got = pid.cpu().numpy().reshape(F, C)
    np.testing.assert_array_equal(got, ref)
    np.testing.assert_array_equal(got, pc.assign_patterns(w.astype(np.float32), lib))      # and the host entry


@pytest.mark.parametrize("dtype", ["f32", "f16"])
@pytest.mark.parametrize("keep", [0.0, 0.15, 0.28, 0.5, 1.0])
def test_device_connectivity_selection_matches_the_oracle_bit_for_bit(dtype, keep):
    import torch
    import paper_2001_07710_amd as pc
    from workloads import layers as L
    F, C, K = 77, 163, 8                                       # 12551 kernels
    w = rng.normal(rng.stream_seed(94, K), F * C * 9).reshape(F, C, 3, 3)
    w = w.astype(np.float16 if dtype == "f16" else np.float32)
    w[5:9] = w[1:5]                                           # whole filters repeated: many equal norms, ties by index
    w[20, :40] = 0
    lib = np.array(L.drawn_library(4, K), dtype=np.uint16)
    pid = oracle.assign_patterns(w, lib)
    ref = oracle.select_connectivity(w, lib, pid, keep)
    n = F * C
    st = torch.cuda.current_stream().cuda_stream
    need = pc.select_connectivity_device_workspace(n)
    ws = torch.empty(need, dtype=torch.uint8, device="cuda")
    dw = torch.from_numpy(w).cuda()
    dpid = torch.from_numpy(pid.astype(np.int32).reshape(-1)).cuda()
    mask = torch.full((n,), 7, dtype=torch.uint8, device="cuda")
    code = pc.F16 if dtype == "f16" else pc.F32
    pc.select_connectivity_device(dw, code, n, lib, dpid, keep, mask, ws, need, st)
    torch.cuda.synchronize()
    got = mask.cpu().numpy().reshape(F, C)
    np.testing.assert_array_equal(got, np.asarray(ref, dtype=np.uint8))
    assert int(got.sum()) == int(np.floor(keep * n + 0.5))
    np.testing.assert_array_equal(got, pc.select_connectivity(w.astype(np.float32), lib, pid, keep))   # the host entry
    # a workspace that is too small is refused, nothing is written
    mask.fill_(7)
    with pytest.raises(pc.PconvError) as e:
        pc.select_connectivity_device(dw, code, n, lib, dpid, keep, mask, ws, need - 256, st)
    assert e.value.code == pc.ESCRATCH
    torch.cuda.synchronize()
    assert int(mask.min()) == 7


def test_assign_then_select_on_the_device_feed_pack_like_the_host_steps():
    """The two device steps chained, their outputs handed to pconv_pack: the packed layer is the one the host steps
    give (canonical form compared bit for bit)."""
    import torch
    import paper_2001_07710_amd as pc
    from workloads import layers as L
    spec = L.shrink(L.config1(), C=48, F=40)
    w = L.gen_weights(spec).astype(np.float32)
    lib = spec.library()
    n = spec.F * spec.C
    st = torch.cuda.current_stream().cuda_stream
    dw = torch.from_numpy(w).cuda()
    dpid = torch.empty(n, dtype=torch.int32, device="cuda")
    pc.assign_patterns_device(dw, pc.F32, n, lib, dpid, st)
    need = pc.select_connectivity_device_workspace(n)
    ws = torch.empty(need, dtype=torch.uint8, device="cuda")
    dmask = torch.empty(n, dtype=torch.uint8, device="cuda")
    pc.select_connectivity_device(dw, pc.F32, n, lib, dpid, spec.keep, dmask, ws, need, st)
    torch.cuda.synchronize()
    pid_d = dpid.cpu().numpy().reshape(spec.F, spec.C).astype(np.uint8)
    mask_d = dmask.cpu().numpy().reshape(spec.F, spec.C)
    pid_h = pc.assign_patterns(w, lib)
    mask_h = pc.select_connectivity(w, lib, pid_h, spec.keep)
    np.testing.assert_array_equal(pid_d, pid_h)
    np.testing.assert_array_equal(mask_d, mask_h)
    a = pc.packed_export(pc.pack(w, lib, pid_d, mask_d, flags=1))
    b = pc.packed_export(pc.pack(w, lib, pid_h, mask_h, flags=1))
    for x, y in zip(a, b):
        np.testing.assert_array_equal(np.asarray(x), np.asarray(y))
