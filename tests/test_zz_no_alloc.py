"""The allocation-free entry point against pconv_conv3x3: same kernels, partial sums of the channel split in the
library's fixed device array instead of the handle's workspace.  Two calls in a row on one handle, the second on a
smaller input, each compared bit for bit with pconv_conv3x3 and, to the usual tolerance, with the oracle."""
import numpy as np
import pytest

import oracle
import paper_2001_07710_amd as pc
from workloads import layers as L

from gpu_util import TOL, GpuLayer, rel_err

pytestmark = pytest.mark.gpu


def say(*a):
    print("[case]", *a, flush=True)


def run_entry(entry, layer, x_np, H, W, stride=1):
    import torch
    s = layer.spec
    N = x_np.shape[0]
    Ho, Wo = (H + 2 * s.pad - 3) // stride + 1, (W + 2 * s.pad - 3) // stride + 1
    dx = torch.from_numpy(np.ascontiguousarray(x_np)).cuda()
    n_out, guard = N * s.F * Ho * Wo, 4096
    buf = torch.full((n_out + 2 * guard,), -777.0, dtype=layer.tdtype, device="cuda")
    dy = buf[guard:guard + n_out]
    entry(dx, dy, layer.packed, layer.d_bias, N, H, W, stride, s.pad, pc.FLAG_RELU,
          torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    out = buf.cpu().numpy()
    assert np.all(out[:guard] == -777.0) and np.all(out[guard + n_out:] == -777.0), "write outside the output buffer"
    return out[guard:guard + n_out].reshape(N, s.F, Ho, Wo)


@pytest.mark.parametrize("dtype", ["f32", "f16"])
def test_noalloc_matches_the_allocating_entry_point(dtype):
    pc.ensure_built()
    assert pc.noalloc_scratch_bytes() == 24 * 2 ** 20 + 4 * 16384
    # batch 1 on 256 -> 256 channels: few output tiles, so the library splits the channels and uses the scratch
    spec = L.shrink(L.config1(), dtype=dtype, relu=True)
    layer = GpuLayer(spec)
    x_big = L.gen_activations(spec)
    x_small = np.ascontiguousarray(x_big[:, :, :28, :28])
    for x, H in ((x_big, 56), (x_small, 28)):           # second call: a smaller input on the same handle
        say("noalloc", dtype, "H = W =", H)
        got = run_entry(pc.conv3x3_noalloc, layer, x, H, H)
        ref = oracle.conv3x3(x, layer.wm, layer.bias, 1, spec.pad, True)
        assert rel_err(got, ref) <= TOL[dtype]
        say("allocating entry point", dtype, "H = W =", H)
        want = run_entry(pc.conv3x3, layer, x, H, H)
        assert np.array_equal(got.view(np.uint8), want.view(np.uint8)), "the two entry points differ"
    # stride 2 before any allocating stride-2 call on the handle: the parity form is not there, and is not built
    # (only the vector kernels need that form: where the library takes the matrix-core kernel the call just runs)
    say("noalloc stride 2 without the parity form")
    if pc.conv3x3_choice(layer.packed, x_big.shape[0], 56, 56, 2, spec.pad)[0] == pc.KERNEL_MFMA:
        run_entry(pc.conv3x3_noalloc, layer, x_big, 56, 56, stride=2)
    else:
        with pytest.raises(pc.PconvError) as e:
            run_entry(pc.conv3x3_noalloc, layer, x_big, 56, 56, stride=2)
        assert e.value.code == pc.ESTATE
    say("allocating stride 2, then noalloc stride 2")
    want = run_entry(pc.conv3x3, layer, x_big, 56, 56, stride=2)
    got = run_entry(pc.conv3x3_noalloc, layer, x_big, 56, 56, stride=2)
    assert np.array_equal(got.view(np.uint8), want.view(np.uint8))
    assert rel_err(got, oracle.conv3x3(x_big, layer.wm, layer.bias, 2, spec.pad, True)) <= TOL[dtype]
    layer.free()


def test_noalloc_rejects_a_launch_beyond_the_arena():
    """512 -> 512 channels at 28x28, batch 64, fp32: 800 output tiles of the four-column kernel are 3.1 rounds over the
    compute units, so the library halves the channels of each tile; 1600 workgroups' partial sums are 105 MB, more
    than the arena holds.  The call must say so and launch nothing; the allocating entry point runs the same launch."""
    import torch
    pc.ensure_built()
    spec = L.LayerSpec(cfg=14, idx=0, name="arena", N=64, C=512, F=512, H=28, W=28, K=8, keep=0.2)
    layer = GpuLayer(spec)
    dx = torch.zeros((64, 512, 28, 28), dtype=torch.float32, device="cuda")
    dy = torch.full((64, 512, 28, 28), -777.0, dtype=torch.float32, device="cuda")
    st = torch.cuda.current_stream().cuda_stream
    say("noalloc beyond the arena")
    with pytest.raises(pc.PconvError) as e:
        pc.conv3x3_noalloc(dx, dy, layer.packed, layer.d_bias, 64, 28, 28, 1, 1, 0, st)
    assert e.value.code == pc.ESCRATCH and "scratch" in str(e.value)
    torch.cuda.synchronize()
    assert bool((dy == -777.0).all()), "a rejected call wrote outputs"
    say("the same launch through the allocating entry point")
    pc.conv3x3(dx, dy, layer.packed, layer.d_bias, 64, 28, 28, 1, 1, 0, st)
    torch.cuda.synchronize()
    want = torch.from_numpy(layer.bias).cuda()[None, :, None, None].expand_as(dy)
    assert bool((dy == want).all())          # zero input: the bias alone
    layer.free()
