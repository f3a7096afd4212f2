"""The PyTorch surface (autograd Function + nn.Module) over libsk.

GPU tests compare what autograd returns with the fp64 oracle on the module's own
stored weights; the CPU tests check that nothing computes without a GPU."""
import numpy as np
import pytest
import torch

from oracle import sklinear as O


def split(S_cat, U_cat, l, k):
    """[in, l*k], [l*k, out] -> oracle form S [l, in, k], U [l, k, out] in fp64."""
    S = np.stack([S_cat[:, i * k:(i + 1) * k] for i in range(l)])
    U = np.stack([U_cat[i * k:(i + 1) * k, :] for i in range(l)])
    return S.astype(np.float64), U.astype(np.float64)


def test_no_cpu_path():
    from paper_2601_15473_amd import nn as sknn
    with pytest.raises(RuntimeError, match="GPU only"):
        sknn.SKLinear(64, 64, 1, 16, device="cpu")
    x = torch.zeros(4, 32)
    S = torch.zeros(32, 16)
    U = torch.zeros(16, 48)
    with pytest.raises(RuntimeError, match="GPU only"):
        sknn.sklinear(x, S, U, None, 1, 16)


@pytest.mark.gpu
@pytest.mark.parametrize("dtype,tol", [(torch.bfloat16, 2e-2), (torch.float32, 1e-4)], ids=["bf16", "f32"])
@pytest.mark.parametrize("shape", [(5, 40, 96), (333, 96)], ids=["batched", "flat"])
def test_autograd_matches_oracle(dtype, tol, shape):
    from paper_2601_15473_amd import nn as sknn
    from skgpu import rel_err, to_f64
    l, k, d_out = 3, 16, 80
    print(f"case nn {dtype} x{shape} -> {d_out} l={l} k={k}", flush=True)
    m = sknn.SKLinear(shape[-1], d_out, l, k, bias=True, dtype=dtype, seed=11)
    g = torch.Generator().manual_seed(12)
    x = torch.randn(*shape, generator=g).to(dtype).cuda().requires_grad_(True)
    dY = torch.randn(*shape[:-1], d_out, generator=g).to(dtype).cuda()
    y = m(x)
    assert y.shape == dY.shape and y.dtype == dtype
    y.backward(dY)
    S, U = split(to_f64(m.S_cat), to_f64(m.U_cat), l, k)
    x64 = to_f64(x).reshape(-1, shape[-1])
    dY64 = to_f64(dY).reshape(-1, d_out)
    want = dict(
        y=O.forward(x64, S, U, to_f64(m.bias)),
        dX=O.grad_input(dY64, S, U),
        dU=O.grad_factors(x64, S, dY64).reshape(l * k, d_out),
        db=O.grad_bias(dY64),
    )
    got = dict(y=to_f64(y).reshape(-1, d_out), dX=to_f64(x.grad).reshape(-1, shape[-1]),
               dU=to_f64(m.U_cat.grad), db=to_f64(m.bias.grad))
    assert m.S_cat.requires_grad is False
    for n in want:
        e = rel_err(got[n], want[n])
        print(f"   {n}: {e:.2e}", flush=True)
        assert e <= tol, (n, e)


@pytest.mark.gpu
def test_from_linear_keeps_the_dense_weights():
    """U_i = S_i^T W^T: checked against the product formed in fp64 on the host, and the
    sketched output approaches the dense one as l*k grows (E[S_i S_i^T] = I)."""
    from paper_2601_15473_amd import nn as sknn
    from skgpu import rel_err, to_f64
    torch.manual_seed(3)
    dense = torch.nn.Linear(64, 48).cuda()
    x = torch.randn(200, 64, device="cuda")
    errs = []
    for l, k in ((1, 16), (8, 64)):
        m = sknn.SKLinear.from_linear(dense, l, k, dtype=torch.float32, seed=5)
        want_U = to_f64(m.S_cat).T @ to_f64(dense.weight).T
        assert rel_err(to_f64(m.U_cat), want_U) <= 1e-5
        assert torch.equal(m.bias, dense.bias)
        with torch.no_grad():
            y, ref = m(x), dense(x)
        errs.append(float((y - ref).norm() / ref.norm()))
    print("   relative distance to the dense layer:", errs, flush=True)
    assert errs[1] < 0.5 * errs[0]


@pytest.mark.gpu
def test_no_grad_inputs_skip_their_kernels():
    from paper_2601_15473_amd import nn as sknn
    m = sknn.SKLinear(32, 48, 2, 16, bias=False, dtype=torch.bfloat16, seed=1)
    x = torch.randn(10, 32).bfloat16().cuda()          # no grad wanted for x
    m(x).sum().backward()
    assert m.U_cat.grad is not None and m.U_cat.grad.dtype == torch.bfloat16
    assert x.grad is None and m.bias is None


@pytest.mark.gpu
@pytest.mark.parametrize("dtype,tol", [(torch.bfloat16, 2e-2), (torch.float32, 1e-4)], ids=["bf16", "f32"])
def test_two_sided_module_matches_its_oracle(dtype, tol):
    from oracle import sklinear_two_sided as O2
    from paper_2601_15473_amd import nn as sknn
    from skgpu import rel_err, to_f64
    l, k, d_in, d_out, T = 2, 16, 96, 80, 150
    print(f"case nn two-sided {dtype} T={T} {d_in}->{d_out} l={l}+{l} k={k}", flush=True)
    m = sknn.SKLinearTwoSided(d_in, d_out, l, k, bias=True, dtype=dtype, seed=21)
    g = torch.Generator().manual_seed(22)
    x = torch.randn(T, d_in, generator=g).to(dtype).cuda().requires_grad_(True)
    dY = torch.randn(T, d_out, generator=g).to(dtype).cuda()
    y = m(x)
    y.backward(dY)
    S1c, U1c, U2c, S2Tc = (to_f64(t) for t in (m.S1_cat, m.U1_cat, m.U2_cat, m.S2T_cat))
    S1 = np.stack([S1c[:, i * k:(i + 1) * k] for i in range(l)])             # [l, in, k]
    U2 = np.stack([U2c[:, i * k:(i + 1) * k] for i in range(l)])
    U1 = np.stack([U1c[i * k:(i + 1) * k] for i in range(l)])                # [l, k, out]
    S2 = np.stack([S2Tc[i * k:(i + 1) * k].T for i in range(l)])             # [l, out, k]
    x64, dY64 = to_f64(x), to_f64(dY)
    want = dict(
        y=O2.forward(x64, S1, U1, U2, S2, to_f64(m.bias)),
        dX=O2.grad_input(dY64, S1, U1, U2, S2),
        dU1=O2.grad_second_stage(x64, S1, dY64).reshape(l * k, d_out),
        dU2=np.transpose(O2.grad_first_stage(x64, S2, dY64), (1, 0, 2)).reshape(d_in, l * k),
        db=O2.grad_bias(dY64),
    )
    got = dict(y=to_f64(y), dX=to_f64(x.grad), dU1=to_f64(m.U1_cat.grad), dU2=to_f64(m.U2_cat.grad),
               db=to_f64(m.bias.grad))
    for n in want:
        e = rel_err(got[n], want[n])
        print(f"   {n}: {e:.2e}", flush=True)
        assert e <= tol, (n, e)


@pytest.mark.gpu
def test_two_sided_module_rebuilds_its_stage_matrices_after_an_update():
    """The module keeps [S1 | U2] and [U1 ; S2^T] between calls; an in-place update of a learned
    factor (an optimizer step) must show in the next forward pass, and a second forward pass
    with unchanged factors must reuse the copies."""
    from oracle import sklinear_two_sided as O2
    from paper_2601_15473_amd import nn as sknn
    from skgpu import rel_err, to_f64
    l, k, d_in, d_out, T = 1, 16, 64, 48, 40
    m = sknn.SKLinearTwoSided(d_in, d_out, l, k, bias=True, dtype=torch.float32, seed=5)
    x = torch.randn(T, d_in, generator=torch.Generator().manual_seed(6)).cuda()

    def oracle():
        S1c, U1c, U2c, S2Tc = (to_f64(t) for t in (m.S1_cat, m.U1_cat, m.U2_cat, m.S2T_cat))
        return O2.forward(to_f64(x), S1c[None], U1c[None], U2c[None], S2Tc.T[None], to_f64(m.bias))

    y0 = m(x)
    first = m._stage
    assert rel_err(to_f64(y0), oracle()) <= 1e-4
    m(x)
    assert m._stage is first                       # nothing changed: no new copies
    opt = torch.optim.SGD(m.parameters(), lr=0.5)
    m(x).square().sum().backward()
    opt.step()
    y1 = m(x)
    assert m._stage is not first
    assert rel_err(to_f64(y1), oracle()) <= 1e-4
    assert not torch.allclose(y0, y1)
