"""mlp_train_step_static, the training step for callers that cannot allocate: the same step on the library's own
static workspace.  Two identical MLPs are trained side by side, one through mlp_train_step with a workspace
tensor, one through mlp_train_step_static, on two calls in a row, the second with a smaller batch: weights, biases,
both momentum buffers and the loss must agree (the kernels are the same, so bit for bit, which is inside the
1e-5 * S bar of the parity tests; the first step is also checked against the oracle at that bar)."""
import numpy as np
import pytest

from paper_2407_17437_amd import workloads as wl

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def nb():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2407_17437_amd import binding
    return binding


def _state(M):
    out = []
    for l in M.layers:
        out += [l.values.cpu().numpy().copy(), l.bias.cpu().numpy().copy(),
                l.velocity.cpu().numpy().copy(), l.bias_velocity.cpu().numpy().copy()]
    return out


@pytest.mark.parametrize("sizes,kw,batches", [
    ((3072, 1024, 512, 10), dict(sparsity=0.99), (100, 37)),              # the paper's MLP: fused head, paired launches
    ((100, 300, 10), dict(layer_nnz=(6000, 3000), bias_std=0.1), (64, 24)),   # saturated output layer: streaming kernels
    ((6000, 300, 10), dict(sparsity=0.98, bias_std=0.1), (200, 100)),     # column-tiled SDDMM (partial buffer of the layer)
])
def test_static_step_matches_the_step_with_a_workspace(nb, oracle, sizes, kw, batches):
    import torch
    from test_gpu_parity import close, TOL
    lr, mu = 0.05, 0.9
    mlp = wl.make_mlp(sizes, pattern_seed=120, value_seed=220, **kw)
    A = nb.MLP(mlp, max(batches)); B = nb.MLP(mlp, max(batches))
    assert nb.mlp_workspace_bytes(B.handle, max(batches)) <= nb.NERVA_STATIC_WORKSPACE_BYTES
    ref_state = oracle.new_state(mlp.layers, np.float32)
    loss_b = torch.zeros(1, device="cuda")
    for t, batch in enumerate(batches):
        Xs, Ts = wl.make_batches(sizes[0], sizes[-1], batch, 1, seed=320 + t)
        Xd = nb.to_dense(Xs[0]); lab = torch.as_tensor(Ts[0]).cuda()
        A.train_step(Xd, lab, batch, lr, mu)
        nb.mlp_train_step_static(B.handle, Xd, Xd.stride(0), lab, batch, lr, mu, loss_b)
        torch.cuda.synchronize()
        for k, (a, b) in enumerate(zip(_state(A), _state(B))):
            assert np.array_equal(a, b), f"call {t}: array {k} differs between the two entry points"
        assert float(A.loss.item()) == float(loss_b.item())
        if t == 0:
            masks = [A.view("A", l, batch).cpu().numpy() > 0 for l in range(len(sizes) - 2)] + [None]
            ref = oracle.mlp_step(ref_state, Xs[0], Ts[0], lr, mu, np.float32, relu_masks=masks)
            for l, lay in enumerate(B.layers):
                close(lay.values.cpu().numpy(), ref_state[l]["values"], ref["Sw"][l], what=f"values[{l}] (static step)")
                close(lay.velocity.cpu().numpy(), ref_state[l]["vel_w"], ref["Sv"][l], what=f"velocity[{l}] (static step)")
                close(lay.bias.cpu().numpy(), ref_state[l]["bias"], ref["Sbw"][l], what=f"bias[{l}] (static step)")
            assert abs(float(loss_b.item()) - ref["loss"]) <= TOL * ref["S_loss"]
    A.close(); B.close()


def test_static_step_rejects_what_does_not_fit(nb):
    import torch
    mlp = wl.make_mlp((3072, 8192, 10), sparsity=0.995, pattern_seed=121, value_seed=221)
    M = nb.MLP(mlp, 1024)
    need = nb.mlp_workspace_bytes(M.handle, 1024)
    assert need > nb.NERVA_STATIC_WORKSPACE_BYTES
    Xs, Ts = wl.make_batches(3072, 10, 1024, 1, seed=321)
    Xd = nb.to_dense(Xs[0]); lab = torch.as_tensor(Ts[0]).cuda()
    before = M.layers[0].values.clone()
    with pytest.raises(nb.NervaError) as e:
        nb.mlp_train_step_static(M.handle, Xd, Xd.stride(0), lab, 1024, 0.01, 0.9, M.loss)
    assert e.value.code == nb.NERVA_ERR_WORKSPACE and str(need) in str(e.value) and str(nb.NERVA_STATIC_WORKSPACE_BYTES) in str(e.value)
    torch.cuda.synchronize()
    assert torch.equal(before, M.layers[0].values)          # nothing was enqueued
    # a batch small enough for the static workspace goes through on the same MLP
    nb.mlp_train_step_static(M.handle, Xd, Xd.stride(0), lab, 256, 0.01, 0.9, M.loss)
    torch.cuda.synchronize()
    assert np.isfinite(float(M.loss.item())) and not torch.equal(before, M.layers[0].values)
    M.close()
