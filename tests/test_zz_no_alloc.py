"""cadnn_run_net_noalloc (the entry point for callers that cannot allocate) against
cadnn_run_net on the same nets: a bottleneck block with a 3x3 layer (so the static workspace
holds zero halos that must be cleared again) and a sparse FC behind a pool; two calls in a row on
the shared static workspace, the second with a smaller input, then the first again."""
import numpy as np
import pytest

import oracle
import workloads as wl
from util import TOL_F32, TOL_F16, assert_chain_close, cond_fc

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


def block_ops():
    Op = wl.Op
    return [Op("conv", "a", 0, 1, 64, 32, 1, 1, 0, 0.85, True),
            Op("conv", "b", 1, 2, 32, 32, 3, 1, 1, 0.85, True),
            Op("conv", "c", 2, 3, 32, 64, 1, 1, 0, 0.85, True, res=0),
            Op("conv", "d", 3, 4, 64, 48, 3, 2, 1, 0.8, True),
            Op("avgpool", "gap", 4, 5),
            Op("fc", "fc", 5, 6, 48, 10, sparsity=0.5, relu=False)]


@pytest.mark.parametrize("dtype_name", ["f32", "f16"])
def test_no_alloc_entry_point_matches_run_net(dtype_name):
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_1905_00571_amd as cad
    cad.lib()
    f16 = dtype_name == "f16"
    dtype, npdt, tol = (cad.F16, np.float16, TOL_F16) if f16 else (cad.F32, np.float32, TOL_F32)
    ops = block_ops()
    big, small = (2, 64, 28, 28), (1, 64, 12, 10)
    nets, refs, xs, want = {}, {}, {}, {}
    for name, shape in (("big", big), ("small", small)):
        x, ws, bs = wl.net_tensors(ops, "noalloc", shape, input_relu=True)
        x = x.astype(npdt)
        ref, ins, _ = oracle.run_net(ops, x, ws, bs, dtype=npdt)
        plain = cad.build_net(ops, ws, bs, shape, dtype, use_graph=False)
        static = cad.build_net(ops, ws, bs, shape, dtype, use_graph=False, static_workspace=True)
        xd = torch.from_numpy(x).cuda()
        y = plain.run(xd)
        torch.cuda.synchronize()
        assert_chain_close(y.cpu().numpy(), ref, cond_fc(ins[-1], ws[-1].astype(npdt), bs[-1]), tol, f"run_net {name}")
        nets[name], xs[name], want[name] = static, xd, y.clone()
        plain.free()
    # a plain net must be refused, and so must a net that needs more than the static array holds
    with pytest.raises(cad.CadnnError):
        x, ws, bs = wl.net_tensors(ops, "noalloc", small, input_relu=True)
        other = cad.build_net(ops, ws, bs, small, dtype, use_graph=False)
        try:
            other.run_noalloc(xs["small"], torch.empty_like(want["small"]))
        finally:
            other.free()
    with pytest.raises(cad.CadnnError):
        huge = (8, 64, 160, 160)
        x, ws, bs = wl.net_tensors(ops, "noalloc", (1, 64, 8, 8), input_relu=True)
        cad.build_net(ops, ws, bs, huge, dtype, use_graph=False, static_workspace=True)
    outs = {k: torch.full_like(v, float("nan")) for k, v in want.items()}
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()      # (the binding itself must not allocate tensors either)
    for name in ("big", "small", "big", "small"):
        outs[name].fill_(float("nan"))
        nets[name].run_noalloc(xs[name], outs[name])
        torch.cuda.synchronize()
        # same kernels, same order of sums: the same bits as the existing entry point
        assert torch.equal(outs[name], want[name]), (name, (outs[name].float() - want[name].float()).abs().max().item())
    assert torch.cuda.memory_allocated() == before
    for n_ in nets.values():
        n_.free()
