"""dlf_run_noalloc (the entry point for callers that cannot allocate: its workspace is a static
device array of the library) against dlf_run with a bound workspace: the same plan, the same
kernels, so the outputs must be bit-identical.  Two calls in a row share the static array, the
second on a smaller input; a plan whose workspace exceeds the array is rejected."""
import numpy as np
import pytest
import torch

from synth import nets, gen

pytestmark = pytest.mark.gpu


def _net_with_split_k_fc(hw):
    """conv - pool - conv - conv(+residual) - FC with a long K: tensors that cross group boundaries
    and (split-K forced below) fp32 partial sums, both of which live in the workspace."""
    layers = [nets.conv(8, 128, 3, 1, 1, "relu"), nets.maxpool(128, 2, 2, 0),
              nets.conv(128, 128, 3, 1, 1, "relu"), nets.conv(128, 128, 3, 1, 1, "relu"),
              nets.conv(128, 128, 1, 1, 0, "relu", residual_from=2),
              nets.fc((hw // 2) * (hw // 2) * 128, 96, "none")]
    return dict(name="noalloc", layers=layers, in_h=hw, in_w=hw, in_c=8, input_dist="normal")


def _both(net, batch, seed):
    from paper_2011_05630_amd import binding as B
    from paper_2011_05630_amd.runner import Session
    x, ws, bs = gen.make_params(net, batch, seed)
    n = len(net["layers"])
    # resident 8x8 tiles, the 128 channels of every layer in 4 slices of 32; FC: K in 4 slices
    B.dlf_debug_force_config(8, 8, 2, 4, 32, 0, 32)
    try:
        s = Session(net, batch, ws, bs, mode=B.TUNER_MANUAL, group_last=list(range(n)),
                    group_budget=[64] * n)
    finally:
        B.dlf_debug_force_config(0, 0, 0, 1, 0, 0, 32)
    try:
        need = B.dlf_plan_workspace_bytes(s.plan)
        assert 0 < need <= B.dlf_static_workspace_bytes()
        xt = torch.from_numpy(x).cuda()
        want = s.run(xt).clone()
        torch.cuda.synchronize()
        got = torch.full(s.out_shape, float("nan"), dtype=torch.float16, device="cuda")
        stream = torch.cuda.current_stream().cuda_stream
        B.dlf_run_noalloc(s.plan, xt.data_ptr(), got.data_ptr(), stream)
        torch.cuda.synchronize()
        return want.cpu().numpy(), got.cpu().numpy(), s
    except Exception:
        s.close()
        raise


def test_noalloc_equals_run_twice_in_a_row_second_call_smaller():
    from oracle import oracle as o
    from gpu_util import compare
    for hw, batch, seed in ((40, 3, 11), (24, 1, 12)):
        net = _net_with_split_k_fc(hw)
        want, got, s = _both(net, batch, seed)
        try:
            assert np.all(np.isfinite(got))
            assert np.array_equal(want, got), "hw %d batch %d" % (hw, batch)
            x, ws, bs = gen.make_params(net, batch, seed)
            compare(got, o.run_net(net, x, ws, bs), "noalloc hw %d batch %d" % (hw, batch))
        finally:
            s.close()


def test_noalloc_rejects_a_plan_beyond_the_static_workspace():
    from paper_2011_05630_amd import binding as B
    from paper_2011_05630_amd.runner import Session
    net = nets.chain4(256)
    x, ws, bs = gen.make_params(net, 8)
    s = Session(net, 8, ws, bs, mode=B.TUNER_MANUAL, group_last=[0, 1, 2, 3], group_budget=[64] * 4)
    try:
        assert B.dlf_plan_workspace_bytes(s.plan) > B.dlf_static_workspace_bytes()
        xt = torch.from_numpy(x).cuda()
        out = torch.empty(s.out_shape, dtype=torch.float16, device="cuda")
        with pytest.raises(B.DlfError) as e:
            B.dlf_run_noalloc(s.plan, xt.data_ptr(), out.data_ptr(), None)
        assert e.value.status == B.DLF_ERR_OOM
    finally:
        s.close()
