"""Convenience wrapper used by tests and the benchmark: owns the library handles and the torch
buffers (device memory and stream only; every layer runs inside libdlf's kernels)."""
import numpy as np
import torch

from . import binding as B


class Session:
    def __init__(self, net, batch, weights, biases, device="cuda:0", **plan_kwargs):
        if not torch.cuda.is_available():
            raise RuntimeError("libdlf needs a GPU: no CPU fallback exists")
        self.net_desc = net
        self.batch = batch
        self.device = torch.device(device)
        torch.cuda.set_device(self.device)
        self.net = B.dlf_net_create(net["layers"], net["in_h"], net["in_w"], net["in_c"], weights,
                                    biases)
        self.plan = None
        self.ws = None
        self.replan(**plan_kwargs)
        n = len(net["layers"])
        h, w, c, _ = B.dlf_net_layer_info(self.net, n - 1)
        self.out_shape = (batch, h, w, c)
        self.in_shape = (batch, net["in_h"], net["in_w"], net["in_c"])

    def replan(self, **plan_kwargs):
        if self.plan is not None:
            B.dlf_plan_destroy(self.plan)
            self.plan = None
        self.plan = B.dlf_plan(self.net, self.batch, **plan_kwargs)
        nbytes = B.dlf_plan_workspace_bytes(self.plan)
        self.ws = torch.empty(max(nbytes, 256), dtype=torch.uint8, device=self.device)
        B.dlf_plan_bind_workspace(self.plan, self.ws.data_ptr(), self.ws.numel())
        self.groups = B.dlf_plan_groups(self.plan)

    def refine(self, x, top_k=6, reps=5):
        """Measured refinement of the plan on the input tensor x; -> number of groups changed."""
        assert x.is_cuda and x.dtype == torch.float16 and x.is_contiguous()
        assert tuple(x.shape) == self.in_shape, (x.shape, self.in_shape)
        out = torch.empty(self.out_shape, dtype=torch.float16, device=self.device)
        stream = torch.cuda.current_stream(self.device).cuda_stream
        n = B.dlf_plan_refine(self.plan, x.data_ptr(), out.data_ptr(), stream, top_k, reps)
        self.groups = B.dlf_plan_groups(self.plan)
        return n

    def layer_shape(self, i):
        if i < 0:
            return self.in_shape
        h, w, c, _ = B.dlf_net_layer_info(self.net, i)
        return (self.batch, h, w, c)

    def run(self, x, out=None):
        """x: fp16 cuda tensor [batch,H,W,C] (contiguous). Returns the output tensor (async)."""
        assert x.is_cuda and x.dtype == torch.float16 and x.is_contiguous()
        assert tuple(x.shape) == self.in_shape, (x.shape, self.in_shape)
        if out is None:
            out = torch.empty(self.out_shape, dtype=torch.float16, device=self.device)
        stream = torch.cuda.current_stream(self.device).cuda_stream
        B.dlf_run(self.plan, x.data_ptr(), out.data_ptr(), stream)
        return out

    def run_group(self, g, x, res=None, out=None):
        info = self.groups[g]
        if out is None:
            out = torch.empty(self.layer_shape(info["last"]), dtype=torch.float16,
                              device=self.device)
        stream = torch.cuda.current_stream(self.device).cuda_stream
        B.dlf_run_group(self.plan, g, x.data_ptr(), res.data_ptr() if res is not None else None,
                        out.data_ptr(), stream)
        return out

    def layer_output(self, i):
        """Materialised output of layer i (a view into the workspace), or None."""
        ptr = B.dlf_plan_layer_output(self.plan, i)
        if not ptr:
            return None
        shape = self.layer_shape(i)
        off = ptr - self.ws.data_ptr()
        n = int(np.prod(shape))
        return self.ws[off:off + 2 * n].view(torch.float16).view(shape)

    def run_numpy(self, x_np):
        x = torch.from_numpy(np.ascontiguousarray(x_np, dtype=np.float16)).to(self.device)
        y = self.run(x)
        torch.cuda.synchronize(self.device)
        return y.cpu().numpy()

    def close(self):
        if self.plan is not None:
            B.dlf_plan_destroy(self.plan)
            self.plan = None
        if self.net is not None:
            B.dlf_net_destroy(self.net)
            self.net = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
