"""Helpers for the GPU parity tests: device buffers (torch is used for memory and streams only)
and the mapping between packed memory positions and global parameter indices."""
import numpy as np
import torch

import paper_1906_12043_amd as P
import synth_inputs


def packed_positions(tensor_numel, d):
    """Memory element offset (inside a worker row) of every global parameter index 0..d-1,
    computed independently of the library: tensors in order, each start rounded up to 1024."""
    if not tensor_numel:
        return np.arange(d, dtype=np.int64)
    pos = np.empty(d, dtype=np.int64)
    at = g = 0
    for n in tensor_numel:
        at = (at + 1023) // 1024 * 1024
        pos[g:g + n] = np.arange(at, at + n)
        g += n
        at += n
    return pos


class GpuWorkers:
    """W simulated workers on the GPU behind the C-ABI.  Data arrays are [W][d] in global index order
    and are scattered into the packed layout; results are gathered back the same way."""

    def __init__(self, W, d, *, h=None, c=None, x0=None, tensor_numel=None, bucket_bytes=0, two_streams=True,
                 extra_stride=0, device_fill=False, **hyper):
        self.W, self.d = W, d
        self.dev = torch.device("cuda:0")
        self.padded, _, self.buckets = P.plan_layout(d, tensor_numel, bucket_bytes)
        self.stride = self.padded + extra_stride
        self.pos = None if not tensor_numel else torch.from_numpy(packed_positions(tensor_numel, d)).to(self.dev)
        momentum = hyper.get("momentum", 0.0)
        self.xA = self._upload(x0)
        self.xB = torch.full((W, self.stride), float("nan"), device=self.dev)   # must never be read before written
        self.v = torch.zeros((W, self.stride), device=self.dev) if momentum else None
        self.mean = torch.zeros(self.stride, device=self.dev)
        if device_fill:
            self.h = torch.empty((W, self.stride), device=self.dev)
            self.c = torch.empty((W, self.stride), device=self.dev)
        else:
            self.h, self.c = self._upload(h), self._upload(c)
        # two_streams: True = compute and averaging streams of their own; False = one stream for both;
        # "null" = the null stream for both (no stream objects at all)
        self.s_compute = None if two_streams == "null" else torch.cuda.Stream(device=self.dev)
        self.s_avg = torch.cuda.Stream(device=self.dev) if two_streams is True else self.s_compute
        torch.cuda.synchronize()
        self.ctx = P.Context(W=W, d=d, stride=self.stride, xA=self.xA, xB=self.xB, v=self.v, mean=self.mean,
                             h=self.h, c=self.c, tensor_numel=tensor_numel, bucket_bytes=bucket_bytes,
                             compute_stream=self.s_compute, avg_stream=self.s_avg, **hyper)
        if device_fill:
            self.ctx.fill_quadratic()
            self.ctx.sync()

    def _upload(self, arr):
        buf = torch.zeros((self.W, self.stride), device=self.dev)
        if arr is not None:
            src = torch.from_numpy(np.array(np.broadcast_to(arr, (self.W, self.d)), dtype=np.float32)).to(self.dev)
            if self.pos is None:
                buf[:, :self.d] = src
            else:
                buf[:, self.pos] = src
        return buf

    def _gather(self, buf, cols=None):
        """[..., d] (or the given global columns) of a packed device buffer, as float64 numpy."""
        if cols is None:
            out = buf[..., :self.d] if self.pos is None else buf[..., self.pos]
        else:
            cols_t = torch.from_numpy(np.asarray(cols, dtype=np.int64)).to(self.dev)
            out = buf[..., cols_t] if self.pos is None else buf[..., self.pos[cols_t]]
        return out.cpu().numpy().astype(np.float64)

    def live(self):
        ptr = self.ctx.live_model()
        return self.xA if ptr == self.xA.data_ptr() else self.xB

    def x(self, cols=None):
        self.ctx.sync()
        return self._gather(self.live(), cols)

    def x_raw(self):
        self.ctx.sync()
        return self.live().clone()

    def vel(self, cols=None):
        self.ctx.sync()
        return self._gather(self.v, cols)

    def avg(self, cols=None):
        self.ctx.sync()
        return self._gather(self.mean, cols)

    def data(self, cols=None):
        self.ctx.sync()
        return self._gather(self.h, cols).astype(np.float32), self._gather(self.c, cols).astype(np.float32)

    def close(self):
        self.ctx.close()


def rel_err(got, want):
    """max |got - want| / (1 + |want|): the parity measure of the target."""
    return float(np.max(np.abs(got - want) / (1.0 + np.abs(want))))


class GpuMlp:
    def __init__(self, W, shape, batch, theta0, **hyper):
        n_in, n_hidden, n_out = shape
        self.W, self.shape, self.batch = W, shape, batch
        self.d = synth_inputs.mlp_param_count(*shape)
        self.dev = torch.device("cuda:0")
        self.stride, _, _ = P.plan_layout(self.d)
        self.xA = torch.zeros((W, self.stride), device=self.dev)
        self.xA[:, :self.d] = torch.from_numpy(np.asarray(theta0, dtype=np.float32)).to(self.dev)
        self.xB = torch.full((W, self.stride), float("nan"), device=self.dev)
        self.v = torch.zeros((W, self.stride), device=self.dev)
        self.mean = torch.zeros(self.stride, device=self.dev)
        self.s_compute, self.s_avg = torch.cuda.Stream(device=self.dev), torch.cuda.Stream(device=self.dev)
        torch.cuda.synchronize()
        self.ctx = P.Context(W=W, d=self.d, stride=self.stride, xA=self.xA, xB=self.xB, v=self.v, mean=self.mean,
                             grad=P.GRAD_MLP, mlp=(n_in, n_hidden, n_out, batch),
                             compute_stream=self.s_compute, avg_stream=self.s_avg, **hyper)

    def x(self):
        self.ctx.sync()
        live = self.xA if self.ctx.live_model() == self.xA.data_ptr() else self.xB
        return live[:, :self.d].cpu().numpy().astype(np.float64)

    def vel(self):
        self.ctx.sync()
        return self.v[:, :self.d].cpu().numpy().astype(np.float64)

    def workspace(self):
        """Copies of X, H, dA, dZ, y as numpy arrays (through the library's own copy kernel)."""
        self.ctx.sync()
        ptrs, pitch = self.ctx.mlp_workspace()
        n_in, n_hidden, n_out = self.shape
        sizes = dict(X=self.batch * n_in, H=self.batch * n_hidden, dA=self.batch * n_hidden, dZ=self.batch * pitch, y=self.batch)
        out = {}
        for name, per_worker in sizes.items():
            buf = torch.empty(self.W * per_worker, device=self.dev)
            P.debug_copy(None, ptrs[name], buf, buf.numel())
            torch.cuda.synchronize()
            out[name] = buf.view(torch.int32).cpu().numpy() if name == "y" else buf.cpu().numpy().astype(np.float64)
        out["X"] = out["X"].reshape(self.W, self.batch, n_in)
        out["H"] = out["H"].reshape(self.W, self.batch, n_hidden)
        out["dA"] = out["dA"].reshape(self.W, self.batch, n_hidden)
        out["dZ"] = out["dZ"].reshape(self.W, self.batch, pitch)[:, :, :n_out]
        out["y"] = out["y"].reshape(self.W, self.batch)
        return out

    def close(self):
        self.ctx.close()
