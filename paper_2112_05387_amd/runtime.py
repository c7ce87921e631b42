"""Device-buffer holder for one local step.  PyTorch provides device memory and the stream; every
computation happens in the HIP library behind `binding`."""
import numpy as np
import torch

from . import binding as B


def _dev():
    if not torch.cuda.is_available():
        raise RuntimeError("no GPU visible: the local step runs on an MI355X only (there is no CPU fallback)")
    return torch.device("cuda:0")


class LocalStep:
    """Owns the net handle, workspace, packed parameters and interface tensors of one configuration.

    `desc` is any object with the attributes of the C descriptors (modules, aux, dtype, bn_eps, K)."""

    def __init__(self, desc, keep_gradients=False):
        """keep_gradients: debug layout of the workspace in which no gradient buffer is reused inside a backward pass
        (for the unit-by-unit views of `units` / `fetch`)."""
        self.desc = desc
        self.K = len(desc.modules)
        self.dtype = desc.dtype
        self.tdtype = torch.bfloat16 if desc.dtype == "bf16" else torch.float32
        B.lp_debug_keep_gradients(keep_gradients)
        try:
            self.net = B.lp_net_create(desc.modules, desc.aux, desc.dtype, desc.bn_eps)
        finally:
            B.lp_debug_keep_gradients(False)
        self.dev = _dev()
        self.ws_bytes = B.lp_net_workspace_bytes(self.net)
        self.ws = torch.empty(self.ws_bytes + 256, dtype=torch.uint8, device=self.dev)
        B.lp_net_set_workspace(self.net, self.ws.data_ptr(), self.ws_bytes)
        self.tables = [[B.lp_net_tensor_info(self.net, 0, k, i) for i in range(B.lp_net_num_tensors(self.net, 0, k))]
                       for k in range(self.K)]
        self.aux_tables = []
        if desc.aux is not None:
            self.aux_tables = [[B.lp_net_tensor_info(self.net, 1, j, i) for i in range(B.lp_net_num_tensors(self.net, 1, j))]
                               for j in range(self.K - 1)]
        m = desc.modules
        self.x_shapes = [(mm.N, mm.H, mm.W, mm.C) for mm in m]
        self.y_shapes = [self.x_shapes[k + 1] for k in range(self.K - 1)]
        self.n_classes = m[-1].n_classes
        self.N = m[-1].N
        # device state
        self.params = [None] * self.K
        self.dparams = [None] * self.K
        for k in range(self.K):
            pb, gb = B.lp_net_param_bytes(self.net, 0, k)
            self.params[k] = torch.zeros(pb, dtype=torch.uint8, device=self.dev)
            self.dparams[k] = torch.zeros(gb // 4, dtype=torch.float32, device=self.dev)
        self.aux_params, self.daux_params = [], []
        for j in range(len(self.aux_tables)):
            pb, gb = B.lp_net_param_bytes(self.net, 1, j)
            self.aux_params.append(torch.zeros(pb, dtype=torch.uint8, device=self.dev))
            self.daux_params.append(torch.zeros(gb // 4, dtype=torch.float32, device=self.dev))
        self.aux_loss = torch.zeros((max(self.K - 1, 1),), dtype=torch.float32, device=self.dev)
        self.x = [torch.zeros(s, dtype=self.tdtype, device=self.dev) for s in self.x_shapes]
        self.y = [torch.zeros(s, dtype=self.tdtype, device=self.dev) for s in self.y_shapes]
        self.dy = [torch.zeros(s, dtype=self.tdtype, device=self.dev) for s in self.y_shapes]
        self.dx = [torch.zeros(s, dtype=self.tdtype, device=self.dev) for s in self.x_shapes]
        self.lam = None
        self.logits = torch.zeros((self.N, self.n_classes), dtype=torch.float32, device=self.dev)
        self.dlogits = torch.zeros_like(self.logits)
        self.labels = torch.zeros((self.N,), dtype=torch.int32, device=self.dev)
        self.loss = torch.zeros((self.K,), dtype=torch.float32, device=self.dev)
        self.r2 = torch.zeros((max(self.K - 1, 1),), dtype=torch.float32, device=self.dev)    # |F_k(x_k) - x_{k+1}|^2
        B.lp_net_set_residual_output(self.net, self.r2.data_ptr())

    def set_stream_lanes(self, lanes):
        """lanes[k] in 0..3 (0 = the caller's stream) or None for a single stream."""
        if lanes is not None:
            assert len(lanes) == self.K
        B.lp_net_set_stream_lanes(self.net, lanes)

    def close(self):
        if self.net is not None:
            torch.cuda.synchronize()
            B.lp_net_destroy(self.net)
            self.net = None

    # ---- host <-> device marshalling ---------------------------------------------------------------
    def to_dev(self, a, low=True):
        t = torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32))
        if low and self.dtype == "bf16":
            t = t.to(torch.bfloat16)
        return t.to(self.dev)

    @staticmethod
    def to_host(t):
        return t.detach().float().cpu().numpy().astype(np.float64)

    def _pack(self, buf, table, tensors):
        assert len(table) == len(tensors)
        for info, a in zip(table, tensors):
            assert int(info.numel) == int(np.size(a)), "parameter tensor size mismatch"
            n = int(info.numel)
            if info.dtype == B.LP_BF16:
                src = torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32).reshape(-1)).to(torch.bfloat16)
                buf[info.offset:info.offset + 2 * n].view(torch.bfloat16).copy_(src)
            else:
                src = torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32).reshape(-1))
                buf[info.offset:info.offset + 4 * n].view(torch.float32).copy_(src)

    def set_params(self, k, tensors):
        self._pack(self.params[k], self.tables[k], tensors)

    def set_aux_params(self, j, tensors):
        self._pack(self.aux_params[j], self.aux_tables[j], tensors)

    def get_aux_grads(self, j):
        out = []
        for info in self.aux_tables[j]:
            o = info.grad_offset // 4
            shape = tuple(info.dims[i] for i in range(info.ndim))
            out.append(self.to_host(self.daux_params[j][o:o + int(info.numel)]).reshape(shape))
        return out

    def get_grads(self, k):
        out = []
        for info in self.tables[k]:
            o = info.grad_offset // 4
            shape = tuple(info.dims[i] for i in range(info.ndim))
            out.append(self.to_host(self.dparams[k][o:o + int(info.numel)]).reshape(shape))
        return out

    def set_x(self, k, a):
        self.x[k].copy_(self.to_dev(a))

    def set_lams(self, lams):
        self.lam = None if lams is None else [self.to_dev(l) for l in lams]

    def set_labels(self, labels):
        self.labels.copy_(torch.from_numpy(np.ascontiguousarray(labels, dtype=np.int32)))

    def saved(self, k, which, shape):
        """Copy of a saved activation (debug view)."""
        ptr, n = B.lp_debug_saved_tensor(self.net, k, which)
        assert n == int(np.prod(shape))
        off = ptr - self.ws.data_ptr()
        esz = 2 if self.dtype == "bf16" else 4
        return self.to_host(self.ws[off:off + n * esz].view(self.tdtype).reshape(shape))

    def units(self, k):
        """The conv+BN units of module k (debug views, forward order)."""
        return [B.lp_debug_unit_info(self.net, k, i) for i in range(B.lp_debug_unit_count(self.net, k))]

    def fetch(self, ref, shape, kind="act"):
        """Host copy (float64) of the tensor a debug reference names.  kind: "act" storage type, "f64", "f32", "u8"."""
        n = int(np.prod(shape))
        if ref.space == B.LP_REF_NONE:
            return None
        if ref.space == B.LP_REF_WORKSPACE:
            tdt, esz = {"act": (self.tdtype, 2 if self.dtype == "bf16" else 4), "f64": (torch.float64, 8),
                        "f32": (torch.float32, 4), "u8": (torch.uint8, 1)}[kind]
            t = self.ws[ref.off:ref.off + n * esz].view(tdt).reshape(shape)
            return t.cpu().numpy().astype(np.float64) if kind in ("f64", "u8") else self.to_host(t)
        assert kind == "act" and ref.off == 0
        src = {B.LP_REF_X: self.x, B.LP_REF_Y: self.y, B.LP_REF_DY: self.dy, B.LP_REF_DX: self.dx}[ref.space][ref.idx]
        assert src.numel() == n
        return self.to_host(src).reshape(shape)

    # ---- the five entry points ---------------------------------------------------------------------
    @staticmethod
    def _stream():
        return torch.cuda.current_stream().cuda_stream

    def _mask(self, mask):
        return (1 << self.K) - 1 if mask is None else mask

    @staticmethod
    def _p(ts):
        return [None if t is None else t.data_ptr() for t in ts]

    def auxnet_forward(self, image=None):
        img = self.x[0] if image is None else image
        B.lp_auxnet_forward(self.net, self._stream(), img.data_ptr(), self._p(self.aux_params), self._p(self.x[1:]))

    def module_forward(self, mask=None):
        B.lp_module_forward(self.net, self._stream(), self._mask(mask), self._p(self.x), self._p(self.params),
                            self._p(self.y), self.logits.data_ptr())

    def local_loss_grad(self, rho, scale=1.0, mask=None):
        lam = None if self.lam is None else self._p(self.lam)
        B.lp_local_loss_grad(self.net, self._stream(), self._mask(mask), self._p(self.y), self._p(self.x[1:]), lam,
                             rho, scale, self.logits.data_ptr(), self.labels.data_ptr(), self.loss.data_ptr(),
                             self._p(self.dy), self.dlogits.data_ptr())

    def module_backward(self, mask=None, want_dx0=False):
        dx = self._p(self.dx)
        if not want_dx0:
            dx[0] = None
        B.lp_module_backward(self.net, self._stream(), self._mask(mask), self._p(self.dy), self.dlogits.data_ptr(),
                             self._p(self.params), self._p(self.dparams), dx)

    def al_multiplier_update(self, step):
        B.lp_al_multiplier_update(self.net, self._stream(), self._p(self.lam), self._p(self.y), self._p(self.x[1:]), step)

    def auxnet_distill_grad(self, scale=1.0, image=None, targets=None):
        """loss_j = scale*|AuxNet_j(image) - x_{j+1}|^2 and its gradient (after auxnet_forward)."""
        img = self.x[0] if image is None else image
        tg = self.x[1:] if targets is None else targets
        B.lp_auxnet_distill_grad(self.net, self._stream(), img.data_ptr(), self._p(self.aux_params), self._p(tg), scale,
                                 self.aux_loss.data_ptr(), self._p(self.daux_params))

    def reauxnet_grad(self, rho, scale=1.0, image=None):
        """Gradient of the relaxed objective with respect to the AuxNet parameters when x_k = AuxNet_k(image)
        (after auxnet_forward, module_forward, local_loss_grad and module_backward of the same step)."""
        img = self.x[0] if image is None else image
        dx = [None] + [t.data_ptr() for t in self.dx[1:]]
        B.lp_reauxnet_grad(self.net, self._stream(), img.data_ptr(), self._p(self.aux_params), self._p(self.y), dx,
                           None if self.lam is None else self._p(self.lam), rho, scale, self._p(self.daux_params))

    def sgd_update_aux(self, lr, momentum=0.0, weight_decay=0.0, velocity=None):
        B.lp_sgd_update(self.net, self._stream(), 1, (1 << (self.K - 1)) - 1, self._p(self.aux_params),
                        self._p(self.daux_params), None if velocity is None else self._p(velocity), None,
                        lr, momentum, weight_decay)

    def sgd_update(self, lr, momentum=0.0, weight_decay=0.0, velocity=None, master=None, mask=None):
        """W <- W - lr*(dW [+ wd*W, + momentum]) for the modules in `mask` (default all), in place."""
        B.lp_sgd_update(self.net, self._stream(), 0, self._mask(mask), self._p(self.params), self._p(self.dparams),
                        None if velocity is None else self._p(velocity), None if master is None else self._p(master),
                        lr, momentum, weight_decay)

    def set_fused_update(self, on, lr=0.0, momentum=0.0, weight_decay=0.0, velocity=None, master=None):
        """Parameter update inside the backward pass (in the epilogues of the filter-gradient kernels); `velocity` and
        `master` are lists of K device tensors laid out like the gradients and must stay alive while it is on."""
        self._fused_keep = (velocity, master)
        B.lp_net_set_fused_update(self.net, on, lr, momentum, weight_decay,
                                  None if velocity is None else self._p(velocity),
                                  None if master is None else self._p(master))

    def aux_variable_update(self, rho, scale, eta):
        """x_k <- x_k - eta*(scale*(rho*(x_k - y_{k-1}) - lam_{k-1}) + dx_k) for k = 1..K-1 (in place)."""
        x = [None] + [t.data_ptr() for t in self.x[1:]]
        dx = [None] + [t.data_ptr() for t in self.dx[1:]]
        B.lp_aux_variable_update(self.net, self._stream(), x, self._p(self.y), dx,
                                 None if self.lam is None else self._p(self.lam), rho, scale, eta)

    def local_step(self, rho, scale=1.0, mult_step=0.0, mask=None, want_dx0=False):
        """Forward, losses / terminal adjoints, backward and (mult_step != 0, multipliers set) the multiplier update of
        the selected modules in one call: every stream lane runs through all phases on its own."""
        dx = self._p(self.dx)
        if not want_dx0:
            dx[0] = None
        B.lp_local_step(self.net, self._stream(), self._mask(mask), self._p(self.x), self._p(self.params), self._p(self.y),
                        self._p(self.x[1:]), None if self.lam is None else self._p(self.lam), rho, scale, mult_step,
                        self.labels.data_ptr(), self.loss.data_ptr(), self._p(self.dy), self.logits.data_ptr(),
                        self.dlogits.data_ptr(), self._p(self.dparams), dx)

    def step(self, rho, scale=1.0, mult_step=None, with_aux=False):
        """One synchronous local step of all K modules."""
        if with_aux:
            self.auxnet_forward()
        self.local_step(rho, scale, 0.0 if (mult_step is None or self.lam is None) else mult_step)

    def capture_step(self, rho, scale=1.0, mult_step=None, with_aux=False, warmup=2):
        """The step as a HIP graph: `warmup` eager steps on a side stream (the library creates the streams and events of
        its lanes and sets its kernel attributes on first use, which must not happen inside a capture), then one step
        captured.  The library's fork / join of its stream lanes by events is a capture-legal pattern, it clears with
        kernels (no memset nodes) and allocates nothing per call.  Returns the torch.cuda.CUDAGraph; every replay() is
        one step on the buffers of this object (multipliers are updated in place, as in the eager step)."""
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            for _ in range(warmup):
                self.step(rho, scale, mult_step, with_aux)
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=side):
            self.step(rho, scale, mult_step, with_aux)
        return g
