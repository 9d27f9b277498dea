"""Device-buffer plumbing around the C ABI: torch allocates, libftp computes."""
import numpy as np
import torch

from . import binding as B


def _np_to_dev(a, bf16):
    t = torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32))
    if bf16:
        t = t.to(torch.bfloat16)          # inputs are already bf16-representable: exact
    return t.cuda()


class Session:
    """One plan plus every device buffer it needs.  layers: objects with kind,k,stride,pad,cin,cout,slope."""

    def __init__(self, layers, batch, in_c, in_h, in_w, grid, group_ends, dtype="f32", device="cuda:0"):
        torch.cuda.set_device(device)
        self.layers = list(layers)
        self.bf16 = dtype == "bf16"
        self.tdtype = torch.bfloat16 if self.bf16 else torch.float32
        self.batch = batch
        self.grid = tuple(grid)
        self.plan = B.ftp_plan(self.layers, batch, in_c, in_h, in_w, grid[0], grid[1], list(group_ends),
                               B.FTP_BF16 if self.bf16 else B.FTP_F32)
        self.sizes = B.ftp_plan_sizes(self.plan)
        self.work = B.ftp_plan_work(self.plan)
        L = len(self.layers)
        self.in_shape = (batch,) + B.ftp_plan_map_shape(self.plan, 0)
        self.out_shape = (batch,) + B.ftp_plan_map_shape(self.plan, L)
        self.n_params = self.sizes["n_params"]
        self.stacks = grid[0] * grid[1]
        self.workspace = torch.empty(self.sizes["workspace_bytes"], dtype=torch.uint8, device="cuda")
        self.x = torch.empty(self.in_shape, dtype=self.tdtype, device="cuda")
        self.y = torch.empty(self.out_shape, dtype=self.tdtype, device="cuda")
        self.dy = torch.empty(self.out_shape, dtype=self.tdtype, device="cuda")
        self.dx = torch.empty(self.in_shape, dtype=self.tdtype, device="cuda")
        self.partials = torch.empty((self.stacks, self.n_params), dtype=torch.float32, device="cuda")
        self.wgrad = torch.empty((self.n_params,), dtype=torch.float32, device="cuda")
        self.weights = [None] * L
        self.biases = None

    def close(self):
        if self.plan is not None:
            B.ftp_plan_destroy(self.plan)
            self.plan = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def load(self, x=None, weights=None, dy=None, biases=None):
        if x is not None:
            self.x.copy_(_np_to_dev(x, self.bf16))
        if dy is not None:
            self.dy.copy_(_np_to_dev(dy, self.bf16))
        if weights is not None:
            self.weights = [None if w is None else _np_to_dev(w, self.bf16) for w in weights]
        if biases is not None:
            self.biases = [None if b is None else _np_to_dev(b, self.bf16) for b in biases]

    def _wptrs(self):
        return [0 if w is None else w.data_ptr() for w in self.weights]

    def _bptrs(self):
        if self.biases is None:
            return None
        return [0 if b is None else b.data_ptr() for b in self.biases]

    def set_overlap(self, enable):
        """Filter gradients on a second stream beside the delta back-propagation (same results, shorter pass)."""
        B.ftp_set_overlap(self.plan, enable)

    def _stream(self):
        return torch.cuda.current_stream().cuda_stream

    def forward(self):
        B.ftp_forward(self.plan, self.x.data_ptr(), self._wptrs(), self._bptrs(), self.workspace.data_ptr(),
                      self.y.data_ptr(), self._stream())

    def backward(self):
        B.ftp_backward(self.plan, self.dy.data_ptr(), self.x.data_ptr(), self._wptrs(),
                       self.workspace.data_ptr(), self.dx.data_ptr(), self.partials.data_ptr(), self._stream())

    def reduce(self):
        B.ftp_reduce_wgrad(self.plan, self.partials.data_ptr(), self.wgrad.data_ptr(), self._stream())

    def sgd_step(self, lr, keep_wgrad=True):
        """Gradient sum fused with W <- W - lr * dW on the session's weight tensors."""
        B.ftp_sgd_step(self.plan, self.partials.data_ptr(), self._wptrs(), self._bptrs(), lr,
                       self.wgrad.data_ptr() if keep_wgrad else 0, self._stream())

    def step(self):
        self.forward()
        self.backward()
        self.reduce()

    def train_step(self, lr):
        """One training cycle: forward, back-propagation, gradient sum + filter update."""
        self.forward()
        self.backward()
        self.sgd_step(lr)

    # ---- inspection of the workspace (tests, debugging): plain tensor views and copies, no arithmetic ----
    def _buffer(self, boundary, which):
        info = B.ftp_plan_buffer(self.plan, boundary, which)
        loc = info["location"]
        if loc == 0:
            return None, info
        if loc in (1, 2, 3, 4):
            return {1: self.x, 2: self.y, 3: self.dy, 4: self.dx}[loc], info
        dt = {B.FTP_BUF_MASK: torch.uint8, B.FTP_BUF_SIGN: torch.int32}.get(which, self.tdtype)
        esz = {B.FTP_BUF_MASK: 1, B.FTP_BUF_SIGN: 4}.get(which, 2 if self.bf16 else 4)
        lead = (self.stacks,) if info["per_stack"] else ()
        shape = lead + (self.batch, info["channels"], info["slot_h"], info["slot_w"])
        n = 1
        for d in shape:
            n *= d
        t = self.workspace[info["offset"]:info["offset"] + n * esz].view(dt).view(shape)
        return t, info

    def _rect(self, info, boundary, stack, kind):
        return B.ftp_plan_rect(self.plan, info["group"], boundary, stack // self.grid[1], stack % self.grid[1], kind)

    def get_boundary(self, boundary, which=B.FTP_BUF_ACT, images=None):
        """Whole map at a boundary, assembled from what each stack owns.  None if the plan keeps none.
        images: optional list of image indices to fetch (default: the whole batch)."""
        t, info = self._buffer(boundary, which)
        if t is None:
            return None
        idx = list(range(self.batch)) if images is None else list(images)
        if not info["per_stack"]:
            return self.to_np(t[idx])
        c, h, w = B.ftp_plan_map_shape(self.plan, boundary)
        out = torch.zeros((len(idx), c, h, w), dtype=t.dtype, device=t.device)
        for s in range(self.stacks):
            o = self._rect(info, boundary, s, B.FTP_RECT_OWN)
            r = self._rect(info, boundary, s, info["rect_kind"])
            out[:, :, o[1]:o[3] + 1, o[0]:o[2] + 1] = t[s][idx][:, :, o[1] - r[1]:o[3] - r[1] + 1, o[0] - r[0]:o[2] - r[0] + 1]
        return self.to_np(out)

    def get_slots(self, boundary, which=B.FTP_BUF_ACT, images=None):
        """[(rect, array)] per stack: everything a stack holds at an interior boundary (own tile + halo)."""
        t, info = self._buffer(boundary, which)
        if t is None or not info["per_stack"]:
            return []
        idx = list(range(self.batch)) if images is None else list(images)
        out = []
        for s in range(self.stacks):
            r = self._rect(info, boundary, s, info["rect_kind"])
            out.append((r, self.to_np(t[s][idx][:, :, :r[3] - r[1] + 1, :r[2] - r[0] + 1])))
        return out

    def set_boundary(self, boundary, full_map, which=B.FTP_BUF_ACT, images=None):
        """Writes a whole map into the plan's buffer(s) of a boundary (every stack gets its rectangle).
        images: optional list of image indices the rows of `full_map` belong to (default: the whole batch)."""
        t, info = self._buffer(boundary, which)
        if t is None:
            return
        src = torch.from_numpy(np.ascontiguousarray(full_map))
        src = src.cuda() if which in (B.FTP_BUF_MASK, B.FTP_BUF_SIGN) else src.float().cuda().to(t.dtype)
        idx = slice(None) if images is None else torch.as_tensor(list(images), device=t.device)
        if not info["per_stack"]:
            t[idx] = src
            return
        for s in range(self.stacks):
            r = self._rect(info, boundary, s, info["rect_kind"])
            t[s, idx, :, :r[3] - r[1] + 1, :r[2] - r[0] + 1] = src[:, :, r[1]:r[3] + 1, r[0]:r[2] + 1]

    @staticmethod
    def to_np(t):
        t = t.detach()
        return t.cpu().numpy() if t.dtype in (torch.uint8, torch.int32) else t.float().cpu().numpy()
