"""Device-side plumbing around the binding: uploads numpy inputs as torch tensors, owns the
output/scratch buffers of one layer and hands raw results back.  No arithmetic of the layer
happens here."""
import numpy as np
import torch

from . import astl, gswa, synth

_PARAMS = ("w_qkv", "b_qkv", "w_proj", "b_proj", "table")


def to_device(a, dtype, device="cuda:0"):
    """numpy fp32 values -> device tensor of storage type 'f32' or 'bf16' (RNE on the host)."""
    if dtype == "f32":
        return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(device)
    bits = synth.to_bf16_bits(a).reshape(np.shape(a))
    return torch.from_numpy(bits.view(np.int16)).to(device).view(torch.bfloat16)


def to_host(t):
    return t.detach().float().cpu().numpy()


class DeviceLayer:
    """Buffers of one GSWA layer call on the GPU (inputs, outputs, saved state, scratch)."""

    def __init__(self, B, H, W, C, heads, groups, window, shift, dtype, flags=0, device="cuda:0",
                 dqk=0):
        self.desc = gswa.make_desc(B, H, W, C, heads, groups, window, shift, dtype, flags, dqk)
        self.dtype, self.device = dtype, device
        self.shape = (B, H, W, C)
        tdt = torch.float32 if dtype == "f32" else torch.bfloat16
        self.saved_bytes, self.fwd_ws_bytes, self.bwd_ws_bytes = gswa.gswa_query_bytes(self.desc)
        self.y = torch.empty(self.shape, dtype=tdt, device=device)
        self.dx = torch.empty(self.shape, dtype=tdt, device=device)
        self.saved = torch.empty(self.saved_bytes, dtype=torch.uint8, device=device)
        ws_bytes = max(self.fwd_ws_bytes + self.saved_bytes, self.bwd_ws_bytes)
        self.ws = torch.empty(ws_bytes, dtype=torch.uint8, device=device)
        shp = synth.param_shapes(C, heads, groups, window, dqk)
        self.grads = {k: torch.empty(shp[k], dtype=torch.float32, device=device) for k in _PARAMS}
        self.params = None
        self.x = self.dy = None

    def set_params(self, p):
        self.params = {k: to_device(p[k], self.dtype, self.device) for k in _PARAMS}

    def set_inputs(self, x, dy=None):
        self.x = to_device(x, self.dtype, self.device)
        self.dy = None if dy is None else to_device(dy, self.dtype, self.device)

    def forward(self, keep=True, stream=None):
        p = self.params
        gswa.gswa_forward(self.desc, self.x, p["w_qkv"], p["b_qkv"], p["w_proj"], p["b_proj"],
                          p["table"], self.y, self.saved if keep else None, self.ws, stream)

    def backward(self, stream=None):
        p, g = self.params, self.grads
        gswa.gswa_backward(self.desc, self.x, self.dy, p["w_qkv"], p["b_qkv"], p["w_proj"],
                           p["b_proj"], p["table"], self.saved, self.dx, g["w_qkv"], g["b_qkv"],
                           g["w_proj"], g["b_proj"], g["table"], self.ws, stream)

    def results(self):
        out = {"y": to_host(self.y), "dx": to_host(self.dx)}
        out.update({"d" + k: to_host(v) for k, v in self.grads.items()})
        return out


class DeviceBlock:
    """Buffers of one whole-layer call (LayerNorms, attention, MLP, skips) on the GPU."""

    def __init__(self, B, H, W, C, heads, groups, window, shift, dtype, hidden, eps=1e-5, flags=0,
                 device="cuda:0", dqk=0):
        self.desc = astl.make_desc(B, H, W, C, heads, groups, window, shift, dtype, hidden, eps, flags, dqk)
        self.dtype, self.device = dtype, device
        self.shape = (B, H, W, C)
        tdt = torch.float32 if dtype == "f32" else torch.bfloat16
        self.saved_bytes, self.fwd_ws_bytes, self.bwd_ws_bytes = astl.astl_query_bytes(self.desc)
        self.y = torch.empty(self.shape, dtype=tdt, device=device)
        self.dx = torch.empty(self.shape, dtype=tdt, device=device)
        self.saved = torch.empty(self.saved_bytes, dtype=torch.uint8, device=device)
        ws_bytes = max(self.fwd_ws_bytes + self.saved_bytes, self.bwd_ws_bytes)
        self.ws = torch.empty(ws_bytes, dtype=torch.uint8, device=device)
        shp = synth.astl_param_shapes(C, heads, groups, window, hidden, dqk)
        self.grads = {k: torch.empty(s, dtype=torch.float32, device=device) for k, s in shp.items()}
        self.params = None
        self.x = self.dy = None

    @staticmethod
    def _fields(d):
        """synth's names -> the field names of the C structs (the bias table is `table` there)."""
        return {("bias_table" if k == "table" else k): v for k, v in d.items()}

    def set_params(self, p):
        self.params = {k: to_device(v, self.dtype, self.device) for k, v in p.items()}

    def set_inputs(self, x, dy=None):
        self.x = to_device(x, self.dtype, self.device)
        self.dy = None if dy is None else to_device(dy, self.dtype, self.device)

    def forward(self, keep=True, stream=None):
        astl.astl_forward(self.desc, self.x, self._fields(self.params), self.y,
                          self.saved if keep else None, self.ws, stream)

    def backward(self, stream=None):
        astl.astl_backward(self.desc, self.x, self.dy, self._fields(self.params), self.saved, self.dx,
                           self._fields(self.grads), self.ws, stream)

    def results(self):
        out = {"y": to_host(self.y), "dx": to_host(self.dx)}
        out.update({"d" + k: to_host(v) for k, v in self.grads.items()})
        return out


class DeviceStack:
    """Buffers of a sequence of whole layers (alternating shift) behind the stack entry points."""

    def __init__(self, B, H, W, C, heads, groups, window, shift, dtype, hidden, n_layers, checkpoint_every=0,
                 eps=1e-5, flags=0, device="cuda:0", dqk=0, band_windows=0, inference_only=False):
        """band_windows > 0: inference runs band by band (forward(keep=False)), with that many window rows
        per band.  inference_only: no buffers for the backward pass."""
        self.band_windows = band_windows
        self.desc = astl.make_stack_desc(B, H, W, C, heads, groups, window, shift, dtype, hidden, n_layers,
                                         checkpoint_every, eps, flags, dqk)
        self.dtype, self.device, self.n_layers = dtype, device, n_layers
        self.shape = (B, H, W, C)
        tdt = torch.float32 if dtype == "f32" else torch.bfloat16
        self.saved_bytes, self.fwd_ws_bytes, self.bwd_ws_bytes = astl.astl_stack_query_bytes(self.desc)
        self.y = torch.empty(self.shape, dtype=tdt, device=device)
        if band_windows:
            self.fwd_ws_bytes = astl.astl_stack_tiled_query_bytes(self.desc, band_windows)
        if inference_only:
            self.saved_bytes = self.bwd_ws_bytes = 0
            self.dx = self.saved = None
            self.grads = []
        else:
            self.dx = torch.empty(self.shape, dtype=tdt, device=device)
            self.saved = torch.empty(self.saved_bytes, dtype=torch.uint8, device=device)
            shp = synth.astl_param_shapes(C, heads, groups, window, hidden, dqk)
            self.grads = [{k: torch.empty(s, dtype=torch.float32, device=device) for k, s in shp.items()}
                          for _ in range(n_layers)]
        self.ws = torch.empty(max(self.fwd_ws_bytes, self.bwd_ws_bytes), dtype=torch.uint8, device=device)
        self.params = None
        self.x = self.dy = None

    def set_params(self, per_layer):
        self.params = [{k: to_device(v, self.dtype, self.device) for k, v in p.items()} for p in per_layer]

    def set_inputs(self, x, dy=None):
        self.x = to_device(x, self.dtype, self.device)
        self.dy = None if dy is None else to_device(dy, self.dtype, self.device)

    def forward(self, keep=True, stream=None):
        if self.band_windows and not keep:
            astl.astl_stack_forward_tiled(self.desc, self.x, [DeviceBlock._fields(p) for p in self.params], self.y,
                                          self.band_windows, self.ws, stream)
            return
        astl.astl_stack_forward(self.desc, self.x, [DeviceBlock._fields(p) for p in self.params], self.y,
                                self.saved if keep else None, self.ws, stream)

    def forward_tiled(self, band_windows, stream=None):
        """Inference band by band; the scratch is allocated here, at the size the library asks for."""
        need = astl.astl_stack_tiled_query_bytes(self.desc, band_windows)
        ws = torch.empty(need, dtype=torch.uint8, device=self.device)
        astl.astl_stack_forward_tiled(self.desc, self.x, [DeviceBlock._fields(p) for p in self.params], self.y,
                                      band_windows, ws, stream)
        return need

    def backward(self, stream=None):
        astl.astl_stack_backward(self.desc, self.x, self.dy, [DeviceBlock._fields(p) for p in self.params],
                                 self.saved, self.dx, [DeviceBlock._fields(g) for g in self.grads], self.ws, stream)

    def results(self):
        out = {"y": to_host(self.y), "dx": to_host(self.dx)}
        for l, g in enumerate(self.grads):
            out.update({f"{l}.d{k}": to_host(v) for k, v in g.items()})
        return out
