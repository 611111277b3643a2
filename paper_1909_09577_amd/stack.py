"""Forward + backward of a Jasper 10x5-shaped encoder stack, chained through the C ABI.

The stack is the paper's ASR encoder (Section 4.1.1) as the synthetic workload list describes it:
a stride-2 prolog, ten blocks of five conv1d sub-blocks whose fifth takes the block's residual --
a K=1 projection of the block input (affine, no ReLU) -- and three epilog layers.  This module only
wires layers: every tensor operation is a call into libnmconv1d (block forward, fused backward);
torch provides device memory and the stream.  All activations, gradients and the workspace are
allocated once, so a step allocates nothing.

Backward wiring of a block: the residual gradient `dres` of the fifth sub-block is the upstream
gradient of the projection; the block-input gradient is dx(first sub-block) + dx(projection), formed
by the projection's input-gradient call with NM_ACCUM_DX on the first sub-block's dx (one rounding).
"""
from __future__ import annotations

from typing import List, Optional

from . import binding as nm


class StackLayer:
    """One conv1d sub-block of the stack: parameters, saved tensors, gradients (device tensors)."""

    def __init__(self, cfg, role, block, w, scale, shift):
        self.cfg, self.role, self.block = cfg, role, block
        self.w, self.scale, self.shift = w, scale, shift
        self.kw = dict(stride=cfg.stride, dilation=cfg.dilation, pad=cfg.pad)
        self.x = self.residual = self.dy = None   # references to other layers' tensors, set while running
        self.y = self.dx = self.dres = self.dw = None  # owned outputs


class EncoderStack:
    def __init__(self, layers: List[dict], params: List[dict], device="cuda", record_partial_dx: bool = False):
        """layers: entries {"cfg", "role", "block"} (inputs.jasper_10x5_layers); params: per layer
        {"w", "scale", "shift"} device tensors (scale/shift None where the layer has no affine).
        record_partial_dx keeps a copy of every first sub-block's dx before the projection's gradient is
        accumulated into it (for checks; costs one device copy per block)."""
        import torch
        self.record_partial_dx = record_partial_dx
        self.partial_dx = {}
        self.layers = [StackLayer(e["cfg"], e["role"], e["block"], p["w"], p.get("scale"), p.get("shift"))
                       for e, p in zip(layers, params)]
        roles = [l.role for l in self.layers]
        assert roles[0] == "prolog"
        self.prolog = self.layers[0]
        self.blocks = []
        i = 1
        while i < len(roles) and roles[i] == "proj":
            assert roles[i + 1:i + 6] == ["sub"] * 5
            self.blocks.append((self.layers[i], self.layers[i + 1:i + 6]))
            i += 6
        self.epilog = self.layers[i:]
        assert all(l.role == "epilog" for l in self.epilog)
        bf = torch.bfloat16
        ws_bytes = 256
        for l in self.layers:
            c = l.cfg
            l.y = torch.empty((c.B, c.Cout, c.T_out), dtype=bf, device=device)
            l.dx = torch.empty((c.B, c.Cin, c.T), dtype=bf, device=device)
            l.dw = torch.empty((c.Cout, c.Cin, c.K), dtype=torch.float32, device=device)
            l.dres = torch.empty((c.B, c.Cout, c.T_out), dtype=bf, device=device) if c.residual else None
            for op in (nm.NM_OP_FWD, nm.NM_OP_BWD):
                ws_bytes = max(ws_bytes, nm.nm_conv1d_workspace_bytes(op, *c.dims(), nm.NM_BF16, nm.NM_RELU))
        # a projection writes its input gradient into the first sub-block's dx
        for proj, subs in self.blocks:
            proj.dx = subs[0].dx
        self.workspace = torch.empty(ws_bytes, dtype=torch.uint8, device=device)

    # ---- one layer ----------------------------------------------------------------------------
    def _fwd(self, l: StackLayer, x, residual=None):
        l.x, l.residual = x, residual
        nm.nm_conv1d_block_fwd(x, l.w, l.scale, l.shift, residual, y=l.y, relu=l.cfg.relu, workspace=self.workspace,
                               **l.kw)
        return l.y

    def _bwd(self, l: StackLayer, dy, accumulate_dx=False, accumulate_dw=False):
        l.dy = dy
        nm.nm_conv1d_bwd(l.x, dy, l.w, y=l.y if l.cfg.relu else None, scale=l.scale, dx=l.dx, dres=l.dres, dw=l.dw,
                         relu=l.cfg.relu, accumulate=accumulate_dw, accumulate_dx=accumulate_dx,
                         workspace=self.workspace, **l.kw)
        return l.dx

    # ---- the stack ----------------------------------------------------------------------------
    def forward(self, x):
        h = self._fwd(self.prolog, x)
        for proj, subs in self.blocks:
            r = self._fwd(proj, h)
            g = h
            for j, sub in enumerate(subs):
                g = self._fwd(sub, g, residual=r if j == 4 else None)
            h = g
        for ep in self.epilog:
            h = self._fwd(ep, h)
        return h

    def backward(self, dy, accumulate_dw: bool = False):
        """Gradients of every layer's weights (layer.dw) and of the stack input (returned) from the
        gradient of the last layer's output.  accumulate_dw adds into the existing dw tensors."""
        g = dy
        for ep in reversed(self.epilog):
            g = self._bwd(ep, g, accumulate_dw=accumulate_dw)
        for bi in range(len(self.blocks) - 1, -1, -1):
            proj, subs = self.blocks[bi]
            for sub in reversed(subs):
                g = self._bwd(sub, g, accumulate_dw=accumulate_dw)
            if self.record_partial_dx:
                self.partial_dx[bi] = g.clone()
            g = self._bwd(proj, subs[4].dres, accumulate_dx=True, accumulate_dw=accumulate_dw)
        return self._bwd(self.prolog, g, accumulate_dw=accumulate_dw)

    def step(self, x, dy):
        """One training step's worth of layer work: forward, then backward."""
        y = self.forward(x)
        return y, self.backward(dy)

    @property
    def flops_per_step(self) -> int:
        return sum(3 * l.cfg.flops_per_pass for l in self.layers)


def random_parameters(layers: List[dict], seed: Optional[int] = 0, device="cuda"):
    """Random-initialised parameters of the stack on the device (weights ~ N(0, 1/(Cin*K)) in bf16,
    scale ~ U(0.5, 1.5), shift ~ N(0, 0.1) in float32), generated on the device: for timing runs."""
    import torch
    gen = torch.Generator(device=device)
    gen.manual_seed(int(seed or 0))
    out = []
    for e in layers:
        c = e["cfg"]
        w = (torch.randn(c.Cout, c.Cin, c.K, device=device, generator=gen) / (c.Cin * c.K) ** 0.5).bfloat16()
        scale = (torch.rand(c.Cout, device=device, generator=gen) + 0.5) if c.affine else None
        shift = (torch.randn(c.Cout, device=device, generator=gen) * 0.1) if c.affine else None
        out.append({"w": w, "scale": scale, "shift": shift})
    return out
