"""Device-buffer bookkeeping around the C ABI: allocates the caller-owned arrays once and forwards every step
to the library.  No arithmetic happens here."""
from __future__ import annotations

import numpy as np

from . import binding as B


def to_device(a: np.ndarray, device="cuda"):
    """Host array -> device tensor.  uint16 arrays are bf16 bit patterns and become torch.bfloat16."""
    import torch
    a = np.ascontiguousarray(a)
    if a.dtype == np.uint16:
        return torch.from_numpy(a.view(np.int16)).to(device).view(torch.bfloat16)
    return torch.from_numpy(a).to(device)


def from_device_bf16_bits(t) -> np.ndarray:
    import torch
    return t.view(torch.int16).cpu().numpy().view(np.uint16)


class MoELayer:
    """All device state of one layer: routing outputs, dispatch tables, packed weights, workspaces, y."""

    def __init__(self, cfg, device="cuda", unfused: bool = False):
        import torch
        self.cfg = cfg
        self.device = device
        self.shape = B.shape_of(cfg)
        s = self.shape
        self.elt_dtype = torch.bfloat16 if cfg.dtype == B.MOE_BF16 else torch.float32
        n = max(1, s.T * s.k)
        self.topk_idx = torch.empty(n, dtype=torch.int32, device=device)
        self.topk_w = torch.empty(n, dtype=torch.float32, device=device)
        self.tables = B.DispatchTables(s, device)
        self.dispatch_ws = torch.empty(max(1, B.moe_dispatch_workspace_bytes(s)), dtype=torch.uint8, device=device)
        nbytes = B.moe_unfused_workspace_bytes(s) if unfused else B.moe_forward_workspace_bytes(s)
        self.forward_ws = torch.empty(max(1, nbytes), dtype=torch.uint8, device=device)
        self.y = torch.empty((max(1, s.T), s.d), dtype=self.elt_dtype, device=device)
        self.packed_gate_up = None
        self.packed_down = None

    def load_weights(self, W_gate: np.ndarray, W_up: np.ndarray, W_down: np.ndarray) -> None:
        import torch
        s = self.shape
        self.packed_gate_up = torch.empty(B.moe_packed_weight_bytes(s, 0), dtype=torch.uint8, device=self.device)
        self.packed_down = torch.empty(B.moe_packed_weight_bytes(s, 1), dtype=torch.uint8, device=self.device)
        g, u, d = (to_device(a, self.device) for a in (W_gate, W_up, W_down))
        B.moe_pack_weights(s, g, u, d, self.packed_gate_up, self.packed_down)
        torch.cuda.synchronize()
        del g, u, d

    def load_weights_fp8(self, W_gate: np.ndarray, W_up: np.ndarray, W_down: np.ndarray, h_scale: np.ndarray) -> None:
        """Quantise and pack the weights for the FP8 form of the GEMMs; h_scale [E_loc] is the static scale of h."""
        import torch
        s = self.shape
        self.fp8_gate_up = torch.empty(B.moe_fp8_packed_weight_bytes(s, 0), dtype=torch.uint8, device=self.device)
        self.fp8_down = torch.empty(B.moe_fp8_packed_weight_bytes(s, 1), dtype=torch.uint8, device=self.device)
        self.fp8_ws = torch.empty(max(1, B.moe_fp8_forward_workspace_bytes(s)), dtype=torch.uint8, device=self.device)
        self.h_scale = to_device(np.ascontiguousarray(h_scale, dtype=np.float32), self.device)
        g, u, d = (to_device(a, self.device) for a in (W_gate, W_up, W_down))
        B.moe_fp8_pack_weights(s, g, u, d, self.fp8_gate_up, self.fp8_down)
        torch.cuda.synchronize()
        del g, u, d

    def forward_fp8(self, x, events=None) -> None:
        B.moe_fp8_fused_forward(self.shape, x, self.topk_idx, self.topk_w, self.tables, self.fp8_gate_up,
                                self.fp8_down, self.h_scale, self.y, self.fp8_ws, events)

    def enable_training(self, W_gate: np.ndarray, W_up: np.ndarray, W_down: np.ndarray, wgrad: bool = True) -> None:
        """Buffers of the training path: transposed weight packs, the kept activations, gradients, workspace."""
        import torch
        s = self.shape
        dev = self.device
        self.packed_down_t = torch.empty(B.moe_backward_packed_weight_bytes(s, 0), dtype=torch.uint8, device=dev)
        self.packed_gate_up_t = torch.empty(B.moe_backward_packed_weight_bytes(s, 1), dtype=torch.uint8, device=dev)
        g, u, d = (to_device(a, dev) for a in (W_gate, W_up, W_down))
        B.moe_pack_weights_backward(s, g, u, d, self.packed_down_t, self.packed_gate_up_t)
        torch.cuda.synchronize()
        del g, u, d
        self.kept = torch.empty(max(1, B.moe_train_kept_bytes(s)), dtype=torch.uint8, device=dev)
        self.backward_ws = torch.empty(max(1, B.moe_backward_workspace_bytes(s)), dtype=torch.uint8, device=dev)
        self.dx = torch.empty((max(1, s.T), s.d), dtype=torch.bfloat16, device=dev)
        self.d_topk_w = torch.empty(max(1, s.T * s.k), dtype=torch.float32, device=dev)
        El = self.cfg.E_loc
        if wgrad:
            self.dW_gate = torch.empty((El, s.d, s.f), dtype=torch.bfloat16, device=dev)
            self.dW_up = torch.empty((El, s.d, s.f), dtype=torch.bfloat16, device=dev)
            self.dW_down = torch.empty((El, s.f, s.d), dtype=torch.bfloat16, device=dev)
        else:
            self.dW_gate = self.dW_up = self.dW_down = None

    def forward_train(self, x) -> None:
        B.moe_fused_forward_train(self.shape, x, self.topk_idx, self.topk_w, self.tables, self.packed_gate_up,
                                  self.packed_down, self.y, self.kept, self.forward_ws)

    def backward(self, x, dy) -> None:
        B.moe_fused_backward(self.shape, x, dy, self.topk_idx, self.topk_w, self.tables, self.packed_down_t,
                             self.packed_gate_up_t, self.kept, self.dx, self.d_topk_w, self.dW_gate, self.dW_up,
                             self.dW_down, self.backward_ws)

    def route(self, logits) -> None:
        B.moe_route_topk(self.shape, logits, self.topk_idx, self.topk_w)

    def build_dispatch(self) -> None:
        B.moe_build_dispatch(self.shape, self.topk_idx, self.tables, self.dispatch_ws)

    def forward(self, x) -> None:
        B.moe_fused_forward(self.shape, x, self.topk_idx, self.topk_w, self.tables, self.packed_gate_up,
                            self.packed_down, self.y, self.forward_ws)

    def forward_two_launch(self, x, events=None) -> None:
        B.moe_fused_forward_two_launch(self.shape, x, self.topk_idx, self.topk_w, self.tables, self.packed_gate_up,
                                       self.packed_down, self.y, self.forward_ws, events)

    def forward_one_launch(self, x, events=None) -> None:
        B.moe_fused_forward_one_launch(self.shape, x, self.topk_idx, self.topk_w, self.tables, self.packed_gate_up,
                                       self.packed_down, self.y, self.forward_ws, events)

    def forward_resident(self, x, events=None) -> None:
        """GEMM-1, GEMM-2 and Combine in one launch."""
        B.moe_fused_forward_resident(self.shape, x, self.topk_idx, self.topk_w, self.tables, self.packed_gate_up,
                                     self.packed_down, self.y, self.forward_ws, events)

    def forward_unfused(self, x) -> None:
        B.moe_unfused_forward(self.shape, x, self.topk_idx, self.topk_w, self.tables, self.packed_gate_up,
                              self.packed_down, self.y, self.forward_ws)

    def step(self, logits, x) -> None:
        """One pass of the whole hot path."""
        self.route(logits)
        self.build_dispatch()
        self.forward(x)

    def y_host(self) -> np.ndarray:
        """y as float64 on the host (bf16 values widened exactly)."""
        import torch
        return self.y[: self.shape.T].to(torch.float64).cpu().numpy()
