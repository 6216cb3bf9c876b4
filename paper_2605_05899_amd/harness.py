"""Device-side plumbing shared by the benchmark, the smoke check and the GPU tests: upload one synthetic layer,
allocate its workspace and output buffers, run the fused call. Torch is used for device memory only; no arithmetic
of the method lives here."""
import numpy as np


def bf16_dev(u16, torch):
    """uint16 bf16 bit patterns (numpy) -> bf16 device tensor."""
    return torch.from_numpy(np.ascontiguousarray(u16).view(np.int16)).cuda().view(torch.bfloat16)


def bf16_host(t, torch):
    """bf16 device tensor -> float32 numpy array (exact widening)."""
    u = t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)
    return (u.astype(np.uint32) << 16).view(np.float32)


class DeviceLayer:
    """Device copies of one synthetic layer plus workspace and output buffers."""

    def __init__(self, inp, torch, moe, max_tokens=None):
        self.inp, self.torch, self.moe = inp, torch, moe
        self.cfg = moe.MoEConfig(H=inp.H, I=inp.I, E=inp.E, k=inp.k, S=inp.S, norm_topk=inp.norm_topk,
                                 max_tokens=max_tokens if max_tokens is not None else max(inp.T, 1))
        d = lambda a: None if a is None else bf16_dev(a, torch)
        self.x = d(inp.x)
        self.keep = None if inp.keep_idx is None else torch.from_numpy(inp.keep_idx).cuda()
        self.w_router, self.w_gate, self.w_up, self.w_down = d(inp.w_router), d(inp.w_gate), d(inp.w_up), d(inp.w_down)
        self.ws_gate, self.ws_up, self.ws_down = d(inp.ws_gate), d(inp.ws_up), d(inp.ws_down)
        self.ws = moe.alloc_workspace(self.cfg)
        T, k, H = inp.T, inp.k, inp.H
        self.out = torch.zeros((T, H), dtype=torch.bfloat16, device="cuda")
        self.ids = torch.zeros((T, k), dtype=torch.int32, device="cuda")
        self.w = torch.zeros((T, k), dtype=torch.float32, device="cuda")

    def layer_args(self, want_routing=False):
        """Positional arguments of moe.moe_layer_forward for this layer."""
        i = self.inp
        return (self.cfg, self.x, i.T_in, self.keep, i.T, self.w_router, self.w_gate, self.w_up, self.w_down,
                self.ws_gate, self.ws_up, self.ws_down, self.out, self.ids if want_routing else None,
                self.w if want_routing else None, self.ws)

    def forward(self, want_routing=True):
        self.moe.moe_layer_forward(*self.layer_args(want_routing))
        self.torch.cuda.synchronize()
        return bf16_host(self.out, self.torch), self.ids.cpu().numpy(), self.w.cpu().numpy()
