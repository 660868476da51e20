"""Device-side harness of the binding: uploads one seeded case and runs pe_block_fwd / pe_block_bwd on it.
Argument marshalling only (no arithmetic of the method); used by the tests, the smoke check and bench.py."""
import numpy as np
import torch

from . import binding as pe


def tdtype(dims):
    return torch.bfloat16 if dims["dtype"] == pe.PE_BF16 else torch.float32


def to_dev(a, dt):
    return torch.from_numpy(np.ascontiguousarray(a)).to(torch.float32).to("cuda").to(dt).contiguous()


def to_np(t):
    return t.detach().to(torch.float32).cpu().numpy().astype(np.float64)


class BlockRun:
    """Uploads one seeded case and runs pe_block_fwd / pe_block_bwd on it."""

    def __init__(self, dims, inp, two_streams=True, sync_debug=False):
        self.dims, self.dt = dims, tdtype(dims)
        self.h = pe.Handle()
        if sync_debug:
            self.h.set_option(2, 1)
        f32 = torch.float32
        self.msa, self.pair = to_dev(inp["msa"], self.dt), to_dev(inp["pair"], self.dt)
        self.msa_mask, self.pair_mask = to_dev(inp["msa_mask"], f32), to_dev(inp["pair_mask"], f32)
        self.params = to_dev(inp["params"], f32)
        self.d_msa_out, self.d_pair_out = to_dev(inp["d_msa_out"], self.dt), to_dev(inp["d_pair_out"], self.dt)
        self.msa_out, self.pair_out = torch.empty_like(self.msa), torch.empty_like(self.pair)
        self.d_msa_in, self.d_pair_in = torch.empty_like(self.msa), torch.empty_like(self.pair)
        self.d_params = torch.zeros_like(self.params)
        self.ctx = torch.empty(pe.ctx_bytes(dims), dtype=torch.uint8, device="cuda")
        self.ws = torch.empty(pe.workspace_bytes(dims, 1), dtype=torch.uint8, device="cuda")
        self.sm = torch.cuda.Stream() if two_streams else torch.cuda.current_stream()
        self.sp = torch.cuda.Stream() if two_streams else self.sm
        torch.cuda.synchronize()

    def fwd(self, use_ctx=True):
        pe.block_fwd(self.h, self.dims, self.msa, self.pair, self.msa_mask, self.pair_mask, self.params,
                     self.msa_out, self.pair_out, self.ctx if use_ctx else None, self.ws, self.sm, self.sp)

    def bwd(self, use_ctx=True):
        pe.block_bwd(self.h, self.dims, self.msa, self.pair, self.msa_mask, self.pair_mask, self.params,
                     self.d_msa_out, self.d_pair_out, self.d_msa_in, self.d_pair_in, self.d_params,
                     self.ctx if use_ctx else None, self.ws, self.sm, self.sp)

    def sync(self):
        torch.cuda.synchronize()

    def ctx_entry(self, name):
        for e in pe.ctx_table(self.dims):
            if e["name"] == name:
                dt = torch.bfloat16 if e["dtype"] == pe.PE_BF16 else torch.float32
                nb = e["count"] * (2 if e["dtype"] == pe.PE_BF16 else 4)
                return to_np(self.ctx[e["offset_bytes"]:e["offset_bytes"] + nb].view(dt))
        raise KeyError(name)
