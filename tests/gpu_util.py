"""Helpers shared by the GPU parity tests (marshalling only)."""
import numpy as np
import torch

from paper_2512_04226_amd import binding as g


def to_dev(bits):
    """numpy uint16 (bf16 bits) or uint8 (e4m3 codes) -> device tensor of the same bits."""
    if bits.dtype == np.uint16:
        return torch.from_numpy(bits.view(np.int16)).cuda()
    return torch.from_numpy(bits).cuda()


_ws = {}


def workspace_for(cfg):
    need = g.gemm_workspace_bytes(cfg)
    if need == 0:
        return None
    cur = _ws.get("t")
    if cur is None or cur.numel() * 4 < need:
        cur = torch.empty((need + 3) // 4, dtype=torch.float32, device="cuda")
        _ws["t"] = cur
        g.gemm_set_workspace(cur)
    return cur


def run_cfg(cfg, dA, dB, M, N, alpha=1.0, poison=True):
    """Run one configuration; returns bf16 bit patterns as numpy uint16 (M x N)."""
    workspace_for(cfg)
    c = cfg.copy()
    c.alpha = alpha
    dC = torch.empty((M, N), dtype=torch.int16, device="cuda")
    if poison:
        dC.fill_(0x7FC0)   # NaN pattern: unwritten outputs fail the compare
    g.gemm_run(c, dA, dB, dC)
    torch.cuda.synchronize()
    return dC.cpu().numpy().view(np.uint16)


def bf16_to_f64(bits):
    return (bits.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
