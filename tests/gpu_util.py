"""Helpers shared by the GPU parity tests: device buffers in, numpy out, one call through the C ABI each."""
import numpy as np
import torch

from paper_2506_17615_amd import binding as eq


def dev_bf16(u16: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(u16, np.uint16).view(np.int16)).cuda().view(torch.bfloat16)


def host_u16(t: torch.Tensor) -> np.ndarray:
    return t.view(torch.int16).cpu().numpy().view(np.uint16)


def bf16_of(v: np.ndarray) -> np.ndarray:
    """fp32 numpy -> raw bf16 bits via torch's CPU cast."""
    t = torch.from_numpy(np.ascontiguousarray(v, np.float32)).to(torch.bfloat16)
    return t.view(torch.int16).numpy().view(np.uint16).copy()


def gpu_quantize(x_u16, B):
    x = dev_bf16(x_u16)
    n = x.numel()
    codes = torch.full((n,), 99, dtype=torch.int8, device="cuda")
    scales = torch.full((max(eq.num_blocks(n, B), 1),), -7.0, dtype=torch.float32, device="cuda")
    eq.equarx_quantize(x, B, codes, scales)
    torch.cuda.synchronize()
    return codes.cpu().numpy(), scales.cpu().numpy()[: eq.num_blocks(n, B)]


def gpu_dequantize(codes, scales, B):
    c = torch.from_numpy(np.ascontiguousarray(codes, np.int8)).cuda()
    s = torch.from_numpy(np.ascontiguousarray(scales, np.float32)).cuda()
    out = torch.full((c.numel(),), 7.0, dtype=torch.bfloat16, device="cuda")
    eq.equarx_dequantize(c, s, B, out)
    torch.cuda.synchronize()
    return host_u16(out)


def gpu_hop(codes_in, scales_in, local_u16, B, in_place=False):
    c = torch.from_numpy(np.ascontiguousarray(codes_in, np.int8)).cuda()
    s = torch.from_numpy(np.ascontiguousarray(scales_in, np.float32)).cuda()
    x = dev_bf16(local_u16)
    if in_place:
        co, so = c, s
    else:
        co = torch.full_like(c, 99)
        so = torch.full_like(s, -7.0)
    eq.equarx_reduce_stage(c, s, x, B, co, so)
    torch.cuda.synchronize()
    return co.cpu().numpy(), so.cpu().numpy()


def gpu_chain(partials_u16, B, keep_wire=True):
    """Runs equarx_reduce_quantized; returns out (u16) and, with keep_wire, wire codes [P,n] and scales [P,nb]."""
    parts = [dev_bf16(p) for p in partials_u16]
    P, n = len(parts), parts[0].numel()
    nb = eq.num_blocks(n, B)
    out = torch.full((n,), 7.0, dtype=torch.bfloat16, device="cuda")
    if keep_wire:
        rc, rs = eq.wire_row_codes(n), eq.wire_row_scales(n, B)
        wc = torch.full((P, rc), 99, dtype=torch.int8, device="cuda")
        ws = torch.full((P, rs), -7.0, dtype=torch.float32, device="cuda")
        eq.equarx_reduce_quantized(parts, B, out, None, wc, ws)
        torch.cuda.synchronize()
        return host_u16(out), wc[:, :n].cpu().numpy(), ws[:, :nb].cpu().numpy(), (wc, ws)
    work = eq.alloc_workspace(P, n, B)
    eq.equarx_reduce_quantized(parts, B, out, work)
    torch.cuda.synchronize()
    return host_u16(out)


def gpu_chain_fused(partials_u16, B, keep_wire=True):
    """Runs equarx_reduce_fused (one launch); same returns as gpu_chain."""
    parts = [dev_bf16(p) for p in partials_u16]
    P, n = len(parts), parts[0].numel()
    nb = eq.num_blocks(n, B)
    out = torch.full((n,), 7.0, dtype=torch.bfloat16, device="cuda")
    if keep_wire:
        rc, rs = eq.wire_row_codes(n), eq.wire_row_scales(n, B)
        wc = torch.full((P, rc), 99, dtype=torch.int8, device="cuda")
        ws = torch.full((P, rs), -7.0, dtype=torch.float32, device="cuda")
        eq.equarx_reduce_fused(parts, B, out, wc, ws)
        torch.cuda.synchronize()
        return host_u16(out), wc[:, :n].cpu().numpy(), ws[:, :nb].cpu().numpy()
    eq.equarx_reduce_fused(parts, B, out)
    torch.cuda.synchronize()
    return host_u16(out)


def gpu_chain_fused_ends(partials_u16, B):
    """Runs equarx_reduce_quantized_fused_ends (P-1 launches); returns the bf16 output bits."""
    parts = [dev_bf16(p) for p in partials_u16]
    P, n = len(parts), parts[0].numel()
    out = torch.full((n,), 7.0, dtype=torch.bfloat16, device="cuda")
    eq.equarx_reduce_quantized_fused_ends(parts, B, out, eq.alloc_workspace(P, n, B))
    torch.cuda.synchronize()
    return host_u16(out)


def gpu_chain_per_step(partials_u16, B):
    """The chain composed by hand from the per-step entry points (quantize, P-1 hops, dequantize: the calls a device
    of a ring makes, with their non-temporal wire accesses); returns out (u16), wire codes [P,n], scales [P,nb]."""
    parts = [dev_bf16(p) for p in partials_u16]
    P, n = len(parts), parts[0].numel()
    nb = eq.num_blocks(n, B)
    rows_c = [torch.full((n,), 99, dtype=torch.int8, device="cuda") for _ in range(P)]       # one allocation per wire:
    rows_s = [torch.full((nb,), -7.0, dtype=torch.float32, device="cuda") for _ in range(P)]  # each is aligned
    eq.equarx_quantize(parts[0], B, rows_c[0], rows_s[0])
    for i in range(1, P):
        eq.equarx_reduce_stage(rows_c[i - 1], rows_s[i - 1], parts[i], B, rows_c[i], rows_s[i])
    out = torch.full((n,), 7.0, dtype=torch.bfloat16, device="cuda")
    eq.equarx_dequantize(rows_c[P - 1], rows_s[P - 1], B, out)
    torch.cuda.synchronize()
    return host_u16(out), torch.stack(rows_c).cpu().numpy(), torch.stack(rows_s).cpu().numpy()


def gpu_chain_static(partials_u16, B):
    """Runs equarx_reduce_quantized_static (wire buffers in the library's static device array)."""
    parts = [dev_bf16(p) for p in partials_u16]
    out = torch.full((parts[0].numel(),), 7.0, dtype=torch.bfloat16, device="cuda")
    eq.equarx_reduce_quantized_static(parts, B, out)
    torch.cuda.synchronize()
    return host_u16(out)


def gpu_variant(partials_u16, B, flags):
    parts = [dev_bf16(p) for p in partials_u16]
    out = torch.full((parts[0].numel(),), 7.0, dtype=torch.bfloat16, device="cuda")
    eq.equarx_reduce_variant(parts, B, flags, out)
    torch.cuda.synchronize()
    return host_u16(out)
