"""Helpers for the GPU parity tests: move seeded inputs to the device, call the C ABI, fetch results.
torch is used for device memory and streams only."""
from __future__ import annotations

import numpy as np

import paper_2503_01873_amd as P
from oracle import pasa_oracle as po

ORACLE_POLICY = {P.MIXED: po.MIXED, P.STRICT16: po.STRICT16, P.S16: po.PARTIAL16}
VARIANT_NAME = {P.MIXED: "MIXED", P.STRICT16: "STRICT16", P.NAIVE16: "NAIVE16", P.S16: "S16", P.DIRECT: "DIRECT"}


def f32(x: float) -> float:
    """The value a C float argument will carry."""
    return float(np.float32(x))


def bf16_bits(x32):
    """float32 array holding bf16-representable values -> their 16-bit patterns (input plumbing only)."""
    x32 = np.ascontiguousarray(x32, np.float32)
    u = x32.view(np.uint32)
    assert not (u & 0xFFFF).any(), "not bf16 values"
    return (u >> 16).astype(np.uint16)


def gpu_attn(q, k, v, causal, scale, variant=P.MIXED, beta=-1.0, counters=False, entry="ex",
             shift_mode=P.SHIFT_MEAN, bf16=False):
    """Run the HIP path on numpy fp16 inputs [B,H,N,d]; returns (o fp16 numpy, counters or None).
    bf16=True: inputs are float32 arrays of bf16 values, passed to the device as bf16; o comes back as float32."""
    import torch
    dev = torch.device("cuda:0")
    B, Hq, N, d = q.shape
    Hkv = k.shape[1]
    if bf16:   # same 2-byte element size: the fp16-typed torch buffers below only carry the bits
        q, k, v = (bf16_bits(x).view(np.float16) for x in (q, k, v))
    tq, tk, tv = (torch.from_numpy(np.ascontiguousarray(x)).to(dev) for x in (q, k, v))
    guard = 4096                        # sentinel elements after the output: nothing may write past its end
    flat = torch.full((tq.numel() + guard,), float("nan"), dtype=torch.float16, device=dev)
    to = flat[:tq.numel()].view(tq.shape)
    cnt = torch.zeros(2, dtype=torch.int64, device=dev) if counters else None
    stream = torch.cuda.current_stream()
    if entry == "plain":
        P.pasa_attn_fwd(tq, tk, tv, to, B, Hq, Hkv, N, d, causal, scale, stream)
    else:
        wsb = P.pasa_attn_fwd_workspace(B, Hq, Hkv, N, d)
        ws = torch.empty(wsb, dtype=torch.uint8, device=dev)
        kw = dict(beta=beta, variant=variant, shift_mode=shift_mode, io_dtype=P.IO_BF16 if bf16 else P.IO_F16)
        if entry == "ex":
            P.pasa_attn_fwd_ex(tq, tk, tv, to, B, Hq, Hkv, N, d, causal, scale, ws, wsb, stream,
                               overflow_s=cnt[0:1] if counters else None,
                               nonfinite_o=cnt[1:2] if counters else None, **kw)
        elif entry == "split":
            P.pasa_prepare_kv(tk, tv, B, Hkv, N, d, scale, ws, wsb, stream, **kw)
            P.pasa_attn_fwd_prepared(tq, to, B, Hq, Hkv, N, d, causal, scale, ws, wsb, stream, **kw)
        else:
            raise ValueError(entry)
    torch.cuda.synchronize()
    assert bool(torch.isnan(flat[tq.numel():]).all()), "the kernel wrote past the end of the output"
    o = to.cpu().numpy()
    if bf16:
        o = (o.view(np.uint16).astype(np.uint32) << 16).view(np.float32)
    return o, (cnt.cpu().numpy() if counters else None)


def gpu_attn_chunks(q, k, v, causal, scale, chunks, variant=P.MIXED, beta=-1.0):
    """K/V prepared once, then one pasa_attn_fwd_chunk call per (first query row, row count, row0) of `chunks`.
    q: [B,Hq,Nq,d] numpy fp16; each chunk's rows are copied to a buffer of their own.  Returns o [B,Hq,Nq,d]."""
    import torch
    dev = torch.device("cuda:0")
    B, Hq, Nq, d = q.shape
    Hkv, N = k.shape[1], k.shape[2]
    tk, tv = (torch.from_numpy(np.ascontiguousarray(x)).to(dev) for x in (k, v))
    wsb = P.pasa_attn_fwd_workspace(B, Hq, Hkv, N, d)
    ws = torch.empty(wsb, dtype=torch.uint8, device=dev)
    stream = torch.cuda.current_stream()
    P.pasa_prepare_kv(tk, tv, B, Hkv, N, d, scale, ws, wsb, stream, beta=beta, variant=variant)
    out = np.full(q.shape, np.nan, np.float16)
    guard = 4096
    for first, count, row0 in chunks:
        tq = torch.from_numpy(np.ascontiguousarray(q[:, :, first:first + count])).to(dev)
        flat = torch.full((tq.numel() + guard,), float("nan"), dtype=torch.float16, device=dev)
        to = flat[:tq.numel()].view(tq.shape)
        P.pasa_attn_fwd_chunk(tq, to, B, Hq, Hkv, count, row0, N, d, causal, scale, ws, wsb, stream,
                              beta=beta, variant=variant)
        torch.cuda.synchronize()
        assert bool(torch.isnan(flat[tq.numel():]).all()), "the kernel wrote past the end of the output"
        out[:, :, first:first + count] = to.cpu().numpy()
    return out


def compare(o, ref):
    d = np.abs(o.astype(np.float64) - ref.astype(np.float64))
    return dict(maxabs=float(d.max()), p999=float(np.quantile(d, 0.999)), p99=float(np.quantile(d, 0.99)),
                mismatch=float((o != ref).mean()))
