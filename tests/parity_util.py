"""Shared helpers of the GPU parity tests: device buffers in, oracle on the
host copy of the same bytes, bitwise comparison."""
import numpy as np
import torch

import oracle
from paper_2408_14158_amd import hfr, synth

DT = {torch.float32: (hfr.HFR_F32, oracle.F32), torch.bfloat16: (hfr.HFR_BF16, oracle.BF16),
      torch.float16: (hfr.HFR_F16, oracle.F16),
      torch.float8_e4m3fn: (hfr.HFR_FP8_E4M3, oracle.FP8_E4M3),
      torch.float8_e5m2: (hfr.HFR_FP8_E5M2, oracle.FP8_E5M2)}


def bits(arr: np.ndarray) -> np.ndarray:
    return arr.view(np.uint32) if arr.dtype == np.float32 else arr


def is_nan_bits(u: np.ndarray, f16: bool = False) -> np.ndarray:
    if u.dtype == np.uint32:
        return ((u & 0x7F800000) == 0x7F800000) & ((u & 0x007FFFFF) != 0)
    if f16:
        return ((u & 0x7C00) == 0x7C00) & ((u & 0x03FF) != 0)
    return ((u & 0x7F80) == 0x7F80) & ((u & 0x007F) != 0)


def is_nan_fp8(u: np.ndarray, fmt: str) -> np.ndarray:
    if fmt == "e4m3":
        return (u & 0x7F) == 0x7F
    return ((u & 0x7C) == 0x7C) & ((u & 0x03) != 0)


def assert_bitwise(got: np.ndarray, want: np.ndarray, what="", f16: bool = False, fp8: str = ""):
    """0 ULP: identical bit patterns, except that any NaN matches any NaN
    (f16 / fp8 tell which format uint16 / uint8 patterns are)."""
    g, w = bits(got), bits(want)
    assert g.shape == w.shape, (what, g.shape, w.shape)
    bad = g != w
    if bad.any():
        if g.dtype == np.uint8:
            bad &= ~(is_nan_fp8(g, fp8) & is_nan_fp8(w, fp8))
        else:
            bad &= ~(is_nan_bits(g, f16) & is_nan_bits(w, f16))
    if bad.any():
        i = int(np.flatnonzero(bad)[0])
        raise AssertionError("%s: %d mismatches, first at %d: got %#x want %#x"
                             % (what, int(bad.sum()), i, int(g[i]), int(w[i])))


def from_bits(arr: np.ndarray, device="cuda", f16: bool = False) -> torch.Tensor:
    """numpy float32 / uint32 bits / uint16 bits (bf16, or fp16 with f16=True)
    -> device tensor of the matching type."""
    if arr.dtype == np.float32:
        return torch.from_numpy(arr.copy()).to(device)
    if arr.dtype == np.uint32:
        return torch.from_numpy(arr.view(np.int32).copy()).view(torch.float32).to(device)
    if arr.dtype == np.uint16:
        return torch.from_numpy(arr.view(np.int16).copy()).view(torch.float16 if f16 else torch.bfloat16).to(device)
    raise TypeError(arr.dtype)


def gpu_reduce_sum(ins, out=None, stream=None):
    """Calls the C ABI on device tensors; returns the output tensor."""
    hdt, _ = DT[ins[0].dtype]
    n = ins[0].numel()
    if out is None:
        out = torch.empty_like(ins[0])
    hfr.hfr_reduce_sum(ins, len(ins), out, n, hdt, stream)
    return out


def oracle_reduce_sum(ins):
    _, odt = DT[ins[0].dtype]
    return oracle.reduce_sum([synth.as_numpy_bits(t) for t in ins], odt)


FP8_NAME = {torch.float8_e4m3fn: "e4m3", torch.float8_e5m2: "e5m2"}


def check_reduce_sum(ins, what=""):
    want = oracle_reduce_sum(ins)
    out = gpu_reduce_sum(ins)
    torch.cuda.synchronize()
    assert_bitwise(synth.as_numpy_bits(out), want, what, f16=ins[0].dtype == torch.float16,
                   fp8=FP8_NAME.get(ins[0].dtype, ""))
    return out


def make_peers(dtype, K, n, seed, device="cuda", std=1e-3):
    """K seeded peer buffers of the given torch dtype."""
    if dtype == torch.float32:
        return synth.peer_buffers_uniform_f32(K, n, seed, device)
    if dtype == torch.float16:
        return synth.peer_buffers_normal_f16(K, n, std, seed, device)
    if dtype in FP8_NAME:
        return synth.peer_buffers_normal_fp8(K, n, std, seed, FP8_NAME[dtype], device)
    return synth.peer_buffers_normal_bf16(K, n, std, seed, device)


def oracle_reduce_sum_threaded(host_ins, odt, threads=16, out=None):
    """The oracle's in-order sum of host arrays, the same single-threaded
    function called on disjoint index ranges from several host threads
    (elementwise independence: identical bits, a fraction of the wall time)."""
    from concurrent.futures import ThreadPoolExecutor
    n = len(host_ins[0])
    if out is None:
        out = np.empty(n, dtype=host_ins[0].dtype)
    bounds = [(n * t // threads, n * (t + 1) // threads) for t in range(threads)]

    def work(be):
        b, e = be
        if e > b:
            oracle.reduce_sum([a[b:e] for a in host_ins], odt, out=out[b:e])

    with ThreadPoolExecutor(max_workers=threads) as pool:
        list(pool.map(work, bounds))
    return out
