"""Helpers for the GPU parity tests: device buffers from numpy and back."""
import ctypes as C

import numpy as np
import torch

from paper_2410_08791_amd import synth

DEV = "cuda:0"


def dev_u16(a):
    """uint16 numpy -> cuda tensor holding the same bits."""
    return torch.from_numpy(np.ascontiguousarray(a).view(np.int16)).to(DEV)


def host_u16(t):
    return t.cpu().numpy().view(np.uint16)


def dev_f32(a):
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(DEV)


def rand_bf16(rng, shape, scale=1.0):
    """(bits uint16, exact values float64)"""
    bits = synth.f32_to_bf16_bits((rng.standard_normal(shape) * scale).astype(np.float32))
    return bits, synth.bf16_bits_to_f32(bits).astype(np.float64)


def bf16_vals(bits):
    return synth.bf16_bits_to_f32(bits).astype(np.float64)


def ptr(t):
    return C.c_void_p(t.data_ptr()) if t is not None else None


def stream_ptr():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def max_rel(got, ref):
    """max |got - ref| / max |ref|  (the bound the benchmark spec is quoted in)."""
    return float(np.max(np.abs(np.asarray(got, dtype=np.float64) - ref)) / np.max(np.abs(ref)))


def stack_errs(got, ref, x):
    """Errors of a stack (or layer) output `got` against the oracle's `ref`, both [T, d], for the
    input x [T, d] of that stack:
      out     = max |got - ref| / max |ref|          the bound the benchmark spec is quoted in
      contrib = max |got - ref| / max |ref - x|      the same error against what the layers ADDED to
                the residual stream -- with x ~ N(0,1) and weights ~ N(0,0.02) the identity path
                dominates max |ref|, and a badly wrong sub-block would still pass `out`
      fro     = ||got - ref||_F / ||ref - x||_F
    """
    got = np.asarray(got, dtype=np.float64).reshape(ref.shape)
    ref = np.asarray(ref, dtype=np.float64)
    x = np.asarray(x, dtype=np.float64).reshape(ref.shape)
    d = np.abs(got - ref)
    added = ref - x
    return dict(out=float(d.max() / np.abs(ref).max()), contrib=float(d.max() / np.abs(added).max()),
                fro=float(np.sqrt((d * d).sum() / (added * added).sum())))
