"""Shared helpers of the GPU parity tests (imported only by tests marked `gpu`)."""
import sys

import numpy as np
import torch

import moe_workloads as wl
import paper_2510_19470_amd as moe
from paper_2510_19470_amd.layer import (MoELayer, layer_from_inputs, to_device, to_host_bits,
                                        to_host_f32)

DEV = "cuda:0"

# Tolerances (max |got - want| divided by max |want| over the tensor):
#   bf16 storage, fp32 accumulation: 2e-2 (the target stated for the path)
#   fp32 storage: 1e-4 (fp32 accumulation order vs the fp64 oracle over K <= 256 terms)
TOL = {"bf16": 2e-2, "f32": 1e-4}


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def nerr(got, want):
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    scale = np.max(np.abs(want))
    if scale == 0:
        return float(np.max(np.abs(got)))
    return float(np.max(np.abs(got - want)) / scale)


def r7_rate(got, want, rel=2e-2):
    """Fraction of the elements with |got - want| <= rel * |want| + rel * rms(want): the
    elementwise report that goes with the normalised maximum (which says nothing about the
    small elements)."""
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    if want.size == 0:
        return 1.0
    rms = float(np.sqrt(np.mean(want * want)))
    return float(np.mean(np.abs(got - want) <= rel * np.abs(want) + rel * rms))


def vals(a, dtype):
    """Stored array -> float64 values."""
    return wl.stored_to_f32(a, dtype).astype(np.float64)


def i32(t):
    return t.cpu().numpy().astype(np.int32)
