"""Shared helpers for the GPU parity tests: run a workload through the C ABI and through the oracle."""
import functools

import numpy as np

from oracle import encoder_oracle as O
from paper_2412_11272_amd import binding as wf
from paper_2412_11272_amd import synth

BF16_TOL = 2e-2      # max|gpu - oracle| / max|oracle| under bf16 MFMA with fp32 accumulation
F32_TOL = 1e-4       # same metric on the fp32 debug path


@functools.lru_cache(maxsize=32)
def inputs(name: str, affine: bool = False):
    wl = synth.workload(name)
    w, hush, mels = synth.materialize(wl, affine_random=affine)
    return wl, w, hush, mels


@functools.lru_cache(maxsize=32)
def oracle_batch(name: str, affine: bool = False):
    wl, w, hush, mels = inputs(name, affine)
    return O.encode_batch(w, wl.shape.n_heads, mels, hush if wl.hush_frames > 0 else None)


def rel_err(got: np.ndarray, ref: np.ndarray) -> float:
    return float(np.abs(got.astype(np.float64) - ref).max() / np.abs(ref).max())


def gpu_encode(name: str, precision: int, affine: bool = False, mel_dtype=None, out_dtype=None):
    import torch
    wl, w, hush, mels = inputs(name, affine)
    enc = wf.encoder_for_workload(wl, w, hush, precision)
    try:
        flat, offs, nf = wf.pack_mels(mels)
        mel = torch.from_numpy(flat).cuda()
        if mel_dtype is not None:
            mel = mel.to(mel_dtype)
        out, cu = enc.encode(mel, offs, nf, out_dtype=out_dtype)
        torch.cuda.synchronize()
        return out.float().cpu().numpy(), cu
    finally:
        enc.close()


def per_stream_report(got, ref, cu):
    rows = []
    for i in range(len(cu) - 1):
        a, b = got[cu[i]:cu[i + 1]], ref[cu[i]:cu[i + 1]]
        rows.append((i, int(cu[i + 1] - cu[i]), float(np.abs(a - b).max() / np.abs(b).max()),
                     float(np.sqrt(((a - b) ** 2).mean()))))
    return rows
