"""Shared helpers of the GPU parity tests (not collected by pytest)."""
from __future__ import annotations

import os
from concurrent.futures import ThreadPoolExecutor

import numpy as np

from oracle import attn_ref
from paper_2604_18616_amd.inputs import bf16_bits_to_f32

# Tolerances of the parity bar (stated with the benchmark definition): O within
# max-abs 2e-2 and mean-abs 2e-3 of the fp64 reference, LSE within max-abs 1e-3.
TOL_O_MAX, TOL_O_MEAN, TOL_LSE_MAX = 2e-2, 2e-3, 1e-3


def to_dev(bits: np.ndarray):
    import torch
    return torch.from_numpy(bits.view(np.int16)).view(torch.bfloat16).cuda()


def from_dev_bf16(t) -> np.ndarray:
    import torch
    return bf16_bits_to_f32(t.view(torch.int16).cpu().numpy().view(np.uint16)).astype(np.float64)


def run_hip(qb, kb, vb, causal, scale, want_lse=True, wg_rows=0):
    """Run the HIP path on bf16 bit arrays; outputs start as NaN so stale memory cannot pass.
    wg_rows: 0 = attn_fwd (the library picks the workgroup shape), 128 / 256 = attn_fwd_tile."""
    import torch
    from paper_2604_18616_amd import binding
    q, k, v = to_dev(qb), to_dev(kb), to_dev(vb)
    o = torch.full(q.shape, float("nan"), dtype=torch.bfloat16, device="cuda")
    lse = torch.full(q.shape[:3], float("nan"), dtype=torch.float32, device="cuda")
    B, Hq, Sq, D = q.shape
    _, Hkv, Sk, _ = k.shape
    rc = binding.attn_fwd_raw(q.data_ptr(), k.data_ptr(), v.data_ptr(), o.data_ptr(),
                              lse.data_ptr() if want_lse else None, B, Hq, Hkv, Sq, Sk, D,
                              causal, scale, torch.cuda.current_stream().cuda_stream, wg_rows=wg_rows)
    assert rc == 0, binding.strerror(rc)
    torch.cuda.synchronize()
    return from_dev_bf16(o), lse.cpu().numpy().astype(np.float64)


def oracle_parallel(qb, kb, vb, causal, scale, rows=None, workers=None):
    """The single-threaded reference, run on independent (batch, kv-head) slices in threads."""
    B, Hq, Sq, D = qb.shape
    _, Hkv, Sk, _ = kb.shape
    g = Hq // Hkv
    R = Sq if rows is None else np.asarray(rows).reshape(B * Hq, -1).shape[1]
    rows3 = None if rows is None else np.asarray(rows, dtype=np.int32).reshape(B, Hq, R)
    o = np.empty((B, Hq, R, D))
    lse = np.empty((B, Hq, R))

    def one(job):
        b, hk = job
        hs = slice(hk * g, (hk + 1) * g)
        r = None if rows3 is None else rows3[b, hs].reshape(g, R)
        oo, ll = attn_ref(qb[b:b + 1, hs], kb[b:b + 1, hk:hk + 1], vb[b:b + 1, hk:hk + 1], causal, scale, rows=r)
        o[b, hs], lse[b, hs] = oo[0], ll[0]

    workers = workers or min(16, os.cpu_count() or 1)
    with ThreadPoolExecutor(workers) as ex:
        list(ex.map(one, [(b, hk) for b in range(B) for hk in range(Hkv)]))
    return o, lse


def check(o_hip, lse_hip, o_ref, lse_ref, what=""):
    """Element-wise comparison at the parity bar; returns the error figures."""
    assert o_hip.shape == o_ref.shape and lse_hip.shape == lse_ref.shape, what
    assert np.isfinite(o_hip).all(), "non-finite O " + what
    err = np.abs(o_hip - o_ref)
    fin = np.isfinite(lse_ref)
    assert (lse_hip[~fin] == lse_ref[~fin]).all(), "LSE of empty rows " + what
    lerr = np.abs(lse_hip[fin] - lse_ref[fin]) if fin.any() else np.zeros(1)
    assert np.isfinite(lse_hip[fin]).all(), "non-finite LSE " + what
    res = dict(o_max=float(err.max()), o_mean=float(err.mean()), lse_max=float(lerr.max()))
    assert res["o_max"] <= TOL_O_MAX and res["o_mean"] <= TOL_O_MEAN and res["lse_max"] <= TOL_LSE_MAX, (what, res)
    return res
