"""Helpers shared by the tests: moving a synthetic batch to the device, running the oracle
over it, and the error gates."""
import numpy as np
import torch

import oracle
from paper_2502_17421_amd import binding as ls
from paper_2502_17421_amd import synth

# max-abs bound on out: the stated targets for bf16 and f32.  f16 (11 significant bits) is not
# named by the target; its bound follows from the arithmetic: numerators rounded toward zero
# to 11 bits (all weights of a row shrink by up to 2^-10, on average 2^-11, which the fp32 row
# sum does not share), split partials and the result rounded to nearest (2^-12 each):
# <= 1e-3 of the magnitude, gated at twice that.
TOL = {"bf16": 2e-2, "f32": 1e-5, "f16": 2e-3}
LSE_TOL = {"bf16": 2e-3, "f32": 1e-5, "f16": 2e-4}


from paper_2502_17421_amd.device_batch import DeviceBatch, to_dev, torch_dtype  # noqa: F401  (re-exported)


def oracle_full(batch, rows_per_seq=None, rng=None, **kw):
    """Oracle over a batch.  rows_per_seq=None: every row, returns (out [B,Hq,T,D], lse [B,Hq,T]).
    Otherwise samples that many (head, row) pairs per sequence and returns
    (rows [B,n,2], out [B,n,D], lse [B,n])."""
    outs, lses, rows_all = [], [], []
    for s in batch.seqs:
        if rows_per_seq is None:
            o, l = oracle.attn_all(s.q, s.k_cache, s.v_cache, s.k_tree, s.v_tree, s.parents, **kw)
        else:
            hq, t, _ = s.q.shape
            flat = rng.choice(hq * t, size=min(rows_per_seq, hq * t), replace=False)
            rows = np.stack([flat // t, flat % t], axis=1).astype(np.int32)
            o, l = oracle.attn_rows(s.q, s.k_cache, s.v_cache, s.k_tree, s.v_tree, s.parents, rows=rows, **kw)
            rows_all.append(rows)
        outs.append(o)
        lses.append(l)
    if rows_per_seq is None:
        return np.stack(outs), np.stack(lses)
    return np.stack(rows_all), np.stack(outs), np.stack(lses)


def gates(got_out, got_lse, ref_out, ref_lse, dtype_name, what="", stress=False):
    """The parity bar: max-abs on out (the stated tolerance), plus the stricter self-imposed
    gates -- error relative to the largest reference magnitude, normalised RMS, and lse.

    stress=True is for the input variants built to give O(1)..O(10) outputs (not the benchmark
    recipe): there the absolute bound scales with the largest reference magnitude, because
    rounding the result to bf16 alone costs up to 2^-8 of its magnitude (0.0156 at |x| = 4)."""
    got_out = np.asarray(got_out, dtype=np.float64)
    got_lse = np.asarray(got_lse, dtype=np.float64)
    assert np.all(np.isfinite(got_out)), f"{what}: non-finite output"
    err = np.abs(got_out - ref_out)
    max_abs = float(err.max())
    scale = float(np.abs(ref_out).max())
    rms = float(np.sqrt((err ** 2).mean()) / max(np.sqrt((ref_out ** 2).mean()), 1e-30))
    lse_err = float(np.abs(got_lse - ref_lse).max())
    info = f"{what}: max_abs={max_abs:.3e} rel_to_max={max_abs / max(scale, 1e-30):.3e} nrms={rms:.3e} lse={lse_err:.3e}"
    assert max_abs <= TOL[dtype_name] * (max(1.0, scale) if stress else 1.0), info
    if dtype_name == "bf16":
        assert max_abs <= 2e-2 * max(scale, 1e-30), info
        assert rms <= 5e-3, info
    elif dtype_name == "f16":
        assert max_abs <= 2e-3 * max(scale, 1e-30), info
        assert rms <= 1e-3, info
    else:
        assert max_abs <= 1e-5 * max(1.0, scale), info
        assert rms <= 2e-6, info
    lse_scale = max(1.0, float(np.abs(ref_lse[np.isfinite(ref_lse)]).max())) if dtype_name == "f32" else 1.0
    assert lse_err <= LSE_TOL[dtype_name] * lse_scale, info
    return info
