"""Helpers shared by the GPU parity tests (not collected by pytest)."""
from __future__ import annotations

import numpy as np

from paper_2503_05931_amd import binding, workloads as W

# "bf16+fp8kv": bf16 arithmetic with 8-bit key / value caches.  Both sides store the same codes except where the
# kernels' bf16-level error moves a key or value element across the midpoint of two codes; such an element then
# differs by a whole code step (6-12 % of its value), which on a few per cent of the elements amounts to about as
# much as the storage rounding itself (which moves these tests' logits by 4-5e-2).
TOL = {"fp32": 1e-4, "bf16": 3e-2, "bf16+fp8kv": 1e-1}


def make_decoder(wl, max_batch=None, max_total=None, max_dec_len=None, poison=True, kv_pages=0, prefill_rows=0):
    cfg = wl.cfg
    B = len(wl.enc_lens)
    dec = binding.Decoder(cfg, wl.weights,
                          max_batch=max_batch or B,
                          max_total_enc_frames=max_total or int(wl.enc_lens.sum()),
                          max_dec_len=max_dec_len or cfg.max_dec_len, kv_pages=kv_pages, prefill_rows=prefill_rows,
                          # every byte the library has not written itself reads as NaN, so a read of an
                          # unwritten cache slot or of padding shows up in the logits
                          workspace_fill=0xFF if poison else None)
    return dec


def forced_logits_gpu(dec, wl, tokens, rows=None):
    """Teacher-forced run through aed_decode_step: tokens [B, S] -> (logits [B, S, V], argmax ids [B, S]).
    rows: keep only these sequences' logits and ids (a large batch's full logits do not fit the host)."""
    import torch
    B, S = tokens.shape
    dec.aed_cross_kv_precompute(dec.to_device(wl.enc), wl.enc_lens)
    tok_dev = torch.from_numpy(np.ascontiguousarray(tokens.T)).to(dec.device)  # [S, B]
    sel = None if rows is None else torch.as_tensor(list(rows), dtype=torch.long, device=dec.device)
    logits, ids = [], []
    for s in range(S):
        out, lg = dec.aed_decode_step(tok_dev[s].contiguous())
        logits.append(lg if sel is None else lg[sel])
        ids.append(out if sel is None else out[sel])
    torch.cuda.synchronize()
    return (torch.stack(logits, 1).cpu().numpy().astype(np.float64), torch.stack(ids, 1).cpu().numpy())


def check_forced(ref_logits, gpu_logits, gpu_ids, tol):
    """Teacher-forced comparison: every logit within tol; the GPU's argmax equals the
    oracle's wherever the oracle's top-1/top-2 margin exceeds 2*tol, and is otherwise one of the
    ids within 2*tol of the oracle's maximum.  Returns (max abs error, number of near-tie rows)."""
    err = float(np.abs(ref_logits - gpu_logits).max())
    assert np.isfinite(gpu_logits).all(), "non-finite logits from the HIP path"
    assert err <= tol, f"max |logit error| {err:.3e} > {tol}"
    top = ref_logits.max(-1)
    ref_ids = ref_logits.argmax(-1)
    srt = np.sort(ref_logits, axis=-1)
    margin = srt[..., -1] - srt[..., -2]
    clear = margin > 2 * tol
    assert (gpu_ids[clear] == ref_ids[clear]).all(), "argmax differs where the oracle's margin is clear"
    near = ~clear
    if near.any():
        picked = np.take_along_axis(ref_logits, gpu_ids[..., None].astype(np.int64), -1)[..., 0]
        assert (picked[near] >= top[near] - 2 * tol).all(), "argmax outside the near-tie set"
    return err, int(near.sum())


def first_near_tie(ref_logits, tol):
    """Per sequence: index of the first step whose top-1/top-2 margin is <= 2*tol (or S)."""
    srt = np.sort(ref_logits, axis=-1)
    margin = srt[..., -1] - srt[..., -2]
    B, S = margin.shape
    out = np.full(B, S, dtype=np.int64)
    for b in range(B):
        hit = np.where(margin[b] <= 2 * tol)[0]
        if len(hit):
            out[b] = hit[0]
    return out
