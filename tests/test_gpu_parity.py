"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle
on the same seeded inputs.  Tolerances: fp32 mode 1e-4 absolute on logits,
bf16 mode 3e-2; token ids identical wherever the oracle's top-1/top-2 margin
exceeds twice the tolerance (otherwise one of the near-tied ids)."""
import numpy as np
import pytest

from paper_2503_05931_amd import workloads as W

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def torch_cuda():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    return torch


def unit_workload(dtype, d_model, n_heads, head_dim, enc_lens, seed, n_layers=2, d_ffn=512, vocab=256,
                  max_new=40, eos_id=-1, prompt_len=4, **kw):
    cfg = W.DecoderConfig(name="unit", n_layers=n_layers, d_model=d_model, n_heads=n_heads, head_dim=head_dim,
                          d_ffn=d_ffn, vocab=vocab, dtype=dtype, batch=len(enc_lens), prompt_len=prompt_len,
                          max_new=max_new, eos_id=eos_id, **kw)
    return W.custom(cfg, enc_lens, seed, random_ln=True)


def random_tokens(cfg, B, S, seed):
    return np.random.default_rng(seed).integers(0, cfg.vocab, size=(B, S)).astype(np.int32)


# ---------------------------------------------------------------- tiny fp32 configuration
def test_tiny_fp32_teacher_forced_and_greedy(torch_cuda, oracle):
    from tests import gpu_util as G
    wl = W.make("tiny")
    cfg = wl.cfg
    m = oracle.Model(cfg, wl.weights)
    ref_toks, ref_lens, ref_logits = m.greedy_decode(wl.enc, wl.enc_lens, wl.prompt, cfg.max_new, want_logits=True)
    dec = G.make_decoder(wl)
    # teacher-forced on the oracle's tokens
    full = np.concatenate([wl.prompt, ref_toks[:, :-1]], axis=1)
    glog, gids = G.forced_logits_gpu(dec, wl, full)
    P = cfg.prompt_len
    err, near = G.check_forced(ref_logits, glog[:, P - 1:], gids[:, P - 1:], G.TOL["fp32"])
    print(f"tiny fp32: max |dlogit| = {err:.2e}, near-tie steps = {near}")
    # cross K/V and the self cache against the oracle
    for layer in (0, cfg.n_layers - 1):
        for b in (0, len(wl.enc_lens) - 1):
            sub = wl.subset([b])
            Kr, Vr = m.cross_kv(layer, sub.enc)
            Kg, Vg = dec.aed_read_cross_kv(layer, b, int(wl.enc_lens[b]))
            assert np.abs(Kg - Kr).max() < 1e-4 and np.abs(Vg - Vr).max() < 1e-4
            Ks, Vs = dec.aed_read_self_kv(layer, b)
            Kr, Vr = m.self_kv(layer, sub.enc, full[b])
            assert Ks.shape == Kr.shape
            assert np.abs(Ks - Kr).max() < 1e-4 and np.abs(Vs - Vr).max() < 1e-4
    # free-running greedy through the captured graph
    torch = torch_cuda
    dec.aed_cross_kv_precompute(dec.to_device(wl.enc), wl.enc_lens)
    toks, lens = dec.aed_greedy_decode(torch.from_numpy(wl.prompt).to(dec.device), cfg.max_new)
    toks, lens = toks.cpu().numpy(), lens.cpu().numpy()
    assert (lens == cfg.max_new).all()
    first = G.first_near_tie(ref_logits, G.TOL["fp32"])
    for b in range(len(first)):
        assert (toks[b, :first[b]] == ref_toks[b, :first[b]]).all()
    print("tiny fp32: free-running ids identical up to step", first.tolist())
    dec.close()


# ---------------------------------------------------------------- shapes, ragged tails, page boundaries
@pytest.mark.parametrize("dtype,d_model,n_heads,head_dim,enc_lens", [
    ("fp32", 256, 4, 64, [1, 15, 16, 17, 63, 64, 65, 130]),
    ("fp32", 256, 2, 128, [3, 200, 31]),
    ("bf16", 256, 4, 64, [1, 15, 16, 17, 63, 64, 65, 130]),
    ("bf16", 512, 4, 128, [1, 2, 129, 500, 77]),
    ("bf16", 1024, 8, 128, [257, 1, 64]),
    ("bf16", 768, 12, 64, [40]),
    # more than 128 sequences: the LayerNorm runs as its own launch and the GEMMs use the large tiles
    ("bf16", 256, 4, 64, [1 + (7 * i) % 90 for i in range(150)]),
    ("fp32", 256, 4, 64, [1 + (11 * i) % 60 for i in range(131)]),
    ("bf16", 512, 4, 128, [3 + (5 * i) % 40 for i in range(300)]),
    # 512 rows and more: every projection runs on the LDS-tiled MFMA kernel (ragged last tile)
    ("bf16", 256, 4, 64, [2 + (3 * i) % 25 for i in range(530)]),
])
def test_teacher_forced_shapes(torch_cuda, oracle, dtype, d_model, n_heads, head_dim, enc_lens):
    from tests import gpu_util as G
    wl = unit_workload(dtype, d_model, n_heads, head_dim, enc_lens, seed=len(enc_lens) + d_model)
    S = 35 if len(enc_lens) < 100 else 18  # crosses the 16- (and 32-) token page boundaries
    toks = random_tokens(wl.cfg, len(enc_lens), S, 5)
    ref = oracle.Model(wl.cfg, wl.weights).decode_forced(wl.enc, wl.enc_lens, toks)
    dec = G.make_decoder(wl)
    glog, gids = G.forced_logits_gpu(dec, wl, toks)
    err, near = G.check_forced(ref, glog, gids, G.TOL[dtype])
    print(f"{dtype} d={d_model} H={n_heads}x{head_dim}: max |dlogit| = {err:.2e}, near ties {near}")
    # cross K/V of the first and the last sequence against the oracle (bf16 storage rounds the values)
    m = oracle.Model(wl.cfg, wl.weights)
    kv_tol = 1e-4 if dtype == "fp32" else 2e-2
    for b in (0, len(enc_lens) - 1):
        Kr, Vr = m.cross_kv(1, wl.subset([b]).enc)
        Kg, Vg = dec.aed_read_cross_kv(1, b, int(enc_lens[b]))
        assert np.abs(Kg - Kr).max() < kv_tol and np.abs(Vg - Vr).max() < kv_tol
    # determinism: a second run is bit-identical
    glog2, gids2 = G.forced_logits_gpu(dec, wl, toks)
    assert (glog2 == glog).all() and (gids2 == gids).all()
    # the paged self-attention cache (S positions cross one or two page boundaries) against the oracle's keys and
    # values of the fed tokens: a wrong page, slot or head offset in the append shows here
    for b in (0, len(enc_lens) - 1):
        Kr, Vr = m.self_kv(1, wl.subset([b]).enc, toks[b])
        Ks, Vs = dec.aed_read_self_kv(1, b)
        assert Ks.shape == (S, d_model) and np.isfinite(Ks).all() and np.isfinite(Vs).all()
        assert np.abs(Ks - Kr).max() <= G.TOL[dtype] and np.abs(Vs - Vr).max() <= G.TOL[dtype]
    dec.close()


@pytest.mark.parametrize("d_model,n_heads,head_dim,batch,norm_type", [
    (512, 4, 128, 1750, 0),   # QKV product: 14 x 12 tiles of 128 x 128, K = 512 -> direct-to-LDS 128-tile kernel
    (256, 4, 64, 3500, 0),    # QKV product: 28 x 6 tiles, K = 256 -> register-staged 128-tile kernel
    (512, 4, 128, 1750, 1),   # the same two kernels with RMSNorm folded around the products
    (256, 4, 64, 3500, 1),
])
def test_very_large_batches_tiled_projections(torch_cuda, oracle, d_model, n_heads, head_dim, batch, norm_type):
    """Batches large enough for the 128 x 128 tiled kernels to take the QKV product, the normalisation folded
    around it (ragged last row tile); a few teacher-forced steps against the oracle."""
    from tests import gpu_util as G
    enc_lens = [1 + (5 * i) % 7 for i in range(batch)]
    wl = unit_workload("bf16", d_model, n_heads, head_dim, enc_lens, seed=batch, max_new=8, norm_type=norm_type)
    toks = random_tokens(wl.cfg, batch, 4, 6)
    ref = oracle.Model(wl.cfg, wl.weights).decode_forced(wl.enc, wl.enc_lens, toks)
    dec = G.make_decoder(wl)
    glog, gids = G.forced_logits_gpu(dec, wl, toks)
    err, near = G.check_forced(ref, glog, gids, G.TOL["bf16"])
    print(f"batch {batch}, d={d_model}: max |dlogit| = {err:.2e}, near ties {near}")
    dec.close()


def test_wide_ffn_large_batch_row_fastest_tiles(torch_cuda, oracle):
    """700 rows against a 4 096-wide first FFN product: 6 x 32 tiles of 128 x 128 on the direct-to-LDS kernel, which
    then numbers its tiles row-fastest (an XCD's run of 24 tiles = all 6 row panels x 4 column panels), with a
    ragged last row tile (60 rows)."""
    from tests import gpu_util as G
    batch = 700
    enc_lens = [1 + (3 * i) % 5 for i in range(batch)]
    wl = unit_workload("bf16", 512, 4, 128, enc_lens, seed=batch, max_new=8, d_ffn=4096)
    toks = random_tokens(wl.cfg, batch, 3, 8)
    ref = oracle.Model(wl.cfg, wl.weights).decode_forced(wl.enc, wl.enc_lens, toks)
    dec = G.make_decoder(wl)
    glog, gids = G.forced_logits_gpu(dec, wl, toks)
    err, near = G.check_forced(ref, glog, gids, G.TOL["bf16"])
    print(f"batch {batch}, d_ffn 4096: max |dlogit| = {err:.2e}, near ties {near}")
    dec.close()


def test_split_chunks_and_capacity_slack(torch_cuda, oracle):
    """Few long sequences: the work lists cut keys into several chunks per (sequence, head) and
    the last-arriver merge runs; capacities larger than the batch leave unused slots poisoned."""
    from tests import gpu_util as G
    wl = unit_workload("bf16", 256, 4, 64, [500, 300], seed=77, max_new=140)
    S = 140
    toks = random_tokens(wl.cfg, 2, S, 6)
    ref = oracle.Model(wl.cfg, wl.weights).decode_forced(wl.enc, wl.enc_lens, toks)
    dec = G.make_decoder(wl, max_batch=5, max_total=1500, max_dec_len=160)
    glog, gids = G.forced_logits_gpu(dec, wl, toks)
    err, near = G.check_forced(ref, glog, gids, G.TOL["bf16"])
    print(f"split-K case: max |dlogit| = {err:.2e}")
    dec.close()


@pytest.mark.parametrize("dtype,n_short", [("fp32", 2), ("bf16", 2), ("bf16", 31)])
def test_longest_and_shortest_sequence_in_one_batch(torch_cuda, oracle, dtype, n_short):
    """The most frames the library takes for one sequence (65 535: key offsets and counts are 16-bit fields of a
    cross-attention work item) next to sequences of a single frame.  With 3 sequences the long one is cut into the
    largest number of chunks and merged; with 32 (x 4 heads: enough work items not to cut) it is one work item of
    65 535 keys.  One frame more is refused before anything is launched."""
    from tests import gpu_util as G
    from paper_2503_05931_amd import binding
    lens = [1, 65535] + [1] * (n_short - 1)
    wl = unit_workload(dtype, 256, 4, 64, lens, seed=88, max_new=8)
    S = 6
    toks = random_tokens(wl.cfg, len(lens), S, 12)
    ref = oracle.Model(wl.cfg, wl.weights).decode_forced(wl.enc, wl.enc_lens, toks)
    dec = G.make_decoder(wl)
    glog, gids = G.forced_logits_gpu(dec, wl, toks)
    err, near = G.check_forced(ref, glog, gids, G.TOL[dtype])
    print(f"65 535 frames, {dtype}: max |dlogit| = {err:.2e}")
    k_ref, v_ref = oracle.Model(wl.cfg, wl.weights).cross_kv(1, wl.subset([1]).enc)
    k_gpu, v_gpu = dec.aed_read_cross_kv(1, 1, 65535)
    tol_kv = 1e-5 if dtype == "fp32" else 2e-2
    assert np.abs(k_gpu - k_ref).max() <= tol_kv and np.abs(v_gpu - v_ref).max() <= tol_kv
    with pytest.raises(binding.AedError) as ei:
        dec.aed_cross_kv_precompute(dec.to_device(wl.enc), [1, 65536] + [1] * (n_short - 1))
    assert ei.value.status == binding.AED_EUNSUPPORTED
    dec.close()


@pytest.mark.parametrize("dtype", ["fp32", "bf16"])
def test_long_decode_many_self_chunks(torch_cuda, oracle, dtype):
    """A decode of 1 100 positions for a batch of two: the paged self-attention cache grows to 69 pages per sequence and
    is read in the largest number of chunks (the small batch has its long sequences cut), merged by the last arriver."""
    from tests import gpu_util as G
    S = 1100
    wl = unit_workload(dtype, 256, 4, 64, [40, 9], seed=91, max_new=S - 4)
    toks = random_tokens(wl.cfg, 2, S, 13)
    m = oracle.Model(wl.cfg, wl.weights)
    ref = m.decode_forced(wl.enc, wl.enc_lens, toks)
    dec = G.make_decoder(wl)
    glog, gids = G.forced_logits_gpu(dec, wl, toks)
    err, near = G.check_forced(ref, glog, gids, G.TOL[dtype])
    print(f"{S} positions, {dtype}: max |dlogit| = {err:.2e}, near ties {near}")
    Kr, Vr = m.self_kv(1, wl.subset([1]).enc, toks[1])
    Ks, Vs = dec.aed_read_self_kv(1, 1)
    assert Ks.shape == (S, 256)
    assert np.abs(Ks - Kr).max() <= G.TOL[dtype] and np.abs(Vs - Vr).max() <= G.TOL[dtype]
    dec.close()


def test_padded_entry_point_equals_packed(torch_cuda, oracle):
    from tests import gpu_util as G
    torch = torch_cuda
    wl = unit_workload("bf16", 256, 4, 64, [5, 33, 1, 18], seed=9)
    toks = random_tokens(wl.cfg, 4, 6, 7)
    dec = G.make_decoder(wl)
    glog, _ = G.forced_logits_gpu(dec, wl, toks)
    T_max = 40
    pad = np.full((4, T_max, 256), np.nan, np.float32)   # poisoned padding rows
    off = wl.enc_offsets
    for b in range(4):
        pad[b, :wl.enc_lens[b]] = wl.enc[off[b]:off[b + 1]]
    dec.aed_cross_kv_precompute_padded(dec.to_device(pad), wl.enc_lens)
    tok_dev = torch.from_numpy(np.ascontiguousarray(toks.T)).to(dec.device)
    rows = []
    for s in range(toks.shape[1]):
        _, lg = dec.aed_decode_step(tok_dev[s].contiguous())
        rows.append(lg)
    plog = torch.stack(rows, 1).cpu().numpy().astype(np.float64)
    assert np.isfinite(plog).all() and (plog == glog).all()
    dec.close()


# ---------------------------------------------------------------- greedy semantics on the device
def test_greedy_eos_forced_eos_and_padding(torch_cuda, oracle):
    from tests import gpu_util as G
    torch = torch_cuda
    wl0 = unit_workload("fp32", 256, 4, 64, [9, 30, 4, 17, 52], seed=21, max_new=24)
    m0 = oracle.Model(wl0.cfg, wl0.weights)
    free, _ = m0.greedy_decode(wl0.enc, wl0.enc_lens, wl0.prompt, 24)
    eos = int(free[1, 5])                      # sequence 1 emits this id at step 5
    wl = unit_workload("fp32", 256, 4, 64, [9, 30, 4, 17, 52], seed=21, max_new=24, eos_id=eos, pad_id=7)
    m = oracle.Model(wl.cfg, wl.weights)
    target = np.array([3, 24, 1, 12, 30], np.int32)
    ref_t, ref_l, ref_logits = m.greedy_decode(wl.enc, wl.enc_lens, wl.prompt, 24, max_new_per_seq=target,
                                               want_logits=True)
    dec = G.make_decoder(wl)
    dec.aed_cross_kv_precompute(dec.to_device(wl.enc), wl.enc_lens)
    toks, lens = dec.aed_greedy_decode(torch.from_numpy(wl.prompt).to(dec.device), 24, max_new_per_seq=target)
    toks, lens = toks.cpu().numpy(), lens.cpu().numpy()
    first = G.first_near_tie(ref_logits[:, :], G.TOL["fp32"])
    for b in range(5):
        if first[b] >= ref_l[b]:               # no near-tie before this sequence ended: everything is fixed
            assert lens[b] == ref_l[b]
            assert (toks[b] == ref_t[b]).all()  # includes the pad_id tail
    assert lens[2] == 1 and toks[2, 0] == eos and (toks[2, 1:] == 7).all()
    assert (lens <= np.minimum(target, 24)).all()
    # the same decoder, second call without per-sequence limits
    ref_t2, ref_l2 = m.greedy_decode(wl.enc, wl.enc_lens, wl.prompt, 24)
    toks2, lens2 = dec.aed_greedy_decode(torch.from_numpy(wl.prompt).to(dec.device), 24)
    for b in range(5):
        if first[b] >= ref_l2[b]:
            assert lens2.cpu().numpy()[b] == ref_l2[b] and (toks2.cpu().numpy()[b] == ref_t2[b]).all()
    dec.close()


def test_error_paths_on_device(torch_cuda):
    from tests import gpu_util as G
    from paper_2503_05931_amd import binding
    torch = torch_cuda
    wl = unit_workload("bf16", 256, 4, 64, [5, 6], seed=3, max_new=12)
    dec = G.make_decoder(wl, max_batch=2, max_total=20, max_dec_len=16, kv_pages=3)
    tok = torch.zeros(2, dtype=torch.int32, device=dec.device)
    prompt = torch.from_numpy(wl.prompt).to(dec.device)

    def status(fn):
        with pytest.raises(binding.AedError) as ei:
            fn()
        return ei.value.status

    dec.batch = 2
    assert status(lambda: dec.aed_decode_step(tok)) == binding.AED_ESTATE
    assert status(lambda: dec.aed_greedy_decode(prompt, 4)) == binding.AED_ESTATE
    enc = dec.to_device(wl.enc)
    assert status(lambda: dec.aed_cross_kv_precompute(enc, [5, 0])) == binding.AED_EINVAL
    assert status(lambda: dec.aed_cross_kv_precompute(enc, [5, 6, 1])) == binding.AED_ECAPACITY
    assert status(lambda: dec.aed_cross_kv_precompute(enc, [15, 6])) == binding.AED_ECAPACITY
    dec.aed_cross_kv_precompute(enc, wl.enc_lens)
    assert status(lambda: dec.aed_greedy_decode(prompt, 13)) == binding.AED_ECAPACITY      # 4 + 13 > 16
    assert status(lambda: dec.aed_greedy_decode(prompt, 4, max_new_per_seq=[2, 2])) == binding.AED_EINVAL  # eos off
    assert status(lambda: dec.aed_greedy_decode(prompt, 0)) == binding.AED_EINVAL
    # page pool of 3 pages: two sequences need one page each for 16 positions, the 17th position has no page
    for _ in range(16):
        dec.aed_decode_step(tok, want_logits=False)
    assert status(lambda: dec.aed_decode_step(tok)) == binding.AED_ECAPACITY
    dec.aed_cross_kv_precompute(enc, wl.enc_lens)
    toks, lens = dec.aed_greedy_decode(prompt, 12)          # still usable after the errors
    assert (lens.cpu().numpy() == 12).all()
    assert status(lambda: dec.aed_decode_step(tok)) == binding.AED_ESTATE   # greedy consumed the batch
    dec.close()
    # a pool too small for the batch
    dec = G.make_decoder(wl, max_batch=2, max_total=20, max_dec_len=32, kv_pages=3)
    dec.aed_cross_kv_precompute(dec.to_device(wl.enc), wl.enc_lens)
    assert status(lambda: dec.aed_greedy_decode(prompt, 20)) == binding.AED_ECAPACITY       # 2 x 2 pages > 3
    dec.close()


def test_tiled_mfma_cross_kv_precompute(torch_cuda, oracle):
    """Enough encoder frames (2131 x 2048 outputs = 272 tiles of 128 x 128) for the LDS-tiled MFMA kernel,
    with a ragged last row tile; K and V of every sequence against the oracle, then a few decode steps."""
    from tests import gpu_util as G
    enc_lens = [500, 500, 500, 500, 131]
    wl = unit_workload("bf16", 1024, 8, 128, enc_lens, seed=91, n_layers=1, d_ffn=256, vocab=64, max_new=8)
    m = oracle.Model(wl.cfg, wl.weights)
    toks = random_tokens(wl.cfg, 5, 6, 8)
    ref = m.decode_forced(wl.enc, wl.enc_lens, toks)
    dec = G.make_decoder(wl)
    glog, gids = G.forced_logits_gpu(dec, wl, toks)
    for b in range(5):
        Kr, Vr = m.cross_kv(0, wl.subset([b]).enc)
        Kg, Vg = dec.aed_read_cross_kv(0, b, enc_lens[b])
        assert np.abs(Kg - Kr).max() < 2e-2 and np.abs(Vg - Vr).max() < 2e-2
    err, near = G.check_forced(ref, glog, gids, G.TOL["bf16"])
    print(f"tiled cross K/V: max |dlogit| = {err:.2e}")
    dec.close()


@pytest.mark.parametrize("d_model,n_heads,head_dim,enc_lens", [
    (1024, 8, 128, [700] * 7 + [411]),      # 5 311 frames: 21 row tiles (the last one ragged) x 8 column tiles of 256
    (1024, 16, 64, [900] * 5 + [677]),      # K = 1024 with heads of 64: two heads per 128-column wavefront tile
    (512, 8, 64, [1300] * 7 + [1150]),      # 10 250 frames: 41 x 4 tiles, one head per 64 columns
    (768, 12, 64, [1000] * 7 + [77]),       # 7 077 frames, K = 768 (24 k-steps of 32): 28 x 6 tiles
    (768, 12, 64, [500] * 7),               # 3 500 frames: too few 256-tiles, 28 x 12 tiles of 128 x 128 instead
])
def test_direct_to_lds_cross_kv_precompute(torch_cuda, oracle, d_model, n_heads, head_dim, enc_lens):
    """Enough frames for the persistent 256 x 256 kernel that loads its operands straight into LDS
    (at least 160 tiles): K and V of every sequence against the oracle, then a few decode steps."""
    from tests import gpu_util as G
    wl = unit_workload("bf16", d_model, n_heads, head_dim, enc_lens, seed=93, n_layers=1, d_ffn=256, vocab=64, max_new=8)
    m = oracle.Model(wl.cfg, wl.weights)
    B = len(enc_lens)
    toks = random_tokens(wl.cfg, B, 4, 9)
    ref = m.decode_forced(wl.enc, wl.enc_lens, toks)
    dec = G.make_decoder(wl)
    glog, gids = G.forced_logits_gpu(dec, wl, toks)
    worst = 0.0
    for b in range(B):
        Kr, Vr = m.cross_kv(0, wl.subset([b]).enc)
        Kg, Vg = dec.aed_read_cross_kv(0, b, enc_lens[b])
        assert np.isfinite(Kg).all() and np.isfinite(Vg).all()
        worst = max(worst, float(np.abs(Kg - Kr).max()), float(np.abs(Vg - Vr).max()))
    assert worst < 2e-2, f"cross K/V differs by {worst}"
    err, near = G.check_forced(ref, glog, gids, G.TOL["bf16"])
    print(f"direct-to-LDS cross K/V (d {d_model}, head_dim {head_dim}): max |dK,dV| = {worst:.2e}, max |dlogit| = {err:.2e}")
    dec.close()


def test_folded_layernorm_with_a_large_row_mean(torch_cuda, oracle):
    """bf16 mode rounds (x - mu_hat) * g, not LN(x), to bf16 (the LayerNorm is folded around the products), which
    is only as accurate if mu_hat stays close to the row mean.  Rows with a common offset of 8 standard deviations
    (embeddings shifted by a constant) would cost 8x the rounding error with mu_hat = 0; with the previous update's
    mean as mu_hat the logits must stay inside the usual tolerance."""
    from tests import gpu_util as G
    wl = unit_workload("bf16", 512, 4, 128, [40, 7, 130, 64, 1, 99], seed=57, n_layers=3, d_ffn=1024, vocab=256, max_new=12)
    w = wl.weights
    scale = float(wl.cfg.emb_scale)
    sd = float(np.std(scale * w["tok_emb"]))
    w["pos_emb"] = W.bf16_round((w["pos_emb"] + 8.0 * sd).astype(np.float32))
    m = oracle.Model(wl.cfg, w)
    toks = random_tokens(wl.cfg, 6, 10, 58)
    ref = m.decode_forced(wl.enc, wl.enc_lens, toks)
    dec = G.make_decoder(wl)
    glog, gids = G.forced_logits_gpu(dec, wl, toks)
    err, near = G.check_forced(ref, glog, gids, G.TOL["bf16"])
    print(f"rows with mean = 8 sigma: max |dlogit| = {err:.2e}, near ties {near}")
    dec.close()


@pytest.mark.parametrize("dtype,prompt_len,prefill_rows", [
    ("fp32", 6, 16 * 8),     # all five positions before the last in one pass (batch 5 -> 16 rows per position)
    ("fp32", 6, 16 * 2),     # two positions per pass: three passes
    ("bf16", 11, 16 * 4),    # bf16 (LayerNorm folded around the products), ten positions in passes of four
    ("fp32", 1, 16 * 8),     # a one-token prompt has nothing to prefill
])
def test_prompt_prefill_gives_the_same_tokens(torch_cuda, oracle, dtype, prompt_len, prefill_rows):
    """Greedy decoding with the prompt positions before the last going through the layers together: tokens as the
    oracle's (which feeds the prompt one position at a time) up to each sequence's first near-tie, self-attention
    keys and values of the prompt positions as after token-by-token feeding."""
    from tests import gpu_util as G
    torch = torch_cuda
    enc_lens = [33, 7, 130, 64, 1]
    wl = unit_workload(dtype, 256, 4, 64, enc_lens, seed=71, max_new=20, prompt_len=prompt_len)
    m = oracle.Model(wl.cfg, wl.weights)
    ref_t, ref_l, ref_logits = m.greedy_decode(wl.enc, wl.enc_lens, wl.prompt, 20, want_logits=True)
    first = G.first_near_tie(ref_logits, G.TOL[dtype])
    outs = {}
    for rows in (0, prefill_rows):
        dec = G.make_decoder(wl, prefill_rows=rows)
        dec.aed_cross_kv_precompute(dec.to_device(wl.enc), wl.enc_lens)
        toks, lens = dec.aed_greedy_decode(torch.from_numpy(wl.prompt).to(dec.device), 20)
        toks, lens = toks.cpu().numpy(), lens.cpu().numpy()
        assert (lens == 20).all()
        for b in range(len(enc_lens)):
            assert (toks[b, :first[b]] == ref_t[b, :first[b]]).all(), f"prefill_rows {rows}: sequence {b} differs"
        kv = [dec.aed_read_self_kv(1, b) for b in (0, len(enc_lens) - 1)]
        outs[rows] = (toks, kv)
        dec.close()
    tol = 1e-5 if dtype == "fp32" else 4e-2
    for (k0, v0), (k1, v1) in zip(outs[0][1], outs[prefill_rows][1]):
        P = prompt_len
        assert np.isfinite(k1).all() and np.isfinite(v1).all()
        assert np.abs(k0[:P] - k1[:P]).max() <= tol and np.abs(v0[:P] - v1[:P]).max() <= tol
    print(f"prefill {dtype} P={prompt_len} rows={prefill_rows}: tokens as the oracle's up to step {first.tolist()}")


def test_degenerate_shapes_and_reuse(torch_cuda, oracle):
    """Batch of one, one-token prompt, one new token, a decode length that ends exactly on a page boundary,
    EOS as the very first token, repeated greedy calls of different lengths on one batch (the launch graph is
    re-captured), and the step API after a new precompute."""
    from tests import gpu_util as G
    torch = torch_cuda
    tol = G.TOL["fp32"]
    wl = unit_workload("fp32", 256, 4, 64, [23], seed=41, max_new=31, prompt_len=1)   # 1 + 31 = 32 = two full pages
    cfg = wl.cfg
    m = oracle.Model(cfg, wl.weights)
    dec = G.make_decoder(wl)
    enc = dec.to_device(wl.enc)
    prompt = torch.from_numpy(wl.prompt).to(dec.device)
    assert wl.prompt.shape == (1, 1)
    for n_new in (1, 31, 16, 31):
        ref_t, ref_l, ref_logits = m.greedy_decode(wl.enc, wl.enc_lens, wl.prompt, n_new, want_logits=True)
        dec.aed_cross_kv_precompute(enc, wl.enc_lens)
        toks, lens = dec.aed_greedy_decode(prompt, n_new)
        toks, lens = toks.cpu().numpy(), lens.cpu().numpy()
        first = G.first_near_tie(ref_logits, tol)[0]
        assert lens[0] == n_new and (toks[0, :first] == ref_t[0, :first]).all()
    # the cache is exactly full: one more position has no room
    from paper_2503_05931_amd import binding
    with pytest.raises(binding.AedError) as ei:
        dec.aed_greedy_decode(prompt, 32)
    assert ei.value.status == binding.AED_ECAPACITY
    dec.close()
    # EOS as the first emitted token of one sequence: length 1, the rest padding, the other sequence unaffected
    wl0 = unit_workload("fp32", 256, 4, 64, [9, 14], seed=42, max_new=6)
    free, _ = oracle.Model(wl0.cfg, wl0.weights).greedy_decode(wl0.enc, wl0.enc_lens, wl0.prompt, 6)
    eos = int(free[0, 0])
    wl1 = unit_workload("fp32", 256, 4, 64, [9, 14], seed=42, max_new=6, eos_id=eos, pad_id=1)
    ref_t, ref_l, ref_logits = oracle.Model(wl1.cfg, wl1.weights).greedy_decode(wl1.enc, wl1.enc_lens, wl1.prompt, 6,
                                                                               want_logits=True)
    dec = G.make_decoder(wl1)
    dec.aed_cross_kv_precompute(dec.to_device(wl1.enc), wl1.enc_lens)
    toks, lens = dec.aed_greedy_decode(torch.from_numpy(wl1.prompt).to(dec.device), 6)
    toks, lens = toks.cpu().numpy(), lens.cpu().numpy()
    assert ref_l[0] == 1
    first = G.first_near_tie(ref_logits[:, :1], tol)
    if first[0] >= 1:
        assert lens[0] == 1 and toks[0, 0] == eos and (toks[0, 1:] == 1).all()
    # step API on a fresh precompute after greedy: teacher-forced logits still match
    S = 5
    tk = random_tokens(wl1.cfg, 2, S, 3)
    ref = oracle.Model(wl1.cfg, wl1.weights).decode_forced(wl1.enc, wl1.enc_lens, tk)
    glog, gids = G.forced_logits_gpu(dec, wl1, tk)
    G.check_forced(ref, glog, gids, tol)
    dec.close()


def test_same_shape_other_lengths_on_one_decoder(torch_cuda, oracle):
    """Two batches on one decoder with the same batch size, the same number of work items and the same total of
    encoder frames, but the lengths in another order: the launch graphs recorded for the first batch are replayed for
    the second (their shape is the same) and must find the second batch's work list and offsets."""
    from tests import gpu_util as G
    torch = torch_cuda
    lens_a, lens_b = [90, 20, 55, 7], [20, 7, 90, 55]
    wl_a = unit_workload("bf16", 256, 4, 64, lens_a, seed=61, max_new=12)
    wl_b = unit_workload("bf16", 256, 4, 64, lens_b, seed=61, max_new=12)   # same weights (same seed and shapes)
    for k in ("tok_emb", "w_out"):
        assert np.array_equal(wl_a.weights[k], wl_b.weights[k])
    dec = G.make_decoder(wl_a)
    for wl in (wl_a, wl_b, wl_a):
        m = oracle.Model(wl.cfg, wl.weights)
        ref_t, ref_l, ref_logits = m.greedy_decode(wl.enc, wl.enc_lens, wl.prompt, 12, want_logits=True)
        dec.aed_cross_kv_precompute(dec.to_device(wl.enc), wl.enc_lens)
        toks, lens = dec.aed_greedy_decode(torch.from_numpy(wl.prompt).to(dec.device), 12)
        toks = toks.cpu().numpy()
        first = G.first_near_tie(ref_logits, G.TOL["bf16"])
        for b in range(4):
            assert (toks[b, :first[b]] == ref_t[b, :first[b]]).all(), f"sequence {b} forks before a near tie"
        # and teacher-forced through the step path (its own recorded graph), every logit
        forced = np.concatenate([wl.prompt, ref_t[:, :-1]], axis=1)
        glog, gids = G.forced_logits_gpu(dec, wl, forced)
        P = wl.cfg.prompt_len
        G.check_forced(ref_logits, glog[:, P - 1:], gids[:, P - 1:], G.TOL["bf16"])
    dec.close()


# ---------------------------------------------------------------- exact ties in the sampler
@pytest.mark.parametrize("dtype", ["fp32", "bf16"])
@pytest.mark.parametrize("lo,hi", [
    (8, 200),      # two lanes of the sampler's first wavefront
    (8, 1032),     # one thread's first and second 4-vector
    (600, 1030),   # the lower id sits in the third wavefront, the higher one in the first
    (255, 256),    # neighbours across a wavefront boundary
    (1023, 1024),  # last id of the last wavefront's first round, first id of the first wavefront's second round
])
def test_exact_ties_pick_the_lowest_id(torch_cuda, oracle, dtype, lo, hi):
    """Two vocabulary rows with identical weights and bias give bit-equal logits; raised above all others they tie
    for the maximum at every step.  The sampler must return the lower id (as the oracle's argmax does), wherever
    the two ids sit in its reduction: in one thread, in one wavefront, in different wavefronts."""
    from tests import gpu_util as G
    torch = torch_cuda
    wl = unit_workload(dtype, 256, 4, 64, [9, 30, 4], seed=31, vocab=2048, max_new=6)
    w = wl.weights
    w["w_out"][hi] = w["w_out"][lo]
    w["b_out"][lo] = w["b_out"][hi] = 10.0   # random logits of this model stay below 2
    m = oracle.Model(wl.cfg, w)
    toks = random_tokens(wl.cfg, 3, 5, 32)
    ref = m.decode_forced(wl.enc, wl.enc_lens, toks)
    assert (ref[..., lo] == ref[..., hi]).all() and (ref.argmax(-1) == lo).all()   # numpy's argmax: first maximum
    for b in range(3):
        for s in range(5):
            assert oracle.argmax(ref[b, s]) == lo
    dec = G.make_decoder(wl)
    glog, gids = G.forced_logits_gpu(dec, wl, toks)
    assert (glog[..., lo] == glog[..., hi]).all(), "equal rows of the output matrix give unequal logits"
    assert (glog.argmax(-1) == lo).all()
    assert (gids == lo).all(), f"sampler picked {np.unique(gids).tolist()} on a tie of {lo} and {hi}"
    # the greedy path's sampler (prompt feeding, output writes) on the same tie
    dec.aed_cross_kv_precompute(dec.to_device(wl.enc), wl.enc_lens)
    out, lens = dec.aed_greedy_decode(torch.from_numpy(wl.prompt).to(dec.device), 6)
    assert (out.cpu().numpy() == lo).all() and (lens.cpu().numpy() == 6).all()
    dec.close()


# ---------------------------------------------------------------- bf16 logits while sequences finish
def test_bf16_logits_through_finished_and_forced_eos(torch_cuda, oracle):
    """Greedy decoding in bf16 mode with a natural EOS and per-sequence forced ends: the logits of every step,
    read back after greedy runs of 1, 2, ... tokens (a run of n tokens ends with step n's logits in place), against
    the oracle's greedy logits, for every sequence still running at that step and as long as its tokens have
    followed the oracle's.  Finished sequences stay in the batch: their rows go through the products but append
    nothing, attend to nothing and emit padding."""
    from tests import gpu_util as G
    torch = torch_cuda
    tol = G.TOL["bf16"]
    N = 20
    lens_enc = [9, 30, 4, 17, 52, 130]
    wl0 = unit_workload("bf16", 256, 4, 64, lens_enc, seed=23, max_new=N)
    free, _ = oracle.Model(wl0.cfg, wl0.weights).greedy_decode(wl0.enc, wl0.enc_lens, wl0.prompt, N)
    s_eos = next(s for s in range(4, N) if free[1, s] not in free[1, :s])
    eos = int(free[1, s_eos])                  # sequence 1 emits this id for the first time at step s_eos >= 4
    wl = unit_workload("bf16", 256, 4, 64, lens_enc, seed=23, max_new=N, eos_id=eos, pad_id=5)
    m = oracle.Model(wl.cfg, wl.weights)
    target = np.array([3, N, 1, 12, 30, 8], np.int32)
    ref_t, ref_l, ref_logits = m.greedy_decode(wl.enc, wl.enc_lens, wl.prompt, N, max_new_per_seq=target,
                                               want_logits=True)
    assert ref_l[1] == s_eos + 1 and ref_l[2] == 1 and ref_l[0] <= 3
    dec = G.make_decoder(wl)
    prompt = torch.from_numpy(wl.prompt).to(dec.device)
    B = len(lens_enc)
    follows = np.ones(B, bool)     # the GPU's tokens have equalled the oracle's so far
    worst, compared = 0.0, 0
    for n in range(1, N + 1):
        dec.aed_cross_kv_precompute(dec.to_device(wl.enc), wl.enc_lens)
        toks, lens = dec.aed_greedy_decode(prompt, n, max_new_per_seq=target)
        toks, lens = toks.cpu().numpy(), lens.cpu().numpy()
        lg = dec.aed_read_logits().astype(np.float64)
        if (ref_l < n).all():
            break                  # every sequence had finished before step n: the run stopped early
        for b in range(B):
            if ref_l[b] < n or not follows[b]:
                continue           # finished before this step (row unspecified), or on another path
            e = float(np.abs(lg[b] - ref_logits[b, n - 1]).max())
            worst, compared = max(worst, e), compared + 1
            assert e <= tol, f"step {n}, sequence {b}: |dlogit| {e:.3e}"
            srt = np.sort(ref_logits[b, n - 1])
            forced = n >= target[b]
            if forced:
                assert toks[b, n - 1] == eos
            elif srt[-1] - srt[-2] > 2 * tol:
                assert toks[b, n - 1] == ref_t[b, n - 1]
            follows[b] = toks[b, n - 1] == ref_t[b, n - 1]
            if ref_l[b] == n and follows[b]:
                assert lens[b] == n
    assert compared >= 30
    print(f"bf16 greedy logits with finished rows in the batch: {compared} rows compared, max |dlogit| = {worst:.3e}")
    dec.close()


# ---------------------------------------------------------------- RMSNorm variant (norm_type = 1)
@pytest.mark.parametrize("dtype,d_model,n_heads,head_dim,enc_lens,shifts", [
    ("fp32", 256, 4, 64, [1, 15, 16, 17, 63, 64, 65, 130], True),
    ("bf16", 256, 4, 64, [1, 15, 16, 17, 63, 64, 65, 130], True),
    ("bf16", 1024, 8, 128, [257, 1, 64], False),               # no shift vectors (NULL pointers)
    ("fp32", 256, 4, 64, [1 + (11 * i) % 60 for i in range(131)], False),   # the normalisation as its own launch
    ("bf16", 512, 4, 128, [3 + (5 * i) % 40 for i in range(300)], True),    # large tiles, folded normalisation
    ("bf16", 256, 4, 64, [2 + (3 * i) % 25 for i in range(530)], True),     # LDS-tiled kernels
])
def test_rmsnorm_teacher_forced(torch_cuda, oracle, dtype, d_model, n_heads, head_dim, enc_lens, shifts):
    """Every normalisation of the decoder as RMSNorm (no mean subtraction): teacher-forced logits against the
    oracle in both modes, embeddings shifted so that the rows' means are far from zero (a LayerNorm in any of the
    places would give other logits), and the greedy path with prompt prefill."""
    from tests import gpu_util as G
    torch = torch_cuda
    wl = unit_workload(dtype, d_model, n_heads, head_dim, enc_lens, seed=len(enc_lens) + d_model + 1, norm_type=1,
                       max_new=28)
    w = wl.weights
    w["pos_emb"] = W.bf16_round((w["pos_emb"] + 0.05).astype(np.float32)) if dtype == "bf16" else (w["pos_emb"] + 0.05).astype(np.float32)
    if not shifts:
        w["lnf_b"] = None
        for l in w["layers"]:
            l["ln1_b"] = l["ln2_b"] = l["ln3_b"] = None
    S = 20 if len(enc_lens) < 100 else 6
    toks = random_tokens(wl.cfg, len(enc_lens), S, 5)
    m = oracle.Model(wl.cfg, w)
    ref = m.decode_forced(wl.enc, wl.enc_lens, toks)
    import copy
    cfg_ln = copy.copy(wl.cfg)
    cfg_ln.norm_type = 0
    if shifts:
        assert np.abs(oracle.Model(cfg_ln, w).decode_forced(wl.enc[:int(wl.enc_lens[0])], wl.enc_lens[:1], toks[:1]) - ref[:1]).max() > 10 * G.TOL[dtype]
    dec = G.make_decoder(wl, prefill_rows=16 * ((len(enc_lens) + 15) // 16) if len(enc_lens) < 100 else 0)
    glog, gids = G.forced_logits_gpu(dec, wl, toks)
    err, near = G.check_forced(ref, glog, gids, G.TOL[dtype])
    print(f"RMSNorm {dtype} d={d_model} B={len(enc_lens)}: max |dlogit| = {err:.2e}, near ties {near}")
    if len(enc_lens) < 100:
        ref_t, ref_l, ref_logits = m.greedy_decode(wl.enc, wl.enc_lens, wl.prompt, 12, want_logits=True)
        dec.aed_cross_kv_precompute(dec.to_device(wl.enc), wl.enc_lens)
        out, lens = dec.aed_greedy_decode(torch.from_numpy(wl.prompt).to(dec.device), 12)
        out = out.cpu().numpy()
        first = G.first_near_tie(ref_logits, G.TOL[dtype])
        for b in range(len(enc_lens)):
            assert (out[b, :first[b]] == ref_t[b, :first[b]]).all()
    dec.close()
