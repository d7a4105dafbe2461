"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle on the same
seeded inputs.  Indices must match bit for bit; outputs within 1e-5 (fp32) / 2e-2 (bf16) absolute.
"""
import math

import numpy as np
import pytest
import torch

import oracle
from paper_2512_17077_amd import hcsa, synth, workload

pytestmark = pytest.mark.gpu

TOL = {torch.float32: 1e-5, torch.bfloat16: 2e-2}


def say(msg):
    print(msg, flush=True)


def oracle_select(w, pool_w=1):
    return oracle.select(synth.to_bits(w.q), synth.to_bits(w.k), w.cu_q, w.cu_kv, w.cu_k, pool_w)


def oracle_attend(w, idx):
    return oracle.attend(synth.to_bits(w.q), synth.to_bits(w.k), synth.to_bits(w.v), w.cu_q, w.cu_kv, idx, w.cu_k,
                         w.seq_mode, w.softmax_scale)


SELECT_FORMS = [(hcsa.DLLM_SELECT_FORM_TWO_LAUNCHES, "two launches"), (hcsa.DLLM_SELECT_FORM_ONE_LAUNCH, "one launch"),
                (hcsa.DLLM_SELECT_FORM_AUTO, "the library's choice")]


def run_select_in_every_form(dw, ref, call):
    """Selection has two forms with identical results; every parity case goes through both (the one-launch form
    wherever it takes the shape) and through the library's own choice, each against the oracle."""
    try:
        for form, label in SELECT_FORMS:
            hcsa.dllm_hcsa_set_select_form(form)
            dw.idx.fill_(-7)
            call()
            torch.cuda.synchronize()
            got = dw.idx.cpu().numpy()
            if not np.array_equal(got, ref):
                bad = np.argwhere(got != ref)
                h, t = bad[0]
                raise AssertionError(f"{label}: {len(bad)} of {ref.size} indices differ; first at head {h}, slot {t}: "
                                     f"gpu {got[h, t]} oracle {ref[h, t]}")
    finally:
        hcsa.dllm_hcsa_set_select_form(hcsa.DLLM_SELECT_FORM_AUTO)


def check_select(w, pool_w=1, name=""):
    say(f"select {name or w.name} dtype={w.dtype} B={w.batch} Hq={w.n_q_heads} Hkv={w.n_kv_heads} "
        f"D={w.head_dim} maxL={int(w.kv_lens.max())} pool_w={pool_w}")
    dw = workload.DeviceWorkload(w)
    ref = oracle_select(w, pool_w)
    run_select_in_every_form(dw, ref, lambda: dw.select(pool_w))
    return dw, ref


def check_attend(w, idx, name="", dw=None):
    say(f"attend {name or w.name} dtype={w.dtype} B={w.batch} Hq={w.n_q_heads} Hkv={w.n_kv_heads} "
        f"D={w.head_dim} maxk={int(w.keep.max())} maxq={int(w.q_lens.max())}")
    dw = dw or workload.DeviceWorkload(w)
    dw.o.fill_(float("nan"))
    dw.attend(torch.from_numpy(np.ascontiguousarray(idx)).to(dw.device))
    torch.cuda.synchronize()
    got = dw.o.float().cpu().numpy().astype(np.float64)
    ref = oracle_attend(w, idx)
    err = np.abs(got - ref)
    assert np.isfinite(got).all(), "non-finite output"
    assert err.max() <= TOL[w.dtype], f"max abs error {err.max():.3e} at {np.unravel_index(err.argmax(), err.shape)}"
    return float(err.max())


def custom(seed, dtype, Hq, Hkv, D, lens, qlens, keep, mode=None, salient=0.0):
    return synth.make_workload(f"custom{seed}", synth.SEED_BASE + 1000 + seed, dtype, Hq, Hkv, D, lens, qlens, keep,
                               seq_mode=mode, salient_frac=salient)


# ------------------------------------------------------------------ selection

@pytest.mark.parametrize("c", [1, 2])
def test_select_small_configs(c):
    check_select(synth.config(c))


def test_select_config3_full():
    check_select(synth.config(3))


def test_benchmark_workloads_take_the_selection_form_the_documentation_says():
    """On the 256 compute units of an MI355X the mixed grouped-query burst is selected in one launch (also with
    the pooling window), the ragged batch in two; the parity cases above run both forms on both either way."""
    d5, d3 = workload.DeviceWorkload(synth.config(5)), workload.DeviceWorkload(synth.config(3))
    assert hcsa.dllm_hcsa_select_form_of(d5.batch) == hcsa.DLLM_SELECT_FORM_ONE_LAUNCH
    assert hcsa.dllm_hcsa_select_form_of(d5.batch, pool_w=3) == hcsa.DLLM_SELECT_FORM_ONE_LAUNCH
    assert hcsa.dllm_hcsa_select_form_of(d5.batch, head_sum=True) == hcsa.DLLM_SELECT_FORM_TWO_LAUNCHES
    assert hcsa.dllm_hcsa_select_form_of(d3.batch) == hcsa.DLLM_SELECT_FORM_TWO_LAUNCHES


def test_select_config5_gqa_full():
    check_select(synth.config(5))


@pytest.mark.parametrize("dtype,D", [(torch.bfloat16, 128), (torch.bfloat16, 64), (torch.float32, 128), (torch.float32, 64)])
def test_select_ragged_lengths(dtype, D):
    lens = [1, 63, 65, 257, 1000, 64, 300]
    keep = [1, 10, 65, 100, 999, 64, 0]          # k == L, k == 1 and a skipped sequence included
    w = custom(1, dtype, 4, 2, D, lens, [32, 1, 7, 33, 32, 32, 32], keep)
    dw, ref = check_select(w)
    # the skipped sequence has no slots; nothing outside [0, total_k) exists to be clobbered
    assert dw.idx.shape[1] == sum(keep)


def test_select_forced_ties_and_zero_queries():
    w = custom(2, torch.bfloat16, 4, 4, 128, [500, 200], [32, 32], [50, 199])
    # duplicate rows: bit-equal scores, lower position must win
    w.k[100:200] = w.k[0:100].clone()
    w.k[520:560] = w.k[500:540].clone()
    check_select(w, name="duplicated rows")
    w.q.zero_()
    dw, ref = check_select(w, name="zero queries")
    assert np.array_equal(ref[:, :50], np.tile(np.arange(50), (4, 1)))


@pytest.mark.parametrize("pool_w", [3, 5])
def test_select_with_pooling(pool_w):
    w = custom(3, torch.bfloat16, 8, 2, 128, [700, 33, 2, 1500], [32, 32, 32, 32], [350, 5, 1, 150])
    check_select(w, pool_w=pool_w)


def test_select_maximum_lengths():
    w = custom(4, torch.bfloat16, 2, 1, 64, [32768, 5], [32, 32], [3000, 2])
    check_select(w)
    w2 = custom(5, torch.bfloat16, 2, 1, 64, [16384], [32], [8000])
    check_select(w2, pool_w=3)


@pytest.mark.parametrize("pool_w", [1, 3])
def test_select_list_lengths_around_4096(pool_w):
    # lists of up to 4096 positions and longer ones are ranked by different kernels
    w = custom(6, torch.bfloat16, 4, 2, 64, [4096, 4095, 3585, 7], [32, 32, 32, 32], [4096, 1, 2000, 7])
    w.k[4096 + 100:4096 + 164] = w.k[4096:4096 + 64].clone()      # ties
    check_select(w, pool_w=pool_w)
    w2 = custom(7, torch.bfloat16, 4, 2, 64, [4097, 4096, 8192], [32, 32, 32], [4097, 1000, 4000])
    check_select(w2, pool_w=pool_w)


@pytest.mark.parametrize("dtype,Hq,Hkv,D", [(torch.bfloat16, 16, 4, 128), (torch.bfloat16, 8, 4, 64), (torch.float32, 4, 4, 64)])
def test_select_in_one_launch_edges(dtype, Hq, Hkv, D):
    """The shapes the one-launch form is built around: lists that end inside, at and just past a 64-row tile and
    a wave's run of tiles, the longest list it takes (8192), kept counts of 1 and of everything, scores that tie
    exactly across many tiles (equal keys are kept from the lowest position up, so a tile keeps only its share),
    a forced block, and more (sequence, KV head) pairs than one round of workgroups."""
    lens = [8192, 8191, 4160, 1025, 1024, 513, 512, 511, 129, 64, 63, 2, 1]
    keep = [8192, 1, 2080, 1000, 256, 513, 100, 510, 128, 1, 63, 1, 1]
    w = custom(41, dtype, Hq, Hkv, D, lens, [32] * len(lens), keep, salient=0.02)
    check_select(w, name="edges")
    # exact ties: every sequence repeats its first 40 rows many times over, so each score value occurs in up to
    # eight tiles and the threshold value is shared by rows of which only the first few are kept
    off = 0
    for L in lens:
        for r in range(40, L, 40):
            n = min(40, L - r)
            w.k[off + r:off + r + n] = w.k[off:off + n].clone()
        off += L
    check_select(w, name="edges, rows repeated every 40 positions")
    # pooling windows reach across tiles (64 positions) and across the runs of tiles of neighbouring waves
    check_select(w, pool_w=3, name="edges, repeated rows, pooling window 3")
    check_select(w, pool_w=63, name="edges, repeated rows, pooling window 63")
    check_select_ex(w, 1, 1, False, "edges, forced block of 1 on repeated rows")
    # several rounds of workgroups: 80 sequences are taken in batch order, up to 64 longest list first
    many = custom(42, dtype, 8, 8, D, [700] * 80, [32] * 80, [70] * 80)
    check_select(many, name="more pairs than compute units")
    rng = np.random.default_rng(43)
    lens64 = [int(x) for x in rng.integers(1, 1500, size=64)]
    keep64 = [int(rng.integers(0, L + 1)) for L in lens64]      # (some sequences are not scored at all)
    ragged = custom(43, dtype, 8, 8, D, lens64, [32] * 64, keep64)
    check_select(ragged, name="64 ragged sequences, more pairs than compute units")


@pytest.mark.parametrize("dtype,Hq,Hkv,D", [(torch.bfloat16, 32, 8, 128), (torch.bfloat16, 16, 16, 64),
                                            (torch.float32, 16, 8, 64), (torch.bfloat16, 24, 8, 128)])
def test_select_large_ragged_batches(dtype, Hq, Hkv, D):
    """Half a million (token, KV head) rows: ragged lengths around the 16- and 64-row tile sizes,
    sequences that are not scored, one to four query heads per KV head."""
    per_head = 2048 * 256 // Hkv
    lens = [1, 15, 16, 17, 63, 300, 4097, 8192, 31]
    keep = [1, 0, 16, 5, 0, 150, 2000, 4096, 31]
    qlens = [32, 32, 1, 7, 32, 33, 32, 32, 32]
    while sum(lens) < per_head + 64:                  # fill up with long sequences
        lens.append(min(20001, per_head + 64 - sum(lens)))
        keep.append(lens[-1] // 3)
        qlens.append(32)
    w = custom(15, dtype, Hq, Hkv, D, lens, qlens, keep, salient=0.02)
    check_select(w)


def test_select_strided_inputs():
    """q/k/v as views into one fused QKV activation, the layout a model layer would hand over."""
    Hq, Hkv, D, L = 8, 2, 128, 777
    w = custom(6, torch.bfloat16, Hq, Hkv, D, [L], [L], [100])
    fused = torch.zeros((L, Hq + 2 * Hkv, D), dtype=torch.bfloat16, device="cuda:0")
    fused[:, :Hq] = w.q.cuda(); fused[:, Hq:Hq + Hkv] = w.k.cuda(); fused[:, Hq + Hkv:] = w.v.cuda()
    q, k, v = fused[-32:, :Hq], fused[:, Hq:Hq + Hkv], fused[:, Hq + Hkv:]
    w.q = w.q[-32:].contiguous()
    w.cu_q = np.array([0, 32], np.int32)
    cu_q = torch.tensor([0, 32], dtype=torch.int32, device="cuda:0")
    cu_kv = torch.tensor([0, L], dtype=torch.int32, device="cuda:0")
    cu_k = torch.tensor([0, 100], dtype=torch.int32, device="cuda:0")
    batch = hcsa.make_batch(q, k, v, cu_q, cu_kv, 32, L, w.softmax_scale)
    idx = torch.empty((Hq, 100), dtype=torch.int32, device="cuda:0")
    hcsa.dllm_hcsa_select(batch, cu_k, 100, 100, idx)
    ref = oracle_select(w)
    assert np.array_equal(idx.cpu().numpy(), ref)
    o = torch.empty((32, Hq, D), dtype=torch.bfloat16, device="cuda:0")
    hcsa.dllm_hcsa_attend(batch, idx, cu_k, 100, 100, None, o)
    err = np.abs(o.float().cpu().numpy() - oracle_attend(w, ref)).max()
    assert err <= 2e-2


@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float32])
def test_dense_and_pack_on_strided_inputs(dtype):
    """The dense entry point and the pack on views into one fused QKV activation (two ragged sequences)."""
    Hq, Hkv, D = 8, 2, 128
    lens = [300, 77]
    w = custom(16, dtype, Hq, Hkv, D, lens, lens, [0, 0], mode=np.ones(2, np.uint8))
    T = sum(lens)
    fused = torch.zeros((T, Hq + 2 * Hkv, D), dtype=dtype, device="cuda:0")
    fused[:, :Hq] = w.q.cuda(); fused[:, Hq:Hq + Hkv] = w.k.cuda(); fused[:, Hq + Hkv:] = w.v.cuda()
    q, k, v = fused[:, :Hq], fused[:, Hq:Hq + Hkv], fused[:, Hq + Hkv:]
    cu = torch.from_numpy(w.cu_q).cuda()
    batch = hcsa.make_batch(q, k, v, cu, cu, max(lens), max(lens), w.softmax_scale)
    o = torch.full((T, Hq, D), float("nan"), dtype=dtype, device="cuda:0")
    hcsa.dllm_dense_refresh_attend(batch, o)
    torch.cuda.synchronize()
    err = np.abs(o.float().cpu().numpy() - oracle_attend(w, np.zeros((Hq, 0), np.int32))).max()
    assert err <= TOL[dtype]
    # pack a per-head selection of the strided K/V and compare with the oracle's pack, bit for bit
    keep = [120, 77]
    ws = custom(16, dtype, Hq, Hkv, D, lens, lens, keep)   # same seed: same Q, K, V
    assert torch.equal(ws.k, w.k)
    idx = oracle_select(ws)
    cu_k = torch.from_numpy(ws.cu_k).cuda()
    kp = torch.empty((Hq, sum(keep), D), dtype=dtype, device="cuda:0")
    vp = torch.empty_like(kp)
    hcsa.dllm_hcsa_pack(batch, torch.from_numpy(idx).cuda(), cu_k, sum(keep), max(keep), kp, vp)
    torch.cuda.synchronize()
    rk, rv = oracle.pack(synth.to_bits(ws.k), synth.to_bits(ws.v), ws.cu_kv, idx, ws.cu_k)
    assert np.array_equal(synth.to_bits(kp.cpu()), rk) and np.array_equal(synth.to_bits(vp.cpu()), rv)


# ------------------------------------------------------------------ attention over kept rows

@pytest.mark.parametrize("c", [1, 2])
def test_attend_small_configs(c):
    w = synth.config(c)
    check_attend(w, oracle_select(w))


def test_attend_config3_full():
    w = synth.config(3)
    check_attend(w, oracle_select(w))


@pytest.mark.parametrize("dtype,D", [(torch.bfloat16, 128), (torch.bfloat16, 64), (torch.float32, 64), (torch.float32, 128)])
def test_attend_ragged_keep_and_query_counts(dtype, D):
    lens = [40, 300, 65, 1000, 129, 77]
    keep = [1, 33, 65, 517, 0, 77]               # k == 1, k == L, nothing kept, several tiles + ragged tail
    qlens = [1, 7, 33, 32, 32, 70]
    w = custom(7, dtype, 4, 2, D, lens, qlens, keep)
    idx = oracle_select(w)
    check_attend(w, idx)
    # k == 1 returns that V row exactly (bf16 in, bf16 out: no rounding at all)
    dw = workload.DeviceWorkload(w)
    dw.attend(torch.from_numpy(idx).cuda())
    row = int(idx[0, 0])
    assert torch.equal(dw.o[0, 0].cpu(), w.v[row, 0])


def test_attend_unsorted_and_repeated_indices():
    w = custom(8, torch.bfloat16, 4, 4, 128, [600, 90], [32, 32], [200, 90])
    rng = np.random.default_rng(8)
    idx = np.concatenate([rng.integers(0, 600, size=(4, 200)), rng.integers(0, 90, size=(4, 90))], axis=1).astype(np.int32)
    check_attend(w, idx)


def test_attend_chunked_long_keep_lists():
    """Few (sequence, head) pairs with long kept lists are split over workgroups and merged."""
    w = custom(9, torch.bfloat16, 2, 1, 128, [4096, 700], [32, 32], [3000, 100], salient=0.05)
    dw = workload.DeviceWorkload(w)
    assert hcsa.dllm_hcsa_attend_workspace(dw.batch, dw.max_k) > 0
    check_attend(w, oracle_select(w), dw=dw)
    w2 = custom(10, torch.bfloat16, 2, 2, 64, [2048], [45], [2048])
    check_attend(w2, oracle_select(w2))


@pytest.mark.parametrize("D", [128, 64])
def test_attend_more_lists_than_compute_units(D):
    """More (sequence, head, chunk) items than compute units: each workgroup walks several of them."""
    lens = [900, 40, 300, 65, 700, 129, 77, 512, 33, 260, 1000, 90]
    keep = [800, 1, 33, 65, 517, 0, 77, 0, 32, 129, 31, 90]        # nothing kept, single rows, ragged tails
    qlens = [32, 1, 7, 33, 32, 32, 70, 32, 0, 32, 32, 5]           # one and three query tiles, no query
    mode = np.array([0, 0, 0, 0, 0, 0, 0, 1, 0, 0, 0, 0], np.uint8)  # one sequence is left to the dense path
    w = custom(12, torch.bfloat16, 32, 8, D, lens, qlens, keep, mode=mode)
    check_attend(w, oracle_select(w))
    # long lists cut into chunks: 3 sequences x 32 heads x 3 chunks
    w2 = custom(13, torch.bfloat16, 32, 32, D, [5000, 2500, 100], [32, 9, 32], [4500, 2100, 7])
    dw = workload.DeviceWorkload(w2)
    assert hcsa.dllm_hcsa_attend_workspace(dw.batch, dw.max_k) > 0
    check_attend(w2, oracle_select(w2), dw=dw)
    # more than 64 sequences (walked in batch order)
    rng = np.random.default_rng(14)
    lens3 = rng.integers(20, 200, size=70).tolist()
    keep3 = [int(rng.integers(0, l + 1)) for l in lens3]
    w3 = custom(14, torch.bfloat16, 8, 2, D, lens3, [32] * 70, keep3)
    check_attend(w3, oracle_select(w3))


def test_attend_keep_all_equals_dense_entry_point():
    """Keeping every row through the index lists and the dense entry point: both against the oracle's dense
    attention (k = L reproduces dense softmax attention)."""
    w = custom(11, torch.bfloat16, 4, 2, 128, [333, 64], [32, 20], [333, 64])
    idx = oracle_select(w)
    assert all(np.array_equal(idx[h, int(w.cu_k[b]):int(w.cu_k[b + 1])], np.arange(int(w.kv_lens[b])))
               for h in range(4) for b in range(2))
    dense_w = synth.with_keep(w, [0, 0])
    dense_w.seq_mode[:] = 1
    want = oracle_attend(dense_w, np.zeros((4, 0), np.int32))
    dw = workload.DeviceWorkload(w)
    dw.o.fill_(float("nan"))
    dw.attend(torch.from_numpy(idx).cuda())
    torch.cuda.synchronize()
    assert np.abs(dw.o.float().cpu().numpy() - want).max() <= 2e-2
    dw.o.fill_(float("nan"))
    dw.dense_refresh()
    torch.cuda.synchronize()
    assert np.abs(dw.o.float().cpu().numpy() - want).max() <= 2e-2


def test_select_then_attend_end_to_end_gpu_indices():
    w = synth.config(3, scale_down=4)
    dw, ref = check_select(w)
    dw.attend()
    torch.cuda.synchronize()
    err = np.abs(dw.o.float().cpu().numpy() - oracle_attend(w, ref)).max()
    assert err <= 2e-2


# ------------------------------------------------------------------ dense and mixed

def test_dense_small_and_ragged():
    w = custom(12, torch.bfloat16, 4, 2, 128, [100, 129, 64, 1, 300], [100, 5, 64, 3, 257], [0] * 5,
               mode=np.ones(5, np.uint8))
    check_attend(w, np.zeros((4, 0), np.int32), name="dense via attend")
    dw = workload.DeviceWorkload(w)
    dw.o.fill_(float("nan"))
    dw.dense_refresh()
    err = np.abs(dw.o.float().cpu().numpy() - oracle_attend(w, np.zeros((4, 0), np.int32))).max()
    assert err <= 2e-2
    for dtype, D in ((torch.bfloat16, 64), (torch.float32, 64), (torch.float32, 128)):
        w = custom(13, dtype, 4, 4, D, [70, 200], [70, 9], [0, 0], mode=np.ones(2, np.uint8))
        check_attend(w, np.zeros((4, 0), np.int32), name=f"dense {dtype} D={D}")


def test_dense_large_logits():
    """Half of the K rows scaled by 4: base-2 logits reach +-25 and a few keys carry each query.  The
    dense kernel keeps Q as given and scales the fp32 scores (scaling Q and rounding it to bf16 again
    puts 2e-2 of error into the output at such logits)."""
    w = custom(14, torch.bfloat16, 8, 2, 128, [130, 64, 700], [130, 64, 700], [0, 0, 0], mode=np.ones(3, np.uint8),
               salient=0.5)
    err = check_attend(w, np.zeros((8, 0), np.int32), name="dense, large logits")
    say(f"max abs error {err:.3e}")
    assert err <= 1.2e-2   # bf16 rounding of P and of O (|O| < 4: half an ulp is 7.8e-3) and nothing else


@pytest.mark.parametrize("order", ["ascending", "descending", "zero_queries", "huge"])
def test_attend_logit_orders_that_stress_the_online_softmax(order):
    """Keys whose logits grow along the sequence make the running maximum rise at every tile (the lazy
    rescale fires again and again); falling ones never raise it after the first tile; zero queries give
    the plain mean of V; logits of +-150 make the softmax one-hot.  Sparse and dense sequences in one call."""
    lens = [700, 513, 300]
    mode = np.array([0, 1, 0], np.uint8)
    w = custom(15, torch.bfloat16, 4, 2, 128, lens, [32, 513, 32], [333, 0, 300], mode=mode)
    k = w.k.float()
    for b in range(3):
        lo, hi = int(w.cu_kv[b]), int(w.cu_kv[b + 1])
        ramp = torch.linspace(0.0, 1.0, hi - lo)[:, None, None]
        if order == "ascending":
            k[lo:hi] *= 1.0 + 7.0 * ramp
        elif order == "descending":
            k[lo:hi] *= 8.0 - 7.0 * ramp
        elif order == "huge":
            k[lo:hi] *= 12.0
    if order == "zero_queries":
        w.q.zero_()
    w.k.copy_(k.to(torch.bfloat16))
    idx = oracle_select(w)
    err = check_attend(w, idx, name=f"logit order {order}")
    say(f"max abs error {err:.3e}")


def test_dense_config4_scaled():
    w = synth.config(4, scale_down=8)
    check_attend(w, np.zeros((32, 0), np.int32))


def test_mixed_batch_scaled_config5():
    w = synth.config(5, scale_down=16)
    dw, ref = check_select(w)
    check_attend(w, ref, dw=dw)


@pytest.mark.parametrize("Hq,Hkv,D", [(6, 2, 128), (16, 2, 128), (12, 2, 64), (5, 5, 64)])
def test_query_heads_per_kv_head_3_8_6_1(Hq, Hkv, D):
    """Group sizes that the score kernel walks one, two or four heads at a time (with a repeat), through
    select, sparse attend and dense attend in one mixed batch."""
    lens = [333, 64, 1000, 130]
    mode = np.array([0, 0, 0, 1], np.uint8)
    qlens = [32, 9, 32, 130]
    keep = [100, 64, 411, 0]
    w = custom(41, torch.bfloat16, Hq, Hkv, D, lens, qlens, keep, mode=mode, salient=0.05)
    dw, ref = check_select(w)
    check_attend(w, ref, dw=dw)


def test_batches_of_more_than_64_sequences():
    """Above 64 sequences the kernels read their sequence's offsets directly instead of from the
    lane-parallel table: 80 short sequences, sparse and dense mixed, ragged lengths and keep counts."""
    rng = np.random.default_rng(31)
    n = 80
    lens = rng.integers(33, 260, size=n)
    mode = (rng.random(n) < 0.25).astype(np.uint8)
    qlens = np.where(mode == 1, lens, 32)
    keep = np.where(mode == 1, 0, np.maximum(1, (lens * rng.uniform(0.1, 0.9, size=n)).astype(np.int64)))
    w = custom(31, torch.bfloat16, 4, 2, 128, lens.tolist(), qlens.tolist(), keep.tolist(), mode=mode)
    dw, ref = check_select(w)
    check_attend(w, ref, dw=dw)
    # the same batch through the packed layout
    dw.pack()
    dw.o.fill_(float("nan"))
    sparse_rows = np.concatenate([np.arange(w.cu_q[b], w.cu_q[b + 1]) for b in range(n) if mode[b] == 0])
    dw.attend_packed()
    torch.cuda.synchronize()
    got = dw.o.float().cpu().numpy()[sparse_rows]
    assert np.abs(got - oracle_attend(w, ref)[sparse_rows]).max() <= 2e-2


@pytest.mark.parametrize("Hq,Hkv,D,n", [(16, 8, 64, 64), (32, 16, 128, 20), (6, 3, 128, 64), (8, 8, 128, 1)])
def test_dense_tiles_place_themselves_on_ragged_and_mixed_batches(Hq, Hkv, D, n):
    """Up to 64 sequences the dense kernel's workgroups find their own (sequence, head, query tile) from a prefix
    sum over the densely attended sequences: ragged query counts around the 256-row tile, sequences without
    queries, sparse sequences in between, KV-head counts that are and are not multiples of eight, through
    both entry points."""
    rng = np.random.default_rng(1000 + Hq + n)
    lens = rng.integers(1, 700, size=n)
    lens[rng.integers(0, n)] = 256
    lens[rng.integers(0, n)] = 513
    mode = (rng.random(n) < 0.5).astype(np.uint8)
    mode[0] = 1
    qlens = np.where(mode == 1, lens, np.minimum(lens, 32))
    if n > 2:
        qlens[1] = 0          # a sequence that only holds cache
    keep = np.where(mode == 1, 0, np.maximum(1, lens // 3))
    w = custom(40 + n, torch.bfloat16, Hq, Hkv, D, lens.tolist(), qlens.tolist(), keep.tolist(), mode=mode)
    if (mode == 0).any():
        dw, ref = check_select(w)
        check_attend(w, ref, dw=dw)
    # every sequence densely, queries = all its rows where it has any
    wd = custom(41 + n, torch.bfloat16, Hq, Hkv, D, lens.tolist(), np.where(qlens > 0, lens, 0).tolist(), [0] * n,
                mode=np.ones(n, np.uint8))
    dd = workload.DeviceWorkload(wd)
    dd.o.fill_(float("nan"))
    dd.dense_refresh()
    torch.cuda.synchronize()
    got = dd.o.float().cpu().numpy().astype(np.float64)
    want = oracle_attend(wd, np.zeros((Hq, 0), np.int32))
    assert np.isfinite(got).all() and np.abs(got - want).max() <= TOL[wd.dtype]


def block_rows(w, seed):
    """One query row out of every 32-row block of every sequence: every 32-query block of every wave of every
    workgroup of a full-size launch gets one row checked."""
    rng = np.random.default_rng(seed)
    picks, qparts = [], []
    for b in range(w.batch):
        n = int(w.q_lens[b])
        starts = np.arange(0, n, 32)
        r = starts + rng.integers(0, np.minimum(32, n - starts)) + int(w.cu_q[b])
        picks.append(r)
        qparts.append(w.q[torch.from_numpy(r)])
    sub = synth.Workload(w.name + "_blockrows", w.dtype, w.n_q_heads, w.n_kv_heads, w.head_dim, torch.cat(qparts), w.k,
                         w.v, np.concatenate([[0], np.cumsum([len(p) for p in picks])]).astype(np.int32), w.cu_kv,
                         w.cu_k, w.seq_mode, w.softmax_scale)
    return sub, np.concatenate(picks)


def check_whole_sequences(w, dw, seqs, idx):
    """Every output element of the sequences `seqs` against the oracle."""
    for b in seqs:
        say(f"  whole sequence {b}: {int(w.q_lens[b])} query rows x {w.n_q_heads} heads over {int(w.kv_lens[b])} keys")
        sub = synth.subset(w, [b])
        sub_idx = None if idx is None else idx[:, int(w.cu_k[b]):int(w.cu_k[b + 1])]
        if sub_idx is None:
            sub_idx = np.zeros((w.n_q_heads, 0), np.int32)
        want = oracle_attend(sub, np.ascontiguousarray(sub_idx))
        got = dw.o[int(w.cu_q[b]):int(w.cu_q[b + 1])].float().cpu().numpy()
        err = np.abs(got - want)
        assert err.max() <= TOL[w.dtype], f"sequence {b}: max abs error {err.max():.3e} at {np.unravel_index(err.argmax(), err.shape)}"


def test_dense_config4_full_size():
    """Refresh workload at full size, in the launch the benchmark times: two whole sequences element by
    element, and one row of every 32-query block of all of them."""
    w = synth.config(4)
    dw = workload.DeviceWorkload(w)
    say("dense config 4 full size")
    dw.o.fill_(float("nan"))
    dw.dense_refresh()
    torch.cuda.synchronize()
    assert torch.isfinite(dw.o.float()).all()
    check_whole_sequences(w, dw, [0, w.batch - 1], None)
    sub, rows = block_rows(w, 44)
    ref = oracle_attend(sub, np.zeros((w.n_q_heads, 0), np.int32))
    got = dw.o[torch.from_numpy(rows).cuda()].float().cpu().numpy()
    assert np.abs(got - ref).max() <= 2e-2


def test_mixed_config5_full_size():
    """Mixed burst at full size through one attend call: every query row of every Reuse sequence, one whole
    Refresh sequence, and one row of every 32-query block of the other Refresh sequences."""
    w = synth.config(5)
    dw, ref = check_select(w)
    say("attend config 5 full size (mixed, one call)")
    dw.o.fill_(float("nan"))
    dw.attend()
    torch.cuda.synchronize()
    assert torch.isfinite(dw.o.float()).all()
    sparse = [b for b in range(w.batch) if w.seq_mode[b] == 0]
    dense = [b for b in range(w.batch) if w.seq_mode[b] == 1]
    check_whole_sequences(w, dw, sparse + dense[:1], ref)
    sub, rows = block_rows(w, 55)
    want = oracle_attend(sub, ref)
    got = dw.o[torch.from_numpy(rows).cuda()].float().cpu().numpy()
    assert np.abs(got - want).max() <= 2e-2


@pytest.mark.parametrize("c", [3, 5])
def test_paper_defaults_full_size(c):
    """The paper's default setting (Table 2: retention 0.5, pooling kernel 3) on the batched Reuse workload
    and on the mixed burst at full size: selection bit for bit, attention over the kept rows element by
    element (Reuse rows), the Refresh sequences on one row per 32-query block."""
    w = synth.at_retention(synth.config(c), 0.5)
    dw, ref = check_select(w, pool_w=3, name=f"c{c} at retention 0.5, pool_w=3")
    dw.o.fill_(float("nan"))
    dw.attend()
    torch.cuda.synchronize()
    check_whole_sequences(w, dw, [b for b in range(w.batch) if w.seq_mode[b] == 0], ref)
    if (w.seq_mode == 1).any():
        sub, rows = block_rows(w, 66)
        want = oracle_attend(sub, ref)
        got = dw.o[torch.from_numpy(rows).cuda()].float().cpu().numpy()
        assert np.abs(got - want).max() <= 2e-2


# ------------------------------------------------------------------ packing (Section 4.5) and the packed Reuse step

def check_pack_and_packed_attend(w, name):
    say(f"pack {name} dtype={w.dtype} B={w.batch} Hq={w.n_q_heads} Hkv={w.n_kv_heads} D={w.head_dim} "
        f"maxk={int(w.keep.max())}")
    idx = oracle_select(w)
    dw = workload.DeviceWorkload(w)
    dw.idx.copy_(torch.from_numpy(idx))
    dw.pack()
    dw.k_packed.fill_(0)
    dw.v_packed.fill_(0)
    dw.pack()
    torch.cuda.synchronize()
    kp, vp = oracle.pack(synth.to_bits(w.k), synth.to_bits(w.v), w.cu_kv, idx, w.cu_k)
    assert np.array_equal(synth.to_bits(dw.k_packed.cpu()), kp), "packed K differs from the oracle"
    assert np.array_equal(synth.to_bits(dw.v_packed.cpu()), vp), "packed V differs from the oracle"
    # Reuse step over the packed cache against the oracle's attention over the kept rows in place
    dw.o.fill_(float("nan"))
    dw.attend_packed()
    torch.cuda.synchronize()
    got = dw.o.float().cpu().numpy().astype(np.float64)
    ref = oracle_attend(w, idx)
    err = np.abs(got - ref)
    assert np.isfinite(got).all(), "non-finite output"
    assert err.max() <= TOL[w.dtype], f"max abs error {err.max():.3e}"


@pytest.mark.parametrize("dtype,D,Hq,Hkv", [(torch.bfloat16, 128, 8, 8), (torch.bfloat16, 64, 8, 2),
                                            (torch.float32, 64, 4, 4), (torch.float32, 128, 4, 2)])
def test_pack_and_packed_attend_ragged(dtype, D, Hq, Hkv):
    lens = [300, 65, 1, 777, 129]
    keep = [37, 65, 1, 500, 128]
    check_pack_and_packed_attend(custom(61, dtype, Hq, Hkv, D, lens, [32, 5, 1, 40, 32], keep, salient=0.05),
                                 f"ragged {dtype} D={D}")


@pytest.mark.parametrize("D", [128, 64])
def test_packed_attend_long_ragged_lists_over_many_heads(D):
    """The index-free path of the multi-list kernel: more (sequence, head, chunk) items than compute units, lists
    cut into chunks and merged, several query tiles, a list of seven rows and one of none."""
    w = custom(31, torch.bfloat16, 32, 32, D, [5000, 2500, 100, 900], [32, 9, 70, 32], [4500, 2100, 7, 0])
    check_pack_and_packed_attend(w, f"long ragged lists, D={D}")
    w2 = custom(32, torch.bfloat16, 32, 8, D, [900, 40, 300, 65, 700, 129, 77, 512, 33, 260, 1000, 90],
                [32, 1, 7, 33, 32, 32, 70, 32, 0, 32, 32, 5], [800, 1, 33, 65, 517, 0, 77, 11, 32, 129, 31, 90])
    check_pack_and_packed_attend(w2, f"twelve ragged sequences, grouped queries, D={D}")


def test_pack_and_packed_attend_config3_full():
    check_pack_and_packed_attend(synth.config(3), "c3 full size")


# ------------------------------------------------------------------ selection variants (Eq. 4 forced block, Eq. 5 shared list)

def check_select_ex(w, pool_w, forced_tail, head_sum, name):
    say(f"select_ex {name} dtype={w.dtype} B={w.batch} Hq={w.n_q_heads} Hkv={w.n_kv_heads} D={w.head_dim} "
        f"maxL={int(w.kv_lens.max())} pool_w={pool_w} forced_tail={forced_tail} head_sum={head_sum}")
    dw = workload.DeviceWorkload(w)
    ref = oracle.select_ex(synth.to_bits(w.q), synth.to_bits(w.k), w.cu_q, w.cu_kv, w.cu_k, pool_w, forced_tail, head_sum)
    run_select_in_every_form(dw, ref, lambda: dw.select_ex(pool_w, forced_tail, head_sum))
    return dw, ref


@pytest.mark.parametrize("pool_w,forced_tail,head_sum", [(1, 32, False), (3, 32, False), (1, 0, True), (3, 0, True),
                                                         (3, 16, True)])
@pytest.mark.parametrize("dtype,Hq,Hkv", [(torch.bfloat16, 8, 8), (torch.bfloat16, 8, 2), (torch.float32, 4, 4)])
def test_select_ex_ragged(pool_w, forced_tail, head_sum, dtype, Hq, Hkv):
    lens = [300, 65, 33, 1777, 129]
    keep = [60, 65, 32, 500, 100]
    w = custom(71, dtype, Hq, Hkv, 128, lens, [32, 5, 1, 32, 32], keep, salient=0.05)
    check_select_ex(w, pool_w, forced_tail, head_sum, "ragged")


def test_select_ex_config3_forced_block_then_attend():
    """The denoising-loop shape of Eq. 4: the active block (last 32 positions) is always attended."""
    w = synth.config(3)
    dw, ref = check_select_ex(w, 1, 32, False, "c3 forced block")
    for b in range(w.batch):
        tail = ref[:, w.cu_k[b + 1] - 32:w.cu_k[b + 1]]
        assert np.array_equal(tail, np.tile(np.arange(w.kv_lens[b] - 32, w.kv_lens[b]), (w.n_q_heads, 1)))
    check_attend(w, ref, "c3 forced block", dw=dw)


def test_select_ex_config3_head_summed():
    check_select_ex(synth.config(3), 1, 0, True, "c3 shared list")


def test_forced_block_larger_than_a_kept_list_writes_nothing_for_that_sequence():
    """forced_tail <= k_b cannot be checked on the host.  A sequence that breaks it gets no list (its part of
    idx_out keeps what was there) instead of a write in front of its list; the others are selected as usual."""
    w = custom(29, torch.bfloat16, 8, 2, 128, [300, 100, 200], [32, 32, 32], [50, 30, 64])
    dw = workload.DeviceWorkload(w)
    say("select_ex with forced_tail 40 on kept counts 50, 30, 64")
    dw.idx.fill_(-7)
    dw.select_ex(forced_tail=40)
    torch.cuda.synchronize()
    got = dw.idx.cpu().numpy()
    assert (got[:, 50:80] == -7).all()
    ok = synth.subset(w, [0, 2])
    ref = oracle.select_ex(synth.to_bits(ok.q), synth.to_bits(ok.k), ok.cu_q, ok.cu_kv, ok.cu_k, 1, 40, False)
    assert np.array_equal(got[:, :50], ref[:, :50]) and np.array_equal(got[:, 80:], ref[:, 50:])


def test_sequences_without_queries():
    """A sequence may have no query rows this step (it only holds cache): selection then ranks a zero
    block sum (all ties, lowest positions win), attention has nothing to write for it, and its
    neighbours in the batch are unaffected."""
    for dtype in (torch.bfloat16, torch.float32):
        w = custom(17, dtype, 4, 2, 128, [100, 37, 64, 200], [0, 37, 0, 32], [40, 0, 0, 77],
                   mode=np.array([0, 1, 1, 0], np.uint8))
        dw, ref = check_select(w)
        assert np.array_equal(ref[:, :40], np.tile(np.arange(40), (4, 1)))
        check_attend(w, ref, dw=dw)


@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float32])
def test_attend_without_cu_k_zeroes_every_sequence_not_flagged_dense(dtype):
    """cu_k = NULL (allowed with total_k = 0): nothing is kept anywhere, so a sequence not flagged dense gets
    zeros (an empty kept set) and the flagged ones full attention; without modes every row is zero."""
    w = custom(23, dtype, 8, 2, 128, [150, 90, 64], [32, 17, 64], [0, 0, 0], mode=np.array([1, 0, 1], np.uint8))
    dw = workload.DeviceWorkload(w)
    say(f"attend with cu_k = NULL, modes {w.seq_mode.tolist()} dtype={dtype}")
    dw.o.fill_(float("nan"))
    hcsa.dllm_hcsa_attend(dw.batch, None, None, 0, 0, dw.seq_mode, dw.o)
    torch.cuda.synchronize()
    ref = oracle.attend(synth.to_bits(w.q), synth.to_bits(w.k), synth.to_bits(w.v), w.cu_q, w.cu_kv, None, None, w.seq_mode,
                        w.softmax_scale)
    got = dw.o.float().cpu().numpy().astype(np.float64)
    assert np.isfinite(got).all()
    assert np.abs(got - ref).max() <= TOL[dtype]
    assert not got[32:49].any() and np.abs(got[:32]).max() > 0
    dw.o.fill_(float("nan"))
    hcsa.dllm_hcsa_attend(dw.batch, None, None, 0, 0, None, dw.o)
    torch.cuda.synchronize()
    assert not dw.o.float().cpu().numpy().any()


# ------------------------------------------------------------------ HIP graph capture

@pytest.mark.parametrize("which_workload", ["layer-shaped config 2", "ragged batch (config 3 / 4)",
                                            "layer-shaped config 2, selection in one launch"])
def test_select_and_attend_replayed_from_a_hip_graph(which_workload):
    """A serving loop captures the launch-bound step once and replays it.  The library allocates
    nothing, clears nothing with memsets and never synchronises, so a captured select + attend must
    give, on every replay and with eager work in between, exactly what the eager calls give for the
    inputs then in the buffers (and the oracle's indices).  The ragged batch has more lists than
    compute units and takes the multi-list attend kernel."""
    w = synth.config(2) if which_workload.startswith("layer") else synth.config(3, scale_down=4)
    dw = workload.DeviceWorkload(w)
    if which_workload.endswith("one launch"):
        hcsa.dllm_hcsa_set_select_form(hcsa.DLLM_SELECT_FORM_ONE_LAUNCH)
    try:
        replay_select_and_attend(w, dw, which_workload)
    finally:
        hcsa.dllm_hcsa_set_select_form(hcsa.DLLM_SELECT_FORM_AUTO)


def replay_select_and_attend(w, dw, which_workload):
    wss = torch.empty(max(256, hcsa.dllm_hcsa_select_workspace(dw.batch, dw.max_k)), dtype=torch.uint8, device=dw.device)
    wsa = torch.empty(max(256, hcsa.dllm_hcsa_attend_workspace(dw.batch, dw.max_k)), dtype=torch.uint8, device=dw.device)
    q_a = dw.q.clone()
    q_b = torch.flip(dw.q, dims=[-1]).contiguous()   # other queries in the same buffer

    def eager(qv):
        dw.q.copy_(qv)
        dw.select(workspace=wss)
        dw.attend(workspace=wsa)
        torch.cuda.synchronize()
        return dw.idx.clone(), dw.o.clone()

    ref = {"a": eager(q_a), "b": eager(q_b)}
    assert np.array_equal(ref["a"][0].cpu().numpy(), oracle_select(w))
    assert not torch.equal(ref["a"][0], ref["b"][0])

    say(f"capturing select + attend of {which_workload}")
    graph = torch.cuda.CUDAGraph()
    dw.q.copy_(q_a)
    torch.cuda.synchronize()
    with torch.cuda.graph(graph):
        dw.select(workspace=wss)
        dw.attend(workspace=wsa)
    for rep, which in enumerate(["a", "b", "a", "b"]):
        say(f"replay {rep} with queries {which}")
        dw.q.copy_(q_a if which == "a" else q_b)
        dw.idx.fill_(-1)
        dw.o.fill_(float("nan"))
        busy = (dw.k.float() * 2).sum()   # the program's own eager work between replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.isfinite(busy)
        assert torch.equal(dw.idx, ref[which][0]), f"replay {rep}: indices differ from the eager call"
        assert torch.equal(dw.o, ref[which][1]), f"replay {rep}: outputs differ from the eager call"


# ------------------------------------------------------------------ random shapes

@pytest.mark.parametrize("seed", list(range(32)))
def test_random_shapes_through_every_entry_point(seed):
    """Seeded random batches (dtype, head_dim, head grouping, ragged lengths and keep counts, a few dense
    sequences, pooling, forced block, shared lists): selection bit-exact, then attention over the
    selected rows, then pack + packed attention, all against the oracle."""
    rng = np.random.default_rng(1000 + seed)
    dtype = torch.bfloat16 if rng.random() < 0.75 else torch.float32
    D = int(rng.choice([64, 128]))
    Hkv = int(rng.choice([1, 2, 4]))
    Hq = Hkv * int(rng.choice([1, 2, 3, 4, 8]))
    nseq = int(rng.integers(1, 9))
    lens = rng.integers(1, 900, size=nseq)
    mode = (rng.random(nseq) < 0.2).astype(np.uint8)
    qlens = np.where(mode == 1, np.minimum(lens, 200), rng.integers(0, 40, size=nseq))
    keep = np.where(mode == 1, 0, np.maximum(1, (lens * rng.uniform(0.05, 1.0, size=nseq)).astype(np.int64)))
    if mode.all():
        mode[0], keep[0], qlens[0] = 0, max(1, lens[0] // 2), 32
    if qlens.sum() == 0:
        qlens[0] = 7
    w = custom(100 + seed, dtype, Hq, Hkv, D, lens.tolist(), qlens.tolist(), keep.tolist(), mode=mode,
               salient=float(rng.choice([0.0, 0.05])))
    pool_w = int(rng.choice([1, 1, 3, 5]))
    head_sum = bool(rng.random() < 0.25)
    sparse_keep = keep[mode == 0]
    forced_tail = int(rng.integers(0, sparse_keep.min() + 1)) if rng.random() < 0.3 else 0
    dw, ref = check_select_ex(w, pool_w, forced_tail, head_sum, f"random {seed}")
    check_attend(w, ref, dw=dw)
    # the packed layout of the same selection (dense sequences keep nothing and are not packed)
    dw.pack()
    torch.cuda.synchronize()
    kp, vp = oracle.pack(synth.to_bits(w.k), synth.to_bits(w.v), w.cu_kv, ref, w.cu_k)
    assert np.array_equal(synth.to_bits(dw.k_packed.cpu()), kp) and np.array_equal(synth.to_bits(dw.v_packed.cpu()), vp)
    dw.o.fill_(float("nan"))
    dw.attend_packed()
    torch.cuda.synchronize()
    rows = np.concatenate([np.arange(w.cu_q[b], w.cu_q[b + 1]) for b in range(nseq) if mode[b] == 0] + [np.zeros(0, np.int64)]).astype(np.int64)
    if len(rows):
        got = dw.o.float().cpu().numpy()[rows]
        assert np.abs(got - oracle_attend(w, ref)[rows]).max() <= TOL[dtype]
