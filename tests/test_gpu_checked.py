"""The library built with -DDLLM_CHECK_PRECONDITIONS on the GPU: valid calls give the release results and
leave the error word at zero; calls that break a device-side precondition set the matching bit and write
nothing.  Every violating call here is safe by construction: the validators read only the offset arrays
([batch+1]), the index lists ([n_q_heads, total_k]) and the modes ([batch]) at the sizes the call declares,
all of which are real tensors of those sizes, and every other kernel returns when it finds the word set."""
import numpy as np
import pytest
import torch

import oracle
from paper_2512_17077_amd import hcsa, synth, workload

pytestmark = pytest.mark.gpu
SENTINEL = -12345


def say(msg):
    print(msg, flush=True)


@pytest.fixture()
def checked():
    hcsa.use_checked_library(True)
    hcsa.lib()
    hcsa.dllm_hcsa_precondition_errors()          # start from a clean word
    yield
    torch.cuda.synchronize()
    hcsa.dllm_hcsa_precondition_errors()
    hcsa.use_checked_library(False)


def small_batch():
    return synth.make_workload("checked", synth.SEED_BASE + 4242, torch.bfloat16, 8, 2, 128, [300, 100], [32, 32], [50, 30])


def test_release_library_reports_no_checks():
    hcsa.use_checked_library(False)
    with pytest.raises(hcsa.DllmError) as e:
        hcsa.dllm_hcsa_precondition_errors()
    assert e.value.status == hcsa.DLLM_ERR_UNSUPPORTED


def test_valid_calls_match_the_oracle_and_leave_the_word_clear(checked):
    w = small_batch()
    dw = workload.DeviceWorkload(w)
    say("checked library: select, attend, pack, packed attend, dense on a valid batch")
    dw.select()
    ref = oracle.select(synth.to_bits(w.q), synth.to_bits(w.k), w.cu_q, w.cu_kv, w.cu_k)
    assert np.array_equal(dw.idx.cpu().numpy(), ref)
    dw.attend()
    want = oracle.attend(synth.to_bits(w.q), synth.to_bits(w.k), synth.to_bits(w.v), w.cu_q, w.cu_kv, ref, w.cu_k, None,
                         w.softmax_scale)
    assert np.abs(dw.o.float().cpu().numpy() - want).max() <= 2e-2
    dw.pack()
    dw.attend_packed()
    assert np.abs(dw.o.float().cpu().numpy() - want).max() <= 2e-2
    dw.dense_refresh()
    dense = oracle.attend(synth.to_bits(w.q), synth.to_bits(w.k), synth.to_bits(w.v), w.cu_q, w.cu_kv, None, None,
                          np.ones(2, np.uint8), w.softmax_scale)
    assert np.abs(dw.o.float().cpu().numpy() - dense).max() <= 2e-2
    assert hcsa.dllm_hcsa_precondition_errors() == 0


def device_i32(x):
    return torch.tensor(x, dtype=torch.int32, device="cuda:0")


def test_violations_are_reported_and_nothing_is_written(checked):
    w = small_batch()
    dw = workload.DeviceWorkload(w)
    Hq = w.n_q_heads
    good_idx = torch.from_numpy(oracle.select(synth.to_bits(w.q), synth.to_bits(w.k), w.cu_q, w.cu_kv, w.cu_k)).cuda()

    def expect(bit, what, call):
        say(f"checked library: {what}")
        o_before = dw.o.clone()
        call()
        got = hcsa.dllm_hcsa_precondition_errors()
        assert got & bit, f"{what}: error word {got:#x} lacks bit {bit:#x}"
        return o_before

    # an index past the end of its sequence, and a negative one: attend and pack refuse
    for bad in (int(w.kv_lens[0]), -1):
        idx = good_idx.clone()
        idx[3, 7] = bad
        dw.o.fill_(7.0)
        before = expect(hcsa.DLLM_CHECK_IDX, f"attend with index {bad}", lambda: dw.attend(idx))
        assert torch.equal(dw.o, before)
        dw.pack()                                   # allocates the packed buffers (valid call)
        assert hcsa.dllm_hcsa_precondition_errors() == 0
        dw.k_packed.fill_(3.0)
        expect(hcsa.DLLM_CHECK_IDX, f"pack with index {bad}", lambda: dw.pack(idx))
        assert bool((dw.k_packed == 3.0).all())
    # more kept rows than the sequence has (the host bound max_k <= max_kv still holds)
    cu_k = device_i32([0, 50, 250])                 # second sequence: 200 kept of 100
    idx_out = torch.full((Hq, 250), SENTINEL, dtype=torch.int32, device="cuda:0")
    expect(hcsa.DLLM_CHECK_K_OVER_L, "select keeping more rows than a sequence has",
           lambda: hcsa.dllm_hcsa_select(dw.batch, cu_k, 250, 200, idx_out))
    assert bool((idx_out == SENTINEL).all())
    # offsets that run backwards
    cu_k = device_i32([0, 60, 40])
    idx_out = torch.full((Hq, 40), SENTINEL, dtype=torch.int32, device="cuda:0")
    expect(hcsa.DLLM_CHECK_CU_K, "select with decreasing cu_k", lambda: hcsa.dllm_hcsa_select(dw.batch, cu_k, 40, 40, idx_out))
    assert bool((idx_out == SENTINEL).all())
    bad_kv = device_i32([0, 300, 250])              # ends below total_kv = 400 and runs backwards
    batch = hcsa.make_batch(dw.q, dw.k, dw.v, dw.cu_q, bad_kv, dw.max_q, dw.max_kv, w.softmax_scale)
    dw.o.fill_(7.0)
    before = dw.o.clone()
    say("checked library: dense attention with decreasing cu_kv")
    hcsa.dllm_dense_refresh_attend(batch, dw.o)
    assert hcsa.dllm_hcsa_precondition_errors() & hcsa.DLLM_CHECK_CU_KV
    assert torch.equal(dw.o, before)
    # fewer kept rows than forced ones
    idx_out = torch.full((Hq, w.total_k), SENTINEL, dtype=torch.int32, device="cuda:0")
    expect(hcsa.DLLM_CHECK_FORCED, "select with forced_tail above a sequence's kept rows",
           lambda: hcsa.dllm_hcsa_select_ex(dw.batch, dw.cu_k, w.total_k, dw.max_k, idx_out, forced_tail=40))
    assert bool((idx_out == SENTINEL).all())
    # and the library works again once the word has been fetched
    dw.select()
    assert torch.equal(dw.idx, good_idx)
    assert hcsa.dllm_hcsa_precondition_errors() == 0
