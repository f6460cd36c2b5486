"""kivi_decode_attention_static (the entry point that allocates nothing: its workspace is a static
device array inside the library) against kivi_decode_attention on a caller-owned workspace, through
the C ABI: two calls in a row, the second on a smaller input, plus the refusal of a state that does
not fit the array."""
import ctypes

import numpy as np
import pytest

import gpu_harness as gh
from paper_2402_02750_amd import kivi, workloads
from paper_2402_02750_amd.workloads import CONFIGS

pytestmark = pytest.mark.gpu


def _case(w, context, path):
    torch = gh.require_gpu()
    k, v, q = workloads.keys(w, context), workloads.values(w, context), workloads.queries(w)
    layout, cache = gh.gpu_prefill(w, k, v, kivi.KIVI_FLUSH_WINDOW, path)
    qt = torch.from_numpy(q).cuda()
    ref = torch.empty(q.shape, dtype=torch.float32, device="cuda")
    got = torch.full(q.shape, float("nan"), dtype=torch.float32, device="cuda")
    kivi.kivi_decode_attention(layout, cache, qt, w.softmax_scale, ref)
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    kivi.kivi_decode_attention_static(layout, cache, qt, w.softmax_scale, got)
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before
    plan = kivi.kivi_decode_plan(layout, cache)
    return got.cpu().numpy(), ref.cpu().numpy(), plan


@pytest.mark.parametrize("path", [kivi.KIVI_DECODE_AUTO, kivi.KIVI_DECODE_VALU, kivi.KIVI_DECODE_MFMA_TWO],
                         ids=["auto", "valu", "mfma2"])
def test_static_workspace_two_calls_in_a_row(path):
    # first call: 4 sequences x 8 kv-heads, 16 query heads, context 3000 (several splits per unit, so the
    # parts and counters in the static array are used); second call: a smaller batch and context
    big = workloads.scaled(CONFIGS["tiny"], name="static_big", batch=4, n_q_heads=16, n_kv_heads=8, context=3000, seed=77)
    small = workloads.scaled(CONFIGS["tiny"], name="static_small", batch=1, n_q_heads=4, n_kv_heads=4, context=700, seed=78)
    for w, context in ((big, 3000), (small, 700)):
        print(f"case static workspace: {w.name} path={path}", flush=True)
        got, ref, plan = _case(w, context, path)
        assert plan.splits_quantised + plan.splits_fp16 > 1
        assert np.isfinite(got).all()
        gh.check_close(got, ref.astype(np.float64), f"{w.name} static vs caller workspace")


def test_static_workspace_matches_oracle_and_refuses_oversize():
    torch = gh.require_gpu()
    w = CONFIGS["tiny"]
    k, v, q = workloads.keys(w, w.context), workloads.values(w, w.context), workloads.queries(w)
    layout, cache = gh.gpu_prefill(w, k, v, kivi.KIVI_FLUSH_WINDOW, kivi.KIVI_DECODE_AUTO)
    heads = [(b, h) for b in range(w.batch) for h in range(w.n_kv_heads)]
    oc = gh.oracle_cache_for_heads(w, k, v, heads, "window")
    ref = gh.oracle_attention_for_heads(w, oc, q, heads)
    out = torch.empty(q.shape, dtype=torch.float32, device="cuda")
    kivi.kivi_decode_attention_static(layout, cache, torch.from_numpy(q).cuda(), w.softmax_scale, out)
    torch.cuda.synchronize()
    gh.check_close(gh.pick_heads(out.cpu().numpy(), w, heads), ref, "static vs oracle")
    # a state whose parts pass the array's size is refused before anything is launched
    wide = workloads.scaled(CONFIGS["tiny"], name="static_wide", batch=64, n_q_heads=32, n_kv_heads=32, context=4096, seed=79)
    layout2 = kivi.make_layout(wide.batch, wide.n_q_heads, wide.n_kv_heads, wide.bits, wide.residual, 4096, 192,
                               decode_path=kivi.KIVI_DECODE_AUTO)
    cache2 = kivi.Cache(layout2)
    cache2.c.n_kq = cache2.c.n_vq = 3968
    cache2.c.n_kr = cache2.c.n_vr = 128
    plan = kivi.kivi_decode_plan(layout2, cache2)
    need = 64 * 32 * 16 + 520 * 64 * 32 * (plan.splits_quantised + plan.splits_fp16)
    assert need > kivi.KIVI_STATIC_WORKSPACE_BYTES
    out2 = torch.empty(64, 32, 128, dtype=torch.float32, device="cuda")
    q2 = torch.zeros(64, 32, 128, dtype=torch.float16, device="cuda")
    with pytest.raises(kivi.KiviError) as e:
        kivi.kivi_decode_attention_static(layout2, cache2, q2, 1.0, out2)
    assert e.value.status == kivi.KIVI_ERR_WORKSPACE
