"""GPU parity of the streaming path (append -> flush -> decode attention, benchmark configuration 3
shape at a size the oracle finishes quickly): cache state bit-exact after every flush, outputs
within tolerance at every step."""
import numpy as np
import pytest

import gpu_harness as gh
from oracle import kivi_oracle as ko
from paper_2402_02750_amd import kivi, workloads
from paper_2402_02750_amd.workloads import CONFIGS, scaled

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("path", [kivi.KIVI_DECODE_VALU, kivi.KIVI_DECODE_MFMA], ids=["valu", "mfma"])
@pytest.mark.parametrize("policy", [kivi.KIVI_FLUSH_WINDOW, kivi.KIVI_FLUSH_ALG1], ids=["window", "alg1"])
@pytest.mark.parametrize("bits", [2, 4])
def test_streaming_small(path, policy, bits):
    torch = gh.require_gpu()
    w = scaled(CONFIGS["stream"], name="stream_small", batch=2, n_q_heads=4, n_kv_heads=2, bits=bits,
               residual=64, prompt=150, decode_steps=200, seed=4242 + bits)
    total = w.prompt + w.decode_steps
    k, v = workloads.keys(w, total), workloads.values(w, total)
    print(f"case streaming path={path} policy={policy} bits={bits}", flush=True)
    layout, cache = gh.gpu_prefill(w, k[:, :, :w.prompt], v[:, :, :w.prompt], policy, path,
                                   extra_q_tokens=w.decode_steps)
    oc = ko.StreamingCache(w.batch, w.n_kv_heads, 128, bits, w.group, w.residual,
                           "window" if policy == kivi.KIVI_FLUSH_WINDOW else "alg1")
    oc.prefill(k[:, :, :w.prompt], v[:, :, :w.prompt])
    gh.compare_quantized_state(cache, oc)
    kt, vt = torch.from_numpy(k).cuda(), torch.from_numpy(v).cuda()
    out = torch.empty(w.batch, w.n_q_heads, 128, dtype=torch.float32, device="cuda")
    worst = 0.0
    for step in range(w.decode_steps):
        t = w.prompt + step
        kivi.kivi_append_residual(layout, cache, kt[:, :, t].contiguous(), vt[:, :, t].contiguous())
        nk, nv = kivi.kivi_flush_residual(layout, cache, policy)
        onk, onv = oc.append(k[:, :, t], v[:, :, t])
        assert (nk, nv) == (onk, onv), f"step {step}"
        if nk or nv or step % 37 == 0:
            torch.cuda.synchronize()
            gh.compare_quantized_state(cache, oc)
        q = workloads.queries(w, step)
        kivi.kivi_decode_attention(layout, cache, torch.from_numpy(q).cuda(), w.softmax_scale, out)
        if step % 5 == 0 or nk or nv:
            got = out.cpu().numpy()
            worst = max(worst, gh.check_close(got, oc.attention(q, w.softmax_scale), f"step {step}"))
    print(f"streaming worst abs err {worst:.3e}", flush=True)


@pytest.mark.parametrize("path", [kivi.KIVI_DECODE_VALU, kivi.KIVI_DECODE_MFMA, kivi.KIVI_DECODE_MFMA_TWO], ids=["valu", "mfma", "mfma2"])
@pytest.mark.parametrize("policy", [kivi.KIVI_FLUSH_WINDOW, kivi.KIVI_FLUSH_ALG1], ids=["window", "alg1"])
@pytest.mark.parametrize("bits,rep,group", [(2, 1, 32), (4, 2, 32), (2, 4, 32), (2, 1, 64), (4, 1, 128), (2, 12, 32),
                                            (4, 4, 32), (4, 8, 64), (2, 8, 32)])
def test_decode_step_matches_oracle(path, policy, bits, rep, group):
    """kivi_decode_step (append + flush + attention, one launch on the steps without a flush in the
    matrix-core family): the residual rings must hold the new token afterwards (bit-exact cache
    at every step that is checked) and the outputs must match at every step."""
    torch = gh.require_gpu()
    w = scaled(CONFIGS["stream"], name="step_small", batch=2, n_q_heads=2 * rep, n_kv_heads=2, bits=bits,
               group=group, residual=max(64, group), prompt=101 + 2 * group, decode_steps=140 + group,
               seed=777 + bits + rep + group)
    total = w.prompt + w.decode_steps
    k, v = workloads.keys(w, total), workloads.values(w, total)
    print(f"case decode_step path={path} policy={policy} bits={bits} rep={rep} G={group}", flush=True)
    layout, cache = gh.gpu_prefill(w, k[:, :, :w.prompt], v[:, :, :w.prompt], policy, path,
                                   extra_q_tokens=w.decode_steps)
    oc = ko.StreamingCache(w.batch, w.n_kv_heads, 128, bits, w.group, w.residual,
                           "window" if policy == kivi.KIVI_FLUSH_WINDOW else "alg1")
    oc.prefill(k[:, :, :w.prompt], v[:, :, :w.prompt])
    gh.compare_quantized_state(cache, oc)
    kt, vt = torch.from_numpy(k).cuda(), torch.from_numpy(v).cuda()
    out = torch.empty(w.batch, w.n_q_heads, 128, dtype=torch.float32, device="cuda")
    worst = 0.0
    for step in range(w.decode_steps):
        t = w.prompt + step
        q = workloads.queries(w, step)
        k_new, v_new = kt[:, :, t].contiguous(), vt[:, :, t].contiguous()
        kivi.kivi_decode_step(layout, cache, k_new, v_new, torch.from_numpy(q).cuda(), w.softmax_scale, out, policy)
        onk, onv = oc.append(k[:, :, t], v[:, :, t])
        if step % 3 == 0 or onk or onv:
            torch.cuda.synchronize()
            gh.compare_quantized_state(cache, oc)
            worst = max(worst, gh.check_close(out.cpu().numpy(), oc.attention(q, w.softmax_scale), f"step {step}"))
    torch.cuda.synchronize()
    gh.compare_quantized_state(cache, oc)
    print(f"decode_step worst abs err {worst:.3e}", flush=True)


def test_decode_step_launch_form_changes_between_steps():
    """A batch on the automatic choice whose attention changes form from step to step: one launch
    right after a flush (a one-tile window), two launches once the window has grown into a second
    tile.  Both forms must leave the cache and the workspace as the other one expects them; two
    sequences of the batch are followed by the oracle."""
    torch = gh.require_gpu()
    rep, bits, policy = 8, 2, kivi.KIVI_FLUSH_WINDOW
    w = scaled(CONFIGS["stream"], name="form_flip", batch=24, n_q_heads=8 * rep, n_kv_heads=8, bits=bits,
               group=32, residual=32, prompt=690, decode_steps=70, seed=31337)
    total = w.prompt + w.decode_steps
    k, v = workloads.keys(w, total), workloads.values(w, total)
    print("case decode_step form flip", flush=True)
    layout, cache = gh.gpu_prefill(w, k[:, :, :w.prompt], v[:, :, :w.prompt], policy, kivi.KIVI_DECODE_AUTO,
                                   extra_q_tokens=w.decode_steps)
    sel = [3, 17]
    oc = ko.StreamingCache(len(sel), w.n_kv_heads, 128, bits, w.group, w.residual, "window")
    oc.prefill(k[sel, :, :w.prompt], v[sel, :, :w.prompt])
    kt, vt = torch.from_numpy(k).cuda(), torch.from_numpy(v).cuda()
    out = torch.empty(w.batch, w.n_q_heads, 128, dtype=torch.float32, device="cuda")
    forms, worst = set(), 0.0
    for step in range(w.decode_steps):
        t = w.prompt + step
        q = workloads.queries(w, step)
        kivi.kivi_decode_step(layout, cache, kt[:, :, t].contiguous(), vt[:, :, t].contiguous(),
                              torch.from_numpy(q).cuda(), w.softmax_scale, out, policy)
        forms.add(kivi.kivi_decode_plan(layout, cache).launches)      # the form this step's attention took
        oc.append(k[sel, :, t], v[sel, :, t])
        torch.cuda.synchronize()
        assert (cache.c.n_kq, cache.c.n_kr) == (oc.n_kq, oc.n_kr), f"step {step}"
        worst = max(worst, gh.check_close(out.cpu().numpy()[sel], oc.attention(q[sel], w.softmax_scale), f"step {step}"))
    assert forms == {1, 2}, forms
    print(f"form flip worst abs err {worst:.3e}", flush=True)
