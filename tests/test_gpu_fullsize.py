"""GPU parity at the five benchmark configurations' full sizes, in the launch configuration bench.py
times.  The whole batch runs on the GPU and the oracle recomputes every (batch, kv-head) unit,
block by block (bit-exact cache state, outputs within tolerance); only the streaming
configuration's per-step checks and the case beyond 4 GiB work on a sample of units."""
import numpy as np
import pytest

import gpu_harness as gh
from oracle import kivi_oracle as ko
from paper_2402_02750_amd import kivi, workloads
from paper_2402_02750_amd.workloads import CONFIGS

pytestmark = pytest.mark.gpu


def _sample_heads(w, n, seed):
    rng = np.random.default_rng(seed)
    allh = [(b, h) for b in range(w.batch) for h in range(w.n_kv_heads)]
    pick = rng.choice(len(allh), size=min(n, len(allh)), replace=False)
    heads = [allh[i] for i in sorted(pick)]
    for corner in (allh[0], allh[-1]):            # always include the first and the last unit
        if corner not in heads:
            heads.append(corner)
    return heads


PATHS = [("auto", kivi.KIVI_DECODE_AUTO), ("valu", kivi.KIVI_DECODE_VALU), ("mfma2", kivi.KIVI_DECODE_MFMA_TWO)]
UNIT_BLOCK = 64          # units the oracle holds at once (bounds its memory)


@pytest.mark.parametrize("name", ["llama7b", "llama13b_4bit", "mistral_gqa"])
def test_single_step_configs(name):
    """Benchmark configurations 2, 4 and 5: one decode step at the full shape, on all three decode
    paths.  EVERY (batch, kv-head) unit is compared with the oracle: packed codes, scales,
    zero-points and fp16 rows bit-exactly (the cache of the path bench.py times), outputs of every
    path within tolerance.  The oracle walks the units in blocks."""
    torch = gh.require_gpu()
    w = CONFIGS[name]
    print(f"case fullsize {name}: generating inputs", flush=True)
    k, v, q = workloads.keys(w, w.context), workloads.values(w, w.context), workloads.queries(w)
    n_q, n_r = w.split_single_step()
    outs = {}
    caches = {}
    for pname, path in PATHS:
        layout, cache = gh.gpu_prefill(w, k, v, kivi.KIVI_FLUSH_WINDOW, path)
        assert (cache.c.n_kq, cache.c.n_kr, cache.c.n_vq, cache.c.n_vr) == (n_q, n_r, n_q, n_r)
        outs[pname] = gh.gpu_attention(layout, cache, q, w.softmax_scale)
        assert np.isfinite(outs[pname]).all()
        caches[pname] = cache
        print(f"case fullsize {name}: path {pname} done on the GPU", flush=True)
    units = [(b, h) for b in range(w.batch) for h in range(w.n_kv_heads)]
    worst = dict.fromkeys(outs, 0.0)
    for i0 in range(0, len(units), UNIT_BLOCK):
        heads = units[i0:i0 + UNIT_BLOCK]
        oc = gh.oracle_cache_for_heads(w, k, v, heads, "window")
        gh.compare_quantized_state(caches["auto"], oc, heads)
        if i0 == 0:        # the quantise kernels do not depend on the decode path: one block for the others
            gh.compare_quantized_state(caches["valu"], oc, heads)
            gh.compare_quantized_state(caches["mfma2"], oc, heads)
        ref = gh.oracle_attention_for_heads(w, oc, q, heads)
        for pname in outs:
            worst[pname] = max(worst[pname], gh.check_close(gh.pick_heads(outs[pname], w, heads), ref,
                                                            f"{name} path {pname} units {i0}.."))
        print(f"case fullsize {name}: units {i0}..{i0 + len(heads) - 1} of {len(units)} ok, worst abs err {worst}", flush=True)


STREAM_ALL_UNIT_STEPS = (1, 31, 32, 33, 128, 256)
_stream_cache = {}


def _stream_inputs():
    """Keys and values of the streaming configuration (generated once for the tests of this module)."""
    if "kv" not in _stream_cache:
        w = CONFIGS["stream"]
        total = w.prompt + w.decode_steps
        print("case stream: generating inputs", flush=True)
        _stream_cache["kv"] = (workloads.keys(w, total), workloads.values(w, total))
    return _stream_cache["kv"]


def test_streaming_config3():
    """Benchmark configuration 3: batch 64, prompt 2048, 256 decode steps (kivi_decode_step) with a flush
    every 32 steps.  On a sample of units the cache state is compared bit-exactly after every flush
    and every 16th step (the rings must hold what the fused append stored) and the outputs at every
    step."""
    torch = gh.require_gpu()
    w = CONFIGS["stream"]
    k, v = _stream_inputs()
    layout, cache = gh.gpu_prefill(w, k[:, :, :w.prompt], v[:, :, :w.prompt], kivi.KIVI_FLUSH_WINDOW,
                                   kivi.KIVI_DECODE_AUTO, extra_q_tokens=w.decode_steps)
    heads = _sample_heads(w, 3, seed=2)
    oc = gh.oracle_cache_for_heads(w, k[:, :, :w.prompt], v[:, :, :w.prompt], heads, "window")
    gh.compare_quantized_state(cache, oc, heads)
    kt, vt = torch.from_numpy(k).cuda(), torch.from_numpy(v).cuda()
    out = torch.empty(w.batch, w.n_q_heads, 128, dtype=torch.float32, device="cuda")
    flushes, worst = [], 0.0
    for step in range(1, w.decode_steps + 1):
        t = w.prompt + step - 1
        q = workloads.queries(w, step)
        before = cache.c.n_kq
        # the call bench.py times: append + flush + attention, one launch on the steps without a flush
        kivi.kivi_decode_step(layout, cache, kt[:, :, t].contiguous(), vt[:, :, t].contiguous(),
                              torch.from_numpy(q).cuda(), w.softmax_scale, out, kivi.KIVI_FLUSH_WINDOW)
        nk = cache.c.n_kq - before
        knew = np.stack([k[b, h, t] for b, h in heads])[:, None]
        vnew = np.stack([v[b, h, t] for b, h in heads])[:, None]
        assert (nk, nk) == oc.append(knew, vnew)
        if nk or step % 16 == 1:
            if nk:
                flushes.append(step)
            torch.cuda.synchronize()
            gh.compare_quantized_state(cache, oc, heads)
        ref = gh.oracle_attention_for_heads(w, oc, q, heads)
        worst = max(worst, gh.check_close(gh.pick_heads(out.cpu().numpy(), w, heads), ref, f"step {step}"))
        if step % 32 == 0:
            print(f"case stream: step {step} ok, worst abs err so far {worst:.3e}", flush=True)
    assert flushes == [32, 64, 96, 128, 160, 192, 224, 256]
    assert (cache.c.n_kq, cache.c.n_kr) == (2176, 128)


def test_streaming_config3_all_units():
    """Benchmark configuration 3 once more, every unit: the 256 decode steps run on the GPU without
    a pause, the outputs of steps 1, 31, 32, 33, 128 and 256 are kept and compared for ALL 2048
    (batch, kv-head) units, and the final cache state of 64 units bit-exactly.  The oracle replays
    the stream block by block."""
    torch = gh.require_gpu()
    w = CONFIGS["stream"]
    k, v = _stream_inputs()
    layout, cache = gh.gpu_prefill(w, k[:, :, :w.prompt], v[:, :, :w.prompt], kivi.KIVI_FLUSH_WINDOW,
                                   kivi.KIVI_DECODE_AUTO, extra_q_tokens=w.decode_steps)
    kt, vt = torch.from_numpy(k).cuda(), torch.from_numpy(v).cuda()
    out = torch.empty(w.batch, w.n_q_heads, 128, dtype=torch.float32, device="cuda")
    kept = {}
    for step in range(1, w.decode_steps + 1):
        t = w.prompt + step - 1
        kivi.kivi_decode_step(layout, cache, kt[:, :, t].contiguous(), vt[:, :, t].contiguous(),
                              torch.from_numpy(workloads.queries(w, step)).cuda(), w.softmax_scale, out,
                              kivi.KIVI_FLUSH_WINDOW)
        if step in STREAM_ALL_UNIT_STEPS:
            kept[step] = out.cpu().numpy()
    torch.cuda.synchronize()
    assert (cache.c.n_kq, cache.c.n_kr) == (2176, 128)
    print("case stream all units: GPU steps done", flush=True)
    units = [(b, h) for b in range(w.batch) for h in range(w.n_kv_heads)]
    block, worst = 256, 0.0
    for i0 in range(0, len(units), block):
        hb = units[i0:i0 + block]
        ob = gh.oracle_cache_for_heads(w, k[:, :, :w.prompt], v[:, :, :w.prompt], hb, "window")
        for step in range(1, w.decode_steps + 1):
            t = w.prompt + step - 1
            ob.append(np.stack([k[b, h, t] for b, h in hb])[:, None], np.stack([v[b, h, t] for b, h in hb])[:, None])
            if step in STREAM_ALL_UNIT_STEPS:
                ref = gh.oracle_attention_for_heads(w, ob, workloads.queries(w, step), hb)
                worst = max(worst, gh.check_close(gh.pick_heads(kept[step], w, hb), ref, f"units {i0}.. step {step}"))
        if i0 == 0:
            ob64 = ko.StreamingCache(64, 1, w.head_dim, w.bits, w.group, w.residual, "window")
            for name_ in ("k_codes", "k_scale", "k_zero", "v_codes", "v_scale", "v_zero", "k_resid", "v_resid"):
                setattr(ob64, name_, getattr(ob, name_)[:64])
            gh.compare_quantized_state(cache, ob64, hb[:64])
        print(f"case stream all units: units {i0}..{i0 + len(hb) - 1} ok, worst abs err {worst:.3e}", flush=True)


def test_arrays_beyond_4GiB():
    """Maximum sizes: packed code arrays of 4.36 GB each and fp16 prefill inputs of 17.5 GB each, so
    that byte and element offsets pass 2^31 and 2^32 inside every kernel.  Inputs are drawn on the
    device (seeded torch generator, the workload's outlier-channel gains applied) because the host
    generator would need minutes; the sampled units' rows are copied back for the oracle.  Units
    0, 64 (beyond 2 GiB) and 127 (beyond 4 GiB) are compared bit-exactly and on their outputs."""
    torch = gh.require_gpu()
    free, _ = torch.cuda.mem_get_info()
    if free < 80e9:
        pytest.skip("needs 80 GB of free device memory")
    w = workloads.scaled(CONFIGS["llama13b_4bit"], name="beyond4g", batch=16, n_q_heads=8, n_kv_heads=8,
                         context=520 * 1024 + 128, seed=4242)
    T = w.context
    gen = torch.Generator(device="cuda").manual_seed(w.seed)
    gain = torch.from_numpy(np.stack([workloads.channel_gain(w, h) for h in range(w.n_kv_heads)])).cuda()
    print("case beyond4g: generating inputs on the device", flush=True)
    kt = torch.empty(w.batch, w.n_kv_heads, T, 128, dtype=torch.float16, device="cuda")
    vt = torch.empty_like(kt)
    for b in range(w.batch):
        kt[b] = (torch.randn(w.n_kv_heads, T, 128, generator=gen, device="cuda") * gain[:, None, :]).half()
        vt[b] = torch.randn(w.n_kv_heads, T, 128, generator=gen, device="cuda").half()
    heads = [(0, 0), (8, 0), (15, 7)]
    k_s = torch.stack([kt[b, h] for b, h in heads])[:, None].cpu().numpy()
    v_s = torch.stack([vt[b, h] for b, h in heads])[:, None].cpu().numpy()
    n_q, n_r = w.split_single_step()
    print("case beyond4g: oracle prefill of 3 units", flush=True)
    oc = ko.StreamingCache(len(heads), 1, 128, w.bits, w.group, w.residual, "window")
    oc.prefill(k_s, v_s)
    q = workloads.queries(w)
    ref = gh.oracle_attention_for_heads(w, oc, q, heads)
    for path in (kivi.KIVI_DECODE_AUTO, kivi.KIVI_DECODE_VALU, kivi.KIVI_DECODE_MFMA_TWO):
        print(f"case beyond4g: path {path}", flush=True)
        layout = kivi.make_layout(w.batch, w.n_q_heads, w.n_kv_heads, w.bits, w.residual, gh.round_up(T, 32), 192,
                                  decode_path=path)
        cache = kivi.Cache(layout)
        assert cache.buffers["k_codes"].numel() * cache.buffers["k_codes"].element_size() > 2 ** 32
        kivi.kivi_prefill(layout, kt, vt, T, cache, kivi.KIVI_FLUSH_WINDOW)
        torch.cuda.synchronize()
        assert (cache.c.n_kq, cache.c.n_kr) == (n_q, n_r)
        gh.compare_quantized_state(cache, oc, heads)
        out = gh.gpu_attention(layout, cache, q, w.softmax_scale)
        assert np.isfinite(out).all()
        err = gh.check_close(gh.pick_heads(out, w, heads), ref, f"beyond4g path {path}")
        print(f"case beyond4g: path {path} max abs err {err:.3e}", flush=True)
        del cache
