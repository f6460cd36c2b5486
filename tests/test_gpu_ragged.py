"""Batches whose sequences differ in length: per-sequence prefill through kivi_batch_slice, then
decoding steps through kivi_decode_step_ragged; every sequence against an oracle cache of its own
(bit-exact state, outputs within tolerance)."""
import ctypes

import numpy as np
import pytest

import gpu_harness as gh
from oracle import kivi_oracle as ko
from paper_2402_02750_amd import kivi, workloads
from paper_2402_02750_amd.workloads import CONFIGS, scaled

pytestmark = pytest.mark.gpu


class _SeqView:
    """Duck-typed stand-in for kivi.Cache over one sequence, for gh.compare_quantized_state."""

    def __init__(self, cache, b, state):
        self.cache, self.b, self.layout = cache, b, cache.layout
        self.c = state

    def view(self, name):
        return self.cache.view(name)[self.b:self.b + 1]


@pytest.mark.parametrize("path", [kivi.KIVI_DECODE_VALU, kivi.KIVI_DECODE_MFMA, kivi.KIVI_DECODE_MFMA_TWO], ids=["valu", "mfma", "mfma2"])
@pytest.mark.parametrize("policy", [kivi.KIVI_FLUSH_WINDOW, kivi.KIVI_FLUSH_ALG1], ids=["window", "alg1"])
def test_ragged_batch_steps(path, policy):
    torch = gh.require_gpu()
    prompts = [300, 300, 37, 1500, 0, 801]          # two equal neighbours, a short one, an empty slot
    steps = 70
    w = scaled(CONFIGS["stream"], name="ragged", batch=len(prompts), n_q_heads=4, n_kv_heads=2, residual=64,
               prompt=0, decode_steps=0, seed=606)
    total = max(prompts) + steps
    k, v = workloads.keys(w, total), workloads.values(w, total)
    layout = kivi.make_layout(w.batch, w.n_q_heads, w.n_kv_heads, w.bits, w.residual, gh.round_up(total, 32), 128,
                              decode_path=path)
    cache = kivi.Cache(layout)
    states = kivi.make_states(w.batch)
    kt, vt = torch.from_numpy(k).cuda(), torch.from_numpy(v).cuda()
    pol = "window" if policy == kivi.KIVI_FLUSH_WINDOW else "alg1"
    oracles = []
    print(f"case ragged path={path} policy={policy}: per-sequence prefill", flush=True)
    for b, n in enumerate(prompts):
        oc = ko.StreamingCache(1, w.n_kv_heads, 128, w.bits, w.group, w.residual, pol)
        if n:
            sl = kivi.CacheSlice(cache, b, 1)
            kivi.kivi_prefill(sl.layout, kt[b:b + 1], vt[b:b + 1], n, sl, policy)
            states[b] = sl.state()
            oc.prefill(k[b:b + 1, :, :n], v[b:b + 1, :, :n])
        oracles.append(oc)
    out = torch.zeros(w.batch, w.n_q_heads, 128, dtype=torch.float32, device="cuda")
    lengths = list(prompts)
    for step in range(steps):
        q = workloads.queries(w, step)
        # every sequence appends the token at its own position
        k_new = torch.stack([kt[b, :, lengths[b]] for b in range(w.batch)]).contiguous()
        v_new = torch.stack([vt[b, :, lengths[b]] for b in range(w.batch)]).contiguous()
        kivi.kivi_decode_step_ragged(layout, cache, states, k_new, v_new, torch.from_numpy(q).cuda(),
                                     w.softmax_scale, out, policy)
        torch.cuda.synchronize()
        got = out.cpu().numpy()
        for b in range(w.batch):
            oc = oracles[b]
            oc.append(k[b:b + 1, :, lengths[b]], v[b:b + 1, :, lengths[b]])
            lengths[b] += 1
            st = states[b]
            assert (st.n_kq, st.n_kr, st.n_vq, st.n_vr) == (oc.n_kq, oc.n_kr, oc.n_vq, oc.n_vr), f"step {step} seq {b}"
            gh.check_close(got[b:b + 1], oc.attention(q[b:b + 1], w.softmax_scale), f"step {step} seq {b}")
            if step % 16 == 15:
                gh.compare_quantized_state(_SeqView(cache, b, st), oc)
    # how the last step's attention was launched: one pair of launches for the whole batch where the
    # matrix-core family serves a batch whose sequences all split K and V alike, run by run otherwise
    launches = kivi.kivi_decode_launches_ragged(layout, states)
    if policy == kivi.KIVI_FLUSH_WINDOW and path != kivi.KIVI_DECODE_VALU:
        assert launches == 2
    else:
        assert launches >= 5
    # attention only, with one slot emptied: its rows of `out` stay as they are
    states[2] = kivi.kivi_seq_state_t()
    out.fill_(7.0)
    q = workloads.queries(w, steps)
    kivi.kivi_decode_attention_ragged(layout, cache, states, torch.from_numpy(q).cuda(), w.softmax_scale, out)
    torch.cuda.synchronize()
    got = out.cpu().numpy()
    assert (got[2] == 7.0).all()
    for b in (0, 1, 3, 4, 5):
        gh.check_close(got[b:b + 1], oracles[b].attention(q[b:b + 1], w.softmax_scale), f"final seq {b}")


@pytest.mark.parametrize("bits,rep", [(2, 2), (4, 1), (2, 4)])
def test_ragged_64_distinct_lengths(bits, rep):
    """64 sequences, all of different lengths (from shorter than the residual window, nothing
    quantised yet, to several chunks), decoded for 40 steps in one pair of attention launches per
    step: every sequence against an oracle cache of its own, outputs at every 4th step and after every
    flush, cache state at the end."""
    torch = gh.require_gpu()
    n_seq, steps = 64, 40
    prompts = [20 + 41 * i for i in range(n_seq)]            # 20 ... 2603, all distinct
    w = scaled(CONFIGS["stream"], name="ragged64", batch=n_seq, n_q_heads=2 * rep, n_kv_heads=2, bits=bits, residual=128,
               prompt=0, decode_steps=0, seed=707 + bits)
    total = max(prompts) + steps
    k, v = workloads.keys(w, total), workloads.values(w, total)
    layout = kivi.make_layout(w.batch, w.n_q_heads, w.n_kv_heads, w.bits, w.residual, gh.round_up(total, 32), 192)
    cache = kivi.Cache(layout)
    states = kivi.make_states(w.batch)
    kt, vt = torch.from_numpy(k).cuda(), torch.from_numpy(v).cuda()
    oracles = []
    print(f"case ragged64 bits={bits} rep={rep}: per-sequence prefill", flush=True)
    for b, n in enumerate(prompts):
        oc = ko.StreamingCache(1, w.n_kv_heads, 128, w.bits, w.group, w.residual, "window")
        sl = kivi.CacheSlice(cache, b, 1)
        kivi.kivi_prefill(sl.layout, kt[b:b + 1], vt[b:b + 1], n, sl, kivi.KIVI_FLUSH_WINDOW)
        states[b] = sl.state()
        oc.prefill(k[b:b + 1, :, :n], v[b:b + 1, :, :n])
        oracles.append(oc)
    out = torch.zeros(w.batch, w.n_q_heads, 128, dtype=torch.float32, device="cuda")
    lengths = list(prompts)
    worst = 0.0
    for step in range(steps):
        q = workloads.queries(w, step)
        k_new = torch.stack([kt[b, :, lengths[b]] for b in range(w.batch)]).contiguous()
        v_new = torch.stack([vt[b, :, lengths[b]] for b in range(w.batch)]).contiguous()
        before = [states[b].n_kq for b in range(w.batch)]
        kivi.kivi_decode_step_ragged(layout, cache, states, k_new, v_new, torch.from_numpy(q).cuda(),
                                     w.softmax_scale, out, kivi.KIVI_FLUSH_WINDOW)
        torch.cuda.synchronize()
        assert kivi.kivi_decode_launches_ragged(layout, states) == 2       # the whole batch in one pair of launches
        got = out.cpu().numpy()
        for b in range(w.batch):
            oc = oracles[b]
            oc.append(k[b:b + 1, :, lengths[b]], v[b:b + 1, :, lengths[b]])
            lengths[b] += 1
            st = states[b]
            assert (st.n_kq, st.n_kr, st.n_vq, st.n_vr) == (oc.n_kq, oc.n_kr, oc.n_vq, oc.n_vr), f"step {step} seq {b}"
            if step % 4 == 0 or st.n_kq != before[b] or step == steps - 1:
                worst = max(worst, gh.check_close(got[b:b + 1], oc.attention(q[b:b + 1], w.softmax_scale), f"step {step} seq {b}"))
        if step % 10 == 9:
            print(f"case ragged64: step {step} ok, worst abs err {worst:.3e}", flush=True)
    for b in range(w.batch):
        gh.compare_quantized_state(_SeqView(cache, b, states[b]), oracles[b])


@pytest.mark.parametrize("batch,n_q_heads,n_kv_heads", [(300, 2, 1), (6, 32, 2), (256, 16, 8)],
                         ids=["batch300", "16_heads_per_kv_head", "2048_units"])
def test_ragged_wide_batches_and_groups(batch, n_q_heads, n_kv_heads):
    """The one-pair form past its internal piece sizes: more sequences than one host-to-device piece
    of counters holds (256), and more query heads per kv-head than one launch serves (8: a pair of
    launches per group of 8).  Attention only, every sequence against an oracle cache of its own."""
    torch = gh.require_gpu()
    rng = np.random.default_rng(batch)
    prompts = [int(x) for x in rng.integers(1, 700, size=batch)]
    prompts[0] = 1                                  # one fp16 row, nothing quantised
    prompts[-1] = 699
    if batch * n_kv_heads >= 2048:
        # as many units as the chip holds wavefronts and every sequence with quantised tokens: the
        # second launch gives every wavefront whole units, each with its own sequence's length
        prompts = [max(x, 100) for x in prompts]
    w = scaled(CONFIGS["stream"], name="raggedwide", batch=batch, n_q_heads=n_q_heads, n_kv_heads=n_kv_heads, residual=64,
               prompt=0, decode_steps=0, seed=808 + batch)
    total = max(prompts)
    k, v = workloads.keys(w, total), workloads.values(w, total)
    layout = kivi.make_layout(w.batch, w.n_q_heads, w.n_kv_heads, w.bits, w.residual, gh.round_up(total, 32), 128)
    cache = kivi.Cache(layout)
    states = kivi.make_states(w.batch)
    kt, vt = torch.from_numpy(k).cuda(), torch.from_numpy(v).cuda()
    oracles = []
    print(f"case raggedwide batch={batch} heads={n_q_heads}/{n_kv_heads}: per-sequence prefill", flush=True)
    for b, n in enumerate(prompts):
        oc = ko.StreamingCache(1, w.n_kv_heads, 128, w.bits, w.group, w.residual, "window")
        sl = kivi.CacheSlice(cache, b, 1)
        kivi.kivi_prefill(sl.layout, kt[b:b + 1], vt[b:b + 1], n, sl, kivi.KIVI_FLUSH_WINDOW)
        states[b] = sl.state()
        oc.prefill(k[b:b + 1, :, :n], v[b:b + 1, :, :n])
        oracles.append(oc)
    groups = -(-(n_q_heads // n_kv_heads) // 8)
    assert kivi.kivi_decode_launches_ragged(layout, states) == 2 * groups
    q = workloads.queries(w, 0)
    out = torch.zeros(w.batch, w.n_q_heads, 128, dtype=torch.float32, device="cuda")
    kivi.kivi_decode_attention_ragged(layout, cache, states, torch.from_numpy(q).cuda(), w.softmax_scale, out)
    torch.cuda.synchronize()
    got = out.cpu().numpy()
    worst = 0.0
    for b in range(w.batch):
        worst = max(worst, gh.check_close(got[b:b + 1], oracles[b].attention(q[b:b + 1], w.softmax_scale), f"seq {b} (n={prompts[b]})"))
    print(f"case raggedwide: worst abs err {worst:.3e}", flush=True)


@pytest.mark.parametrize("bits,rep", [(2, 1), (4, 2), (2, 4)])
def test_ragged_very_different_lengths(bits, rep):
    """768 units whose sequences run from 40 to 6000 tokens: the padded plan would waste more than
    14 000 four-tile group steps, so the second launch runs as equally long slices of the unit-major
    axis, one per wavefront, with the units that several slices share merged through the workspace.
    Two decoding steps and an attention call, every sequence against an oracle cache of its own."""
    torch = gh.require_gpu()
    n_seq, n_kv = 48, 16
    rng = np.random.default_rng(40 + bits + rep)
    prompts = [int(x) for x in rng.integers(40, 6000, size=n_seq)]
    prompts[0], prompts[1], prompts[-1] = 6000, 97, 5999
    groups = [-(-((n - 64) // 32) // 4) for n in prompts]
    assert n_seq * n_kv * max(groups) - n_kv * sum(groups) >= 14000        # the condition for the sliced form
    w = scaled(CONFIGS["stream"], name="raggedslices", batch=n_seq, n_q_heads=n_kv * rep, n_kv_heads=n_kv, bits=bits,
               residual=64, prompt=0, decode_steps=0, seed=909 + bits + rep)
    steps = 2
    total = max(prompts) + steps
    k, v = workloads.keys(w, total), workloads.values(w, total)
    layout = kivi.make_layout(w.batch, w.n_q_heads, w.n_kv_heads, w.bits, w.residual, gh.round_up(total, 32), 128)
    cache = kivi.Cache(layout)
    states = kivi.make_states(w.batch)
    kt, vt = torch.from_numpy(k).cuda(), torch.from_numpy(v).cuda()
    oracles = []
    print(f"case raggedslices bits={bits} rep={rep}: per-sequence prefill", flush=True)
    for b, n in enumerate(prompts):
        oc = ko.StreamingCache(1, w.n_kv_heads, 128, w.bits, w.group, w.residual, "window")
        sl = kivi.CacheSlice(cache, b, 1)
        kivi.kivi_prefill(sl.layout, kt[b:b + 1], vt[b:b + 1], n, sl, kivi.KIVI_FLUSH_WINDOW)
        states[b] = sl.state()
        oc.prefill(k[b:b + 1, :, :n], v[b:b + 1, :, :n])
        oracles.append(oc)
    out = torch.zeros(w.batch, w.n_q_heads, 128, dtype=torch.float32, device="cuda")
    lengths = list(prompts)
    worst = 0.0
    for step in range(steps + 1):
        q = workloads.queries(w, step)
        if step < steps:
            k_new = torch.stack([kt[b, :, lengths[b]] for b in range(w.batch)]).contiguous()
            v_new = torch.stack([vt[b, :, lengths[b]] for b in range(w.batch)]).contiguous()
            kivi.kivi_decode_step_ragged(layout, cache, states, k_new, v_new, torch.from_numpy(q).cuda(),
                                         w.softmax_scale, out, kivi.KIVI_FLUSH_WINDOW)
            for b in range(w.batch):
                oracles[b].append(k[b:b + 1, :, lengths[b]], v[b:b + 1, :, lengths[b]])
                lengths[b] += 1
        else:
            kivi.kivi_decode_attention_ragged(layout, cache, states, torch.from_numpy(q).cuda(), w.softmax_scale, out)
        torch.cuda.synchronize()
        assert kivi.kivi_decode_launches_ragged(layout, states) == 2
        got = out.cpu().numpy()
        for b in range(w.batch):
            worst = max(worst, gh.check_close(got[b:b + 1], oracles[b].attention(q[b:b + 1], w.softmax_scale), f"step {step} seq {b}"))
        print(f"case raggedslices: step {step} ok, worst abs err {worst:.3e}", flush=True)
