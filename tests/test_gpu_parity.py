"""GPU parity: the HIP path (through the C ABI) against the oracle on the same seeded inputs.

Bar: packed codes, scales, zero-points and residual rows bit-exact; attention outputs within
|gpu - ref| <= 2e-3 + 1e-2 |ref| element-wise.
"""
import numpy as np
import pytest

import gpu_harness as gh
from oracle import kivi_oracle as ko
from paper_2402_02750_amd import kivi, workloads
from paper_2402_02750_amd.workloads import CONFIGS, scaled

pytestmark = pytest.mark.gpu

PATHS = [kivi.KIVI_DECODE_VALU, kivi.KIVI_DECODE_MFMA, kivi.KIVI_DECODE_MFMA_TWO]
RANDOM_PATHS = PATHS + [kivi.KIVI_DECODE_MFMA_ONE]
PATH_IDS = ["valu", "mfma", "mfma2"]


def _run_case(w, length, policy, path, heads=None, units_per_kv_head=None):
    torch = gh.require_gpu()
    k = workloads.keys(w, length)
    v = workloads.values(w, length)
    q = workloads.queries(w)
    layout, cache = gh.gpu_prefill(w, k, v, policy, path)
    if units_per_kv_head is not None:
        assert kivi.kivi_decode_plan(layout, cache).units_per_kv_head == units_per_kv_head
    all_heads = [(b, h) for b in range(w.batch) for h in range(w.n_kv_heads)]
    heads = all_heads if heads is None else heads
    oc = gh.oracle_cache_for_heads(w, k, v, heads, "window" if policy == kivi.KIVI_FLUSH_WINDOW else "alg1")
    gh.compare_quantized_state(cache, oc, heads)
    out = gh.gpu_attention(layout, cache, q, w.softmax_scale)
    ref = gh.oracle_attention_for_heads(w, oc, q, heads)
    return gh.check_close(gh.pick_heads(out, w, heads), ref, f"{w.name} L={length}")


@pytest.mark.parametrize("path", PATHS, ids=PATH_IDS)
def test_config1_tiny(path):
    """Benchmark configuration 1: batch 1, 4 heads, context 1024, 2-bit, R=32."""
    w = CONFIGS["tiny"]
    print(f"case tiny path={path}", flush=True)
    _run_case(w, w.context, kivi.KIVI_FLUSH_WINDOW, path)


@pytest.mark.parametrize("path", PATHS, ids=PATH_IDS)
@pytest.mark.parametrize("bits", [2, 4])
@pytest.mark.parametrize("length", [1, 31, 32, 33, 127, 160, 161, 700, 2085])
def test_lengths_and_ragged_tails(path, bits, length):
    """Contexts shorter than R (nothing quantised), exactly at tile borders, and with ragged
    residual tails; several splits at the long end."""
    w = scaled(CONFIGS["llama7b"], name="small", batch=2, n_q_heads=3, n_kv_heads=3, bits=bits, seed=77 + bits)
    print(f"case lengths path={path} bits={bits} L={length}", flush=True)
    _run_case(w, length, kivi.KIVI_FLUSH_WINDOW, path)


@pytest.mark.parametrize("path", PATHS, ids=PATH_IDS)
@pytest.mark.parametrize("bits", [2, 4])
@pytest.mark.parametrize("rep", [2, 3, 4, 5, 7, 8])
def test_grouped_query(path, bits, rep):
    """2 to 8 query heads per kv-head (8: the 64-query / 8-kv shape of the 70B Llama models; 3, 5
    and 7 run on the next larger instantiation with the surplus heads idle); several workgroups
    per unit, so the cross-workgroup merge runs."""
    w = scaled(CONFIGS["mistral_gqa"], name="gqa_small", batch=2, n_q_heads=2 * rep, n_kv_heads=2, bits=bits,
               seed=500 + rep + bits)
    print(f"case gqa path={path} bits={bits} rep={rep}", flush=True)
    _run_case(w, 1500, kivi.KIVI_FLUSH_WINDOW, path)
    _run_case(w, 6000, kivi.KIVI_FLUSH_ALG1, path, heads=[(0, 1), (1, 0)])


@pytest.mark.parametrize("bits,group,batch,n_kv,length", [(2, 64, 256, 8, 330), (4, 128, 256, 8, 520)], ids=["G64", "G128"])
def test_many_units_larger_groups(bits, group, batch, n_kv, length):
    """The one-unit-per-wavefront kernel with G = 64 / 128 (one scale / zero-point pair per group in
    memory): every unit against the oracle, state bit-exact."""
    w = scaled(CONFIGS["stream"], name="many_units_g", batch=batch, n_q_heads=n_kv, n_kv_heads=n_kv, bits=bits,
               group=group, residual=group, seed=2700 + group)
    print(f"case many_units_g bits={bits} G={group} units={batch * n_kv} L={length}", flush=True)
    _run_case(w, length, kivi.KIVI_FLUSH_WINDOW, kivi.KIVI_DECODE_AUTO)


@pytest.mark.parametrize("bits,rep,batch,n_kv,length", [
    (2, 1, 256, 8, 300),      # 2048 units = one per resident wavefront; 7 all-quantised tiles (a short last group of 3)
    (4, 1, 272, 8, 200),      # 2176 units: a second, sparse round of units; 4 tiles
    (2, 2, 128, 16, 166),     # two query heads per kv-head; 3 tiles (fewer than one group)
    (4, 2, 256, 8, 420),
    (2, 4, 256, 8, 260),      # four query heads per kv-head
    (2, 3, 256, 8, 230),      # three heads on the four-head instantiation
    (2, 16, 256, 8, 200),     # 16 heads per kv-head: two passes of eight on the shared-unit form
], ids=["u2048_b2", "u2176_b4", "rep2_b2", "rep2_b4", "rep4_b2", "rep3_b2", "rep16_b2"])
def test_many_units_one_per_wavefront(bits, rep, batch, n_kv, length):
    """Batches with at least as many (batch, kv-head) units as the chip holds wavefronts: the second
    launch of the two-launch form gives every wavefront whole units (decode_wave_units_kernel; with
    more than four heads per launch the shared-unit form).  Every unit against the oracle, state bit-exact."""
    w = scaled(CONFIGS["stream"], name="many_units", batch=batch, n_q_heads=n_kv * rep, n_kv_heads=n_kv, bits=bits,
               residual=64, seed=2600 + bits + rep)
    print(f"case many_units bits={bits} rep={rep} units={batch * n_kv} L={length}", flush=True)
    _run_case(w, length, kivi.KIVI_FLUSH_WINDOW, kivi.KIVI_DECODE_AUTO)
    _run_case(w, length, kivi.KIVI_FLUSH_WINDOW, kivi.KIVI_DECODE_MFMA_TWO)


@pytest.mark.parametrize("path", PATHS, ids=PATH_IDS)
@pytest.mark.parametrize("bits", [2, 4])
@pytest.mark.parametrize("n_kv,rep", [(2, 9), (2, 16), (1, 71)])
def test_wide_groups(path, bits, n_kv, rep):
    """More than 8 query heads per kv-head (9, 16, and 71 heads on a single kv-head = the multi-query
    shape of Falcon-7B): runs of 4 heads as units of one launch in the matrix-core family's
    single-launch form (the last run shorter: 9 = 4 + 4 + 1, 71 = 17 x 4 + 3), one launch per 8 heads
    in the forced two-launch form and in the vector-ALU family."""
    w = scaled(CONFIGS["mistral_gqa"], name="wide", batch=2, n_q_heads=n_kv * rep, n_kv_heads=n_kv, bits=bits,
               seed=1500 + rep + bits)
    print(f"case wide path={path} bits={bits} kv={n_kv} rep={rep}", flush=True)
    _run_case(w, 1500, kivi.KIVI_FLUSH_WINDOW, path)
    _run_case(w, 3100, kivi.KIVI_FLUSH_ALG1, path)


@pytest.mark.parametrize("path", PATHS, ids=PATH_IDS)
@pytest.mark.parametrize("residual", [0, 32, 96])
def test_residual_lengths(path, residual):
    w = scaled(CONFIGS["llama7b"], name="resid", batch=1, n_q_heads=2, n_kv_heads=2, residual=residual, seed=900)
    print(f"case residual path={path} R={residual}", flush=True)
    _run_case(w, 640 + 17, kivi.KIVI_FLUSH_WINDOW, path)


@pytest.mark.parametrize("path", PATHS, ids=PATH_IDS)
@pytest.mark.parametrize("bits", [2, 4])
@pytest.mark.parametrize("length", [100, 200, 333, 1030])
def test_alg1_split(path, bits, length):
    """Algorithm 1's literal prefill: keys keep l % R tokens in fp16, values keep R, so the K and
    V splits differ and the value part ends inside a tile."""
    w = scaled(CONFIGS["llama7b"], name="alg1", batch=1, n_q_heads=2, n_kv_heads=2, bits=bits, seed=1200 + bits)
    print(f"case alg1 path={path} bits={bits} L={length}", flush=True)
    _run_case(w, length, kivi.KIVI_FLUSH_ALG1, path)


@pytest.mark.parametrize("path", PATHS, ids=PATH_IDS)
@pytest.mark.parametrize("bits", [2, 4])
@pytest.mark.parametrize("group,residual,length", [(64, 64, 777), (64, 128, 1500), (128, 128, 1100), (128, 0, 640)])
def test_larger_groups(path, bits, group, residual, length):
    """G = 64 and 128 (the group sizes of the paper's ablation, Table 5 / Appendix): keys grouped
    over G tokens, values over G channels; codes, scales and zero-points bit-exact, outputs in
    tolerance.  (Scales and zero-points are stored per 32-token tile / 32-channel block, replicated.)"""
    w = scaled(CONFIGS["llama7b"], name=f"g{group}", batch=2, n_q_heads=2, n_kv_heads=2, bits=bits,
               group=group, residual=residual, seed=4000 + group + bits)
    print(f"case group path={path} bits={bits} G={group} R={residual} L={length}", flush=True)
    _run_case(w, length, kivi.KIVI_FLUSH_WINDOW, path)
    if residual:
        _run_case(w, length, kivi.KIVI_FLUSH_ALG1, path)


@pytest.mark.parametrize("bits", [2, 4])
@pytest.mark.parametrize("value_pieces", [((0, 5), (5, 27), (32, 1), (33, 70), (103, 89)),
                                          ((0, 70), (70, 26), (96, 96))], ids=["ragged_pieces", "whole_tiles_and_tails"])
def test_quantize_entry_points_append_in_pieces(bits, value_pieces):
    """kivi_quantize_key_groups / kivi_quantize_value_tokens called piecewise (strided sources,
    value pieces that end inside a tile, and pieces of whole tiles followed by a partly filled one:
    the one-wavefront-per-tile kernels and the general ones write into the same tiles) build the same
    cache as one call."""
    torch = gh.require_gpu()
    w = scaled(CONFIGS["llama7b"], name="pieces", batch=2, n_q_heads=2, n_kv_heads=2, bits=bits, seed=31)
    n = 192
    k = workloads.keys(w, n)
    v = workloads.values(w, n)
    layout = kivi.make_layout(w.batch, w.n_q_heads, w.n_kv_heads, w.bits, w.residual, 256, 192)
    cache = kivi.Cache(layout)
    # sources with padded token stride and swapped (h, b) memory order
    def strided(x):
        t = torch.zeros(w.n_kv_heads, w.batch, n, 136, dtype=torch.float16, device="cuda")
        t[..., :128] = torch.from_numpy(x).cuda().permute(1, 0, 2, 3)
        return t.permute(1, 0, 2, 3)[..., :128]
    kt, vt = strided(k), strided(v)
    for start, cnt in ((0, 64), (64, 32), (96, 96)):
        kivi.kivi_quantize_key_groups(layout, kt[:, :, start:], cnt, cache)
    for start, cnt in value_pieces:
        kivi.kivi_quantize_value_tokens(layout, vt[:, :, start:], cnt, cache)
    torch.cuda.synchronize()
    assert (cache.c.n_kq, cache.c.n_vq) == (n, n)
    ck, sk, zk = ko.quantize_key(k, w.bits, w.group)
    cv, sv, zv = ko.quantize_value(v, w.bits, w.group)
    assert np.array_equal(cache.view("k_codes")[:, :, :6].cpu().numpy().view(np.uint32), ko.pack_key_codes(ck, w.bits))
    assert np.array_equal(cache.view("v_codes")[:, :, :6].cpu().numpy().view(np.uint32), ko.pack_value_codes(cv, w.bits))
    assert np.array_equal(cache.view("k_scale")[:, :, :6].cpu().numpy().view(np.uint16), sk.view(np.uint16))
    assert np.array_equal(cache.view("k_zero")[:, :, :6].cpu().numpy().view(np.uint16), zk.view(np.uint16))
    assert np.array_equal(cache.view("v_scale")[:, :, :n].cpu().numpy().view(np.uint16), sv.view(np.uint16))
    assert np.array_equal(cache.view("v_zero")[:, :, :n].cpu().numpy().view(np.uint16), zv.view(np.uint16))


def test_quantizer_edge_values_bit_exact():
    """Ties, constant groups, fp16 subnormal ranges and large magnitudes through the GPU quantiser."""
    torch = gh.require_gpu()
    rng = np.random.default_rng(5)
    n = 64
    k = np.zeros((1, 1, n, 128), np.float16)
    k[0, 0, :, 0:16] = (rng.integers(-8, 9, size=(n, 16)) * 0.25)           # exact ties
    k[0, 0, :, 16:32] = 0.75                                                 # constant groups
    k[0, 0, :, 32:48] = (rng.integers(0, 6, size=(n, 16)) * 2.0 ** -24)      # subnormal ranges
    k[0, 0, :, 48:64] = rng.standard_normal((n, 16)) * 3000                  # large magnitudes
    k[0, 0, :, 64:] = rng.standard_normal((n, 64)) * 1e-3
    v = np.ascontiguousarray(k[:, :, :, ::-1])
    for bits in (2, 4):
        layout = kivi.make_layout(1, 1, 1, bits, 32, 64, 96)
        cache = kivi.Cache(layout)
        kivi.kivi_quantize_key_groups(layout, torch.from_numpy(k).cuda(), n, cache)
        kivi.kivi_quantize_value_tokens(layout, torch.from_numpy(v).cuda(), n, cache)
        torch.cuda.synchronize()
        ck, sk, zk = ko.quantize_key(k, bits, 32)
        cv, sv, zv = ko.quantize_value(v, bits, 32)
        assert np.array_equal(cache.view("k_scale").cpu().numpy().view(np.uint16), sk.view(np.uint16))
        assert np.array_equal(cache.view("k_zero").cpu().numpy().view(np.uint16), zk.view(np.uint16))
        assert np.array_equal(cache.view("k_codes").cpu().numpy().view(np.uint32), ko.pack_key_codes(ck, bits))
        assert np.array_equal(cache.view("v_scale").cpu().numpy().view(np.uint16), sv.view(np.uint16))
        assert np.array_equal(cache.view("v_zero").cpu().numpy().view(np.uint16), zv.view(np.uint16))
        assert np.array_equal(cache.view("v_codes").cpu().numpy().view(np.uint32), ko.pack_value_codes(cv, bits))


@pytest.mark.parametrize("path", PATHS, ids=PATH_IDS)
def test_run_twice_is_deterministic(path):
    torch = gh.require_gpu()
    w = scaled(CONFIGS["llama7b"], name="det", batch=2, n_q_heads=4, n_kv_heads=4, seed=3)
    k, v, q = workloads.keys(w, 900), workloads.values(w, 900), workloads.queries(w)
    layout, cache = gh.gpu_prefill(w, k, v, kivi.KIVI_FLUSH_WINDOW, path)
    a = gh.gpu_attention(layout, cache, q, w.softmax_scale)
    b = gh.gpu_attention(layout, cache, q, w.softmax_scale)
    assert np.array_equal(a, b)


@pytest.mark.parametrize("path", PATHS, ids=PATH_IDS)
@pytest.mark.parametrize("bits", [2, 4])
def test_probability_accuracy_with_one_hot_values(path, bits):
    """Tighter than the gate: with one-hot value rows the output is the softmax probability of
    each token, so a lost low-order part of the small matrix operand (an error of ~2e-4 in a
    probability) shows up directly.  Probabilities above 1e-3 must be within 5e-5 relative."""
    torch = gh.require_gpu()
    w = scaled(CONFIGS["llama7b"], name="onehot", batch=1, n_q_heads=1, n_kv_heads=1, bits=bits, residual=0, seed=5)
    L = 128
    k = workloads.keys(w, L)
    q = (workloads.queries(w).astype(np.float32) * 0.25).astype(np.float16)
    v = np.zeros((1, 1, L, 128), np.float16)
    v[0, 0, np.arange(L), np.arange(L)] = 1.0
    layout, cache = gh.gpu_prefill(w, k, v, kivi.KIVI_FLUSH_WINDOW, path)
    oc = gh.oracle_cache_for_heads(w, k, v, [(0, 0)], "window")
    out = gh.gpu_attention(layout, cache, q, w.softmax_scale)[0, 0].astype(np.float64)
    ref = gh.oracle_attention_for_heads(w, oc, q, [(0, 0)])[0, 0]
    big = ref > 1e-3
    assert big.sum() > 50
    assert np.abs(out[big] / ref[big] - 1).max() < 5e-5


@pytest.mark.parametrize("bits,rep", [(2, 8), (2, 5), (4, 3), (4, 4), (4, 8)])
@pytest.mark.parametrize("batch,n_kv,length,residual", [(1, 2, 1500, 128), (3, 8, 4200, 128), (2, 5, 700, 192),
                                                        (40, 8, 1100, 96), (70, 8, 600, 64)])
def test_single_launch_weighted_rows(bits, rep, batch, n_kv, length, residual):
    """The single-launch form on the instantiations whose fp16-row chunks weigh two all-quantised
    chunks on the work axis: from fewer chunks than workgroups (every chunk a workgroup of its
    own, a unit's parts merged over a dozen workgroups) to workgroups that own parts of several
    units."""
    w = scaled(CONFIGS["llama7b"], name="rows2", batch=batch, n_q_heads=n_kv * rep, n_kv_heads=n_kv, bits=bits,
               residual=residual, seed=500 + bits + rep)
    rng = np.random.default_rng(batch * 131 + n_kv)
    all_heads = [(b, h) for b in range(w.batch) for h in range(w.n_kv_heads)]
    heads = [all_heads[i] for i in rng.choice(len(all_heads), size=min(3, len(all_heads)), replace=False)]
    print(f"case single-launch rows bits={bits} rep={rep} b={batch} kv={n_kv} L={length} R={residual} heads={heads}", flush=True)
    _run_case(w, length, kivi.KIVI_FLUSH_WINDOW, kivi.KIVI_DECODE_MFMA_ONE, heads=heads)


@pytest.mark.parametrize("path", [kivi.KIVI_DECODE_MFMA, kivi.KIVI_DECODE_MFMA_ONE], ids=["mfma", "mfma1"])
@pytest.mark.parametrize("bits", [2, 4])
@pytest.mark.parametrize("rep", [4, 6, 8])
@pytest.mark.parametrize("batch,n_kv,length,residual,policy", [
    (1, 8, 1500, 128, kivi.KIVI_FLUSH_WINDOW), (3, 2, 5000, 128, kivi.KIVI_FLUSH_WINDOW),
    (2, 8, 700, 32, kivi.KIVI_FLUSH_ALG1), (5, 3, 333, 64, kivi.KIVI_FLUSH_WINDOW), (1, 1, 40, 32, kivi.KIVI_FLUSH_WINDOW)])
def test_query_head_halves_as_units(path, bits, rep, batch, n_kv, length, residual, policy):
    """Small batches with 4, 6 or 8 query heads per kv-head: halves (quarters of 8 heads at 2 bits
    and up to 16 units) of every group are units of their own on the instantiation for a part's
    heads (the plan says so; 4 heads at 2 bits only),
    each reading the kv-head's cache -- one unit spread over many workgroups, several units in one
    workgroup, fp16 rows only."""
    w = scaled(CONFIGS["llama7b"], name="halves", batch=batch, n_q_heads=n_kv * rep, n_kv_heads=n_kv, bits=bits,
               residual=residual, seed=900 + bits + rep)
    print(f"case head halves path={path} bits={bits} rep={rep} b={batch} kv={n_kv} L={length} R={residual}", flush=True)
    expect = 1 if (rep == 4 and bits == 4) else (4 if (rep == 8 and bits == 2 and batch * n_kv <= 16) else 2)
    _run_case(w, length, policy, path, units_per_kv_head=expect)


@pytest.mark.parametrize("seed", range(36))
def test_random_shapes(seed):
    """Seeded random layouts (batch, heads, query heads per kv-head, bits, G, R, context length,
    policy, kernel family): the work partition, the part merging and the fp16 / quantised split
    points land on different corner cases every time; sampled (batch, kv-head) units against the
    oracle."""
    rng = np.random.default_rng(9000 + seed)
    group = int(rng.choice([32, 32, 64, 128]))
    residual = group * int(rng.integers(0, 256 // group + 1))
    rep = int(rng.choice([1, 1, 2, 3, 4, 8, 12]))
    n_kv = int(rng.integers(1, 6))
    w = scaled(CONFIGS["llama7b"], name=f"rand{seed}", batch=int(rng.integers(1, 6)), n_q_heads=n_kv * rep,
               n_kv_heads=n_kv, bits=int(rng.choice([2, 4])), group=group, residual=residual, seed=12000 + seed)
    length = int(rng.choice([rng.integers(1, 200), rng.integers(200, 3000), rng.integers(3000, 9000)]))
    policy = kivi.KIVI_FLUSH_WINDOW if residual == 0 or rng.integers(0, 2) else kivi.KIVI_FLUSH_ALG1
    path = RANDOM_PATHS[int(rng.integers(0, len(RANDOM_PATHS)))]
    all_heads = [(b, h) for b in range(w.batch) for h in range(w.n_kv_heads)]
    heads = [all_heads[i] for i in rng.choice(len(all_heads), size=min(3, len(all_heads)), replace=False)]
    print(f"case random seed={seed} b={w.batch} kv={n_kv} rep={rep} bits={w.bits} G={group} R={residual} "
          f"L={length} policy={policy} path={path} heads={heads}", flush=True)
    _run_case(w, length, policy, path, heads=heads)


@pytest.mark.parametrize("seed", range(10))
def test_random_large_batches(seed):
    """Seeded random layouts with hundreds to thousands of (batch, kv-head) units (short contexts):
    the two-launch form with the one-unit-per-wavefront kernel where the unit count fits it, the
    shared-unit form where it does not, G = 32 / 64 / 128; sampled units against the oracle."""
    rng = np.random.default_rng(9500 + seed)
    group = int(rng.choice([32, 32, 64, 128]))
    residual = group * int(rng.integers(1, 256 // group + 1))
    rep = int(rng.choice([1, 1, 2, 3, 4, 8]))
    n_kv = int(rng.choice([2, 4, 8]))
    batch = int(rng.integers(256, 620))
    w = scaled(CONFIGS["llama7b"], name=f"randbig{seed}", batch=batch, n_q_heads=n_kv * rep, n_kv_heads=n_kv,
               bits=int(rng.choice([2, 4])), group=group, residual=residual, seed=12500 + seed)
    length = int(rng.integers(1, 700))
    policy = kivi.KIVI_FLUSH_WINDOW if rng.integers(0, 3) else kivi.KIVI_FLUSH_ALG1
    path = [kivi.KIVI_DECODE_AUTO, kivi.KIVI_DECODE_MFMA_TWO, kivi.KIVI_DECODE_MFMA_ONE][int(rng.integers(0, 3))]
    all_heads = [(b, h) for b in range(w.batch) for h in range(w.n_kv_heads)]
    heads = [all_heads[i] for i in rng.choice(len(all_heads), size=6, replace=False)]
    print(f"case random large seed={seed} b={w.batch} kv={n_kv} rep={rep} bits={w.bits} G={group} R={residual} "
          f"L={length} policy={policy} path={path}", flush=True)
    _run_case(w, length, policy, path, heads=heads)


@pytest.mark.parametrize("group", [32, 128])
@pytest.mark.parametrize("bits", [2, 4])
@pytest.mark.parametrize("kind", workloads.ADVERSARIAL_KINDS)
def test_quantise_adversarial_inputs(kind, bits, group):
    """Codes, scales and zero-points bit-exact on inputs chosen against the quantise kernels' fast
    path (one multiply-add per code with an exact redo next to rounding ties): lattices full of exact
    ties, large |zero-point / scale|, subnormal fp16 scales, ranges near the top of fp16."""
    torch = gh.require_gpu()
    b, h, T = 2, 3, 1024
    k = workloads.adversarial_values(kind, 11, (b, h, T, 128))
    v = workloads.adversarial_values(kind, 12, (b, h, T, 128))
    print(f"case adversarial {kind} bits={bits} G={group}", flush=True)
    layout = kivi.make_layout(b, h, h, bits, 128, T, 288, group=group)
    cache = kivi.Cache(layout)
    kivi.kivi_quantize_key_groups(layout, torch.from_numpy(k).cuda(), T, cache)
    kivi.kivi_quantize_value_tokens(layout, torch.from_numpy(v).cuda(), T, cache)
    torch.cuda.synchronize()
    oc = ko.StreamingCache(b, h, 128, bits, group, 0, "window")
    oc.k_codes, oc.k_scale, oc.k_zero = ko.quantize_key(k, bits, group)
    oc.v_codes, oc.v_scale, oc.v_zero = ko.quantize_value(v, bits, group)
    oc.k_resid, oc.v_resid = k[:, :, :0], v[:, :, :0]
    gh.compare_quantized_state(cache, oc)
