"""The decode-attention launch under HIP graph capture: a serving loop replays one captured
launch per layer and step.  The kernel must be capturable as it is (no allocation, no memset
node: its workspace counters return to zero by themselves) and every replay must give what the
eager call gives, also after eager launches on the same workspace in between."""
import numpy as np
import pytest

import gpu_harness as gh
from paper_2402_02750_amd import kivi, workloads
from paper_2402_02750_amd.workloads import CONFIGS, scaled

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("path", [kivi.KIVI_DECODE_VALU, kivi.KIVI_DECODE_MFMA, kivi.KIVI_DECODE_MFMA_TWO], ids=["valu", "mfma", "mfma2"])
def test_replayed_launch_matches_eager(path):
    torch = gh.require_gpu()
    # 2 x 2 units of 6000 tokens: several workgroups per unit, so the cross-workgroup merge and
    # its counters are part of the captured launch
    w = scaled(CONFIGS["mistral_gqa"], name="graph", batch=2, n_q_heads=8, n_kv_heads=2, seed=321)
    length = 6000
    k, v = workloads.keys(w, length), workloads.values(w, length)
    layout, cache = gh.gpu_prefill(w, k, v, kivi.KIVI_FLUSH_WINDOW, path)
    heads = [(0, 0), (1, 1)]
    oc = gh.oracle_cache_for_heads(w, k, v, heads, "window")
    qs = [workloads.queries(w, step) for step in range(4)]
    q_static = torch.from_numpy(qs[0]).cuda()
    out_static = torch.empty(w.batch, w.n_q_heads, 128, dtype=torch.float32, device="cuda")
    out_eager = torch.empty_like(out_static)

    kivi.kivi_decode_attention(layout, cache, q_static, w.softmax_scale, out_eager)     # warm-up outside the capture
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        kivi.kivi_decode_attention(layout, cache, q_static, w.softmax_scale, out_static,
                                   stream=torch.cuda.current_stream())
    for trial, q in enumerate(qs):
        print(f"case graph path={path} replay {trial}", flush=True)
        q_static.copy_(torch.from_numpy(q).cuda())
        graph.replay()
        torch.cuda.synchronize()
        got = out_static.cpu().numpy().copy()
        # eager launch on the same cache and workspace between the replays
        kivi.kivi_decode_attention(layout, cache, q_static, w.softmax_scale, out_eager)
        torch.cuda.synchronize()
        assert np.array_equal(got, out_eager.cpu().numpy()), f"replay {trial} differs from the eager launch"
        gh.check_close(gh.pick_heads(got, w, heads), gh.oracle_attention_for_heads(w, oc, q, heads), f"replay {trial}")
