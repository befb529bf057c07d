"""The whole layer path enqueues kernels only (no allocation, no synchronisation, fill kernels
instead of memsets), so a caller can capture it in a HIP graph.  Capture once, replay several
times with new activations in the same buffers and eager work in between, and compare every
replay with the eager result."""
import numpy as np
import pytest

torch = pytest.importorskip("torch")

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def test_layer_path_replays_from_a_graph():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2311_01305_amd import binding, pipeline, synth
    binding.load_library()
    T, K, N = 1536, 1024, 768
    wl = synth.scaled(synth.WORKLOADS[2], T, [synth.Linear("fc", N, K)])
    W = torch.from_numpy(synth.make_weight_np(11, N, K, wl.dtype)).to(DEV)
    b = torch.from_numpy(synth.make_bias_np(11, N, True)).to(DEV)
    Xs = [torch.from_numpy(synth.make_act_np(100 + i, T, K, wl)).to(DEV) for i in range(3)]
    X = torch.empty_like(Xs[0])
    keys = ("s", "codes", "xq", "out_i32", "out_deq", "colsum_acc", "delta", "bias_out", "rowsum_x", "act_step")

    def snapshot(t):
        torch.cuda.synchronize()
        return {k: t[k].clone() for k in keys}

    # eager references
    eager = []
    buf_e = pipeline.LayerBuffers(T, K, N, torch.float16, want_out_i32=True, want_out_deq=True, device=DEV)
    for Xi in Xs:
        X.copy_(Xi)
        eager.append(snapshot(pipeline.calibrate_layer(X, W, b, buf_e, fused_weight_pass=True)))

    buf = pipeline.LayerBuffers(T, K, N, torch.float16, want_out_i32=True, want_out_deq=True, device=DEV)
    X.copy_(Xs[0])
    pipeline.calibrate_layer(X, W, b, buf, fused_weight_pass=True)   # warm-up outside the capture
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        pipeline.calibrate_layer(X, W, b, buf, fused_weight_pass=True)
    for rep in range(2):
        for i, Xi in enumerate(Xs):
            print(f"[gpu-graph] replay {rep}.{i}", flush=True)
            X.copy_(Xi)
            for k in keys:                      # eager work between replays: scribble over the outputs
                buf.t[k].fill_(0)
            torch.cuda.synchronize()
            graph.replay()
            got = snapshot(buf.t)
            for k in keys:
                assert torch.equal(got[k], eager[i][k]), (rep, i, k)
    assert int(buf.t["status"].item()) == 0
