"""GPU: the library's calls are capturable in a HIP graph (no allocation, no synchronisation, no memset inside):
one prune + update-GEMM step of a ViT-sized layer, split-K path included, is captured once and replayed several
times with eager work and synchronisations between the replays; every replay equals the eager result bit for bit."""
import pytest
import torch

from paper_2203_10991_amd import synth
from gpu_util import DEV

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("q8", [False, True])
def test_step_replays_from_a_graph(q8):
    import paper_2203_10991_amd as nm
    nm.load()
    w = synth.WORKLOADS["c4_vit_proj_2of4"]
    T = w.T - w.T % 32
    g, h = synth.make_device(w, seed=1, device=DEV)
    g, h = g[:T].contiguous(), h[:T].contiguous()
    dW = torch.zeros((w.O, w.I), dtype=torch.float32, device=DEV)
    if q8:
        h = h.float().to(torch.float8_e4m3fn).view(torch.uint8)
        vals, meta = nm.alloc_compressed_q8(T, w.O, DEV)
        need = nm.nm_update_gemm_q8_workspace(T, w.O, w.I)
    else:
        vals, meta = nm.alloc_compressed(T, w.O, g.dtype, DEV)
        need = nm.nm_update_gemm_workspace(T, w.O, w.I, g.dtype)
    assert need > 0                                    # this shape takes the split-K path
    ws = torch.empty(need, dtype=torch.uint8, device=DEV)

    def step():
        if q8:
            nm.mvue_prune_2of4_q8(g, seed=4, stream_id=0, mode=0, scale=0.25, vals8=vals, meta32=meta)
            nm.nm_update_gemm_q8(vals, meta, h, dW=dW, alpha=4.0, beta=0.0, workspace=ws)
        else:
            nm.mvue_prune_2of4(g, seed=4, stream_id=0, vals=vals, meta=meta)
            nm.nm_update_gemm(vals, meta, h, dW=dW, beta=0.0, workspace=ws)

    step()
    torch.cuda.synchronize()
    want_dW, want_vals = dW.clone(), vals.clone()
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        step()                                          # warm-up on the capture stream
        side.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            step()
    for i in range(4):
        dW.fill_(float("nan"))                          # eager work between the replays
        vals.zero_()
        ws.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(dW, want_dW), f"replay {i}"
        assert torch.equal(vals.view(torch.uint8), want_vals.view(torch.uint8)), f"replay {i}"


def test_two_host_threads_on_two_streams():
    """The library keeps no state between calls (its error text is per thread): two host threads, each with its own
    stream, buffers and workspace, run different layers at the same time and get what a lone run gets, bit for bit."""
    import threading
    import paper_2203_10991_amd as nm
    nm.load()
    jobs = []
    for k, name in enumerate(["c4_vit_proj_2of4", "c4_vit_fc2_2of4"]):
        w = synth.WORKLOADS[name]
        T = w.T - w.T % 16
        g, h = synth.make_device(w, seed=3 + k, device=DEV)
        g, h = g[:T].contiguous(), h[:T].contiguous()
        vals, meta = nm.alloc_compressed(T, w.O, g.dtype, DEV)
        ws = torch.empty(max(16, nm.nm_update_gemm_workspace(T, w.O, w.I, g.dtype)), dtype=torch.uint8, device=DEV)
        dW = torch.empty((w.O, w.I), dtype=torch.float32, device=DEV)
        jobs.append(dict(g=g, h=h, vals=vals, meta=meta, ws=ws, dW=dW, seed=10 + k))

    def step(j):
        nm.mvue_prune_2of4(j["g"], seed=j["seed"], stream_id=1, vals=j["vals"], meta=j["meta"])
        nm.nm_update_gemm(j["vals"], j["meta"], j["h"], dW=j["dW"], beta=0.0, workspace=j["ws"])

    for j in jobs:                                      # lone runs
        step(j)
        torch.cuda.synchronize()
        j["want"] = j["dW"].clone()
    errors = []

    def worker(j):
        try:
            s = torch.cuda.Stream()
            with torch.cuda.stream(s):
                for _ in range(20):
                    j["dW"].fill_(float("nan"))
                    step(j)
                    s.synchronize()
                    if not torch.equal(j["dW"], j["want"]):
                        errors.append("dW differs")
                        return
        except Exception as e:                          # surfaces in the main thread
            errors.append(repr(e))

    threads = [threading.Thread(target=worker, args=(j,)) for j in jobs]
    for t in threads:
        t.start()
    for t in threads:
        t.join(timeout=100)
    torch.cuda.synchronize()
    assert not errors, errors
    assert not any(t.is_alive() for t in threads)


def test_independent_layers_replay_from_a_branched_graph():
    """Two layers captured as parallel branches of one graph (a second stream forks from and joins the capture
    stream): every replay, with eager work and synchronisations in between, equals the eager results bit for bit."""
    import paper_2203_10991_amd as nm
    nm.load()
    jobs = []
    for k, name in enumerate(["c4_vit_qkv_2of4", "c4_vit_fc2_1of2"]):
        w = synth.WORKLOADS[name]
        T = w.T - w.T % 16
        g, h = synth.make_device(w, seed=7 + k, device=DEV)
        g, h = g[:T].contiguous(), h[:T].contiguous()
        vals, meta = nm.alloc_compressed(T, w.O, g.dtype, DEV)
        ws = torch.empty(max(16, nm.nm_update_gemm_workspace(T, w.O, w.I, g.dtype)), dtype=torch.uint8, device=DEV)
        dW = torch.empty((w.O, w.I), dtype=torch.float32, device=DEV)
        prune = nm.mvue_prune_1of2 if w.nm == "1:2" else nm.mvue_prune_2of4
        jobs.append(dict(g=g, h=h, vals=vals, meta=meta, ws=ws, dW=dW, prune=prune))

    def layer(j):
        j["prune"](j["g"], seed=21, stream_id=3, vals=j["vals"], meta=j["meta"])
        nm.nm_update_gemm(j["vals"], j["meta"], j["h"], dW=j["dW"], beta=0.0, workspace=j["ws"])

    for j in jobs:
        layer(j)
    torch.cuda.synchronize()
    want = [j["dW"].clone() for j in jobs]
    main, branch = torch.cuda.Stream(), torch.cuda.Stream()
    with torch.cuda.stream(main):
        for j in jobs:
            layer(j)                                    # warm-up on the capture stream
        main.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=main):
            branch.wait_stream(main)
            layer(jobs[0])
            with torch.cuda.stream(branch):
                layer(jobs[1])
            main.wait_stream(branch)
    for i in range(4):
        for j in jobs:
            j["dW"].fill_(float("nan"))
            j["vals"].zero_()
            j["ws"].zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for j, x in zip(jobs, want):
            assert torch.equal(j["dW"], x), f"replay {i}"
