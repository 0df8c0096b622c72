"""The entry points allocate nothing, clear nothing with memset calls and keep no state, so a
caller may record them into a HIP graph.  A whole layer (input transform, decode + product,
output transform; Section 2.1) and a quantizer call are captured once and replayed several
times with eager work and new inputs between the replays; every replay must give the bits of
the eager calls on the same inputs."""
import numpy as np
import pytest

import qtip_synth as synth
from qtip_synth import CODE_3INST, CODE_HYB

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def q():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    import paper_2406_11235_amd as q
    q.lib()
    return q


def dev(a):
    import torch
    return None if a is None else torch.from_numpy(np.ascontiguousarray(a)).cuda()


@pytest.mark.parametrize("code_id,k,V,m,n,block", [(CODE_3INST, 2, 1, 1024, 2048, 1024), (CODE_HYB, 4, 2, 512, 12288, 4096)])
def test_layer_replayed_from_a_graph(q, code_id, k, V, m, n, block):
    import torch
    w = synth.Workload("graph_layer", 9, 7, m, n, code_id, k, V, block, 512, row_scale=True)
    inp = synth.make_inputs(w)
    codes, lut, sc = dev(inp.codes), dev(inp.lut), dev(inp.row_scale)
    sn, sm = dev(inp.signs_n), dev(inp.signs_m)
    x = dev(inp.X)
    xt = torch.empty((1, n), dtype=torch.float16, device="cuda")
    z = torch.empty((1, m), dtype=torch.float32, device="cuda")
    y = torch.empty((1, m), dtype=torch.float16, device="cuda")
    z2 = torch.empty(m, dtype=torch.float32, device="cuda")
    scratch = torch.empty(n, dtype=torch.float16, device="cuda")

    def layer():
        q.qtip_rht(x, sn, n, block, 1, 0, xt)
        q.qtip_decode_matmat(codes, 16, k, V, code_id, lut, m, n, xt, 1, sc, z)
        q.qtip_rht_f32(z, sm, m, 512, 1, 1, y)
        q.qtip_rht_decode_matvec(codes, 16, k, V, code_id, lut, m, n, x, sn, block, sc, z2, scratch)

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        layer()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        layer()
    rng = np.random.default_rng(5)
    for replay in range(4):
        x.copy_(dev(rng.standard_normal((1, n)).astype(np.float16)))
        layer()
        torch.cuda.synchronize()
        want = (y.clone(), z.clone(), z2.clone())
        for t in (xt, z, y, z2):
            t.fill_(float("nan"))
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(y.view(torch.int16), want[0].view(torch.int16)), replay
        assert torch.equal(z.view(torch.int32), want[1].view(torch.int32)), replay
        assert torch.equal(z2.view(torch.int32), want[2].view(torch.int32)), replay
        assert torch.equal(z2, z.reshape(-1))


def test_quantizer_replayed_from_a_graph(q):
    import torch
    m, n, k = 32, 64, 2
    ntiles = (m // 16) * (n // 16)
    ws_bytes = q.qtip_quantize_gpu_workspace(k, 1, 3)      # three tiles in flight: three batches
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device="cuda")
    W = torch.empty((m, n), dtype=torch.float32, device="cuda")
    codes = torch.empty((ntiles, 8 * k), dtype=torch.int32, device="cuda")
    err = torch.empty(ntiles, dtype=torch.float32, device="cuda")

    def call():
        q.qtip_quantize_gpu(W, m, n, 16, k, 1, CODE_3INST, None, codes, err, ws, ws_bytes)

    rng = np.random.default_rng(6)
    W.copy_(dev(rng.standard_normal((m, n)).astype(np.float32)))
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        call()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        call()
    for replay in range(3):
        W.copy_(dev((rng.standard_normal((m, n)) * 1.2).astype(np.float32)))
        call()
        torch.cuda.synchronize()
        want = (codes.clone(), err.clone())
        codes.fill_(-1)
        err.fill_(float("nan"))
        ws.fill_(0xA5)                                     # the workspace needs no particular contents
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(codes, want[0]), replay
        assert torch.equal(err.view(torch.int32), want[1].view(torch.int32)), replay


def test_calls_on_two_streams_at_once(q):
    """No state is shared between calls: two layers enqueued on two streams with an explicit
    stream argument, overlapping in time, give the bits of the same calls made one after the
    other on the default stream."""
    import torch
    m, n, k = 2048, 8192, 2
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    jobs = []
    for j, code_id in enumerate((CODE_3INST, CODE_HYB)):
        V = 2 if code_id == CODE_HYB else 1
        w = synth.Workload("two_streams", 9, 20 + j, m, n, code_id, k, V, 4096, 2048)
        inp = synth.make_inputs(w)
        jobs.append(dict(code_id=code_id, V=V, codes=dev(inp.codes), lut=dev(inp.lut), x=dev(inp.X), sn=dev(inp.signs_n),
                         xt=torch.empty((1, n), dtype=torch.float16, device="cuda"),
                         y=torch.empty(m, dtype=torch.float32, device="cuda")))

    def run(job, stream):
        q.qtip_rht(job["x"], job["sn"], n, 4096, 1, 0, job["xt"], stream=stream)
        q.qtip_decode_matvec(job["codes"], 16, k, job["V"], job["code_id"], job["lut"], m, n, job["xt"], job["y"],
                             stream=stream)

    for job in jobs:
        run(job, None)
    torch.cuda.synchronize()
    want = [job["y"].clone() for job in jobs]
    for rep in range(5):
        for job in jobs:
            job["y"].fill_(float("nan"))
            job["xt"].fill_(float("nan"))
        torch.cuda.synchronize()
        for job, st in zip(jobs, streams):
            run(job, st)
        torch.cuda.synchronize()
        for job, ref in zip(jobs, want):
            assert torch.equal(job["y"].view(torch.int32), ref.view(torch.int32)), rep
