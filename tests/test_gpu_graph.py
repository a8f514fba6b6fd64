"""The step of the object-classification workload (one workgroup per cloud) captured as a HIP
graph on four streams (the chain of exact samplers, a stream per stage in turn for mdps_sample
and its cache reader, one for the brute-force ball queries), as bench.py replays it: every replay
must give the eager result, with eager work of the library and synchronisations between the
replays, and the eager result must be the oracle's.
"""
import numpy as np
import pytest

from oracle import ref
from paper_2507_23480_amd import inputs

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu


def rparams(prm):
    return ref.MdpsParams(p=prm.p, nseg=prm.nseg, exponent=prm.exponent, bias=prm.bias,
                          fit_window=prm.fit_window, m_min=prm.m_min, level_scale=prm.level_scale)


def test_graph_replay_of_four_stream_step_equals_eager_and_oracle():
    from paper_2507_23480_amd import binding as fp, calibration
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    fp.load()
    fp.set_wg_per_cloud(0)
    name = "C2"
    wl = inputs.WORKLOADS[name]
    batch = inputs.make_batch(name)
    xyz = torch.from_numpy(batch).cuda()
    B = wl.B
    lanes = [torch.cuda.Stream(), torch.cuda.Stream()]
    bqs = torch.cuda.Stream()
    N = wl.N
    stages = []
    for s, st in enumerate(wl.stages):
        assert fp.plan(B, N)[0] == 1
        stages.append({"n": st.n, "r": st.radius, "k": st.k, "prm": calibration.params_for(name, s),
                       "cache": torch.empty(fp.load().fp_bq_cache_bytes(B, N, st.n, 0), dtype=torch.uint8,
                                            device="cuda"),
                       "ws": [fp.new_workspace(xyz.device, B, N), fp.new_workspace(xyz.device, B, N)]})
        N = st.n

    inputs_alive = []

    def step(keep):
        main = torch.cuda.current_stream()
        x = xyz
        for s, sg in enumerate(stages):
            lane = lanes[s % 2]
            lane.wait_stream(main)
            with torch.cuda.stream(lane):
                midx = fp.mdps_sample(x, sg["n"], sg["prm"], bq_cache=sg["cache"], bq_radius=sg["r"],
                                      ws=sg["ws"][1])
                mbq = fp.ball_query(x, midx, sg["r"], sg["k"], bq_cache=sg["cache"])
            idx = fp.fps_exact(x, sg["n"], ws=sg["ws"][0])
            x_next = None if s + 1 == len(stages) else fp.gather_xyz(x, idx)
            bqs.wait_stream(main)
            with torch.cuda.stream(bqs):
                bq = fp.ball_query(x, idx, sg["r"], sg["k"])
            keep.append((idx, bq[0], bq[1], midx, mbq[0], mbq[1]))
            inputs_alive.append(x)               # a stage's input outlives the calls that read it
            x = x_next
        for other in (lanes[0], lanes[1], bqs):
            main.wait_stream(other)

    eager = []
    step(eager)
    torch.cuda.synchronize()
    eager = [[t.clone() for t in row] for row in eager]

    # the eager result against the oracle (first cloud, every stage)
    x = batch[0]
    for s, st in enumerate(wl.stages):
        idx, _ = ref.fps_exact(x, st.n)
        midx, _ = ref.mdps_sample(x, st.n, rparams(stages[s]["prm"]))
        bq_i, bq_c = ref.ball_query(x, midx, st.radius, st.k)
        assert np.array_equal(eager[s][0][0].cpu().numpy(), idx)
        assert np.array_equal(eager[s][3][0].cpu().numpy(), midx)
        assert np.array_equal(eager[s][4][0].cpu().numpy(), bq_i)
        assert np.array_equal(eager[s][5][0].cpu().numpy(), bq_c)
        x = ref.gather_xyz(x, idx)

    graph = torch.cuda.CUDAGraph()
    held = []
    with torch.cuda.graph(graph):
        step(held)
    for rep in range(4):
        for row in held:                       # a replay has to rewrite every output
            for t in row:
                t.fill_(-7)
        for sg in stages:
            sg["cache"].zero_()
        graph.replay()
        torch.cuda.synchronize()
        for s, (got, want) in enumerate(zip(held, eager)):
            for j, (g, w) in enumerate(zip(got, want)):
                assert torch.equal(g, w), "replay %d, stage %d, output %d differs" % (rep, s, j)
        # eager work of the library on the default stream between the replays
        other = fp.fps_exact(xyz, 64)
        torch.cuda.synchronize()
        assert torch.equal(other, eager[0][0][:, :64])
