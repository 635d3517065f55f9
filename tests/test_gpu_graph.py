"""The graph-launch mode of st_partial_distill (st_distill_opts.use_graph): the cached HIP graph
must give exactly what the plain call gives, on the first launch and on every replay, with other
GPU work and synchronisations between the replays and with buffer contents that change."""
import numpy as np
import pytest
import torch

import paper_2003_10735_amd as st
import workloads as WL
from gpu_util import to_dev_features

pytestmark = pytest.mark.gpu


def outputs(bufs):
    torch.cuda.synchronize()
    return [b.cpu().numpy().copy() for b in bufs]


@pytest.mark.parametrize("mode", ["sgd", "momentum", "adam", "grouped"])
def test_graph_replays_equal_the_plain_call(mode):
    grouped = mode == "grouped"
    wl = WL.small_variant(WL.WORKLOADS["720p"], steps=3, lr=0.02, n_sites=9, n=3 if grouped else 2, c_in=64, h=9,
                          w=35, c1=64, c2=64, n_classes=6, momentum=0.9 if mode == "momentum" else 0.0)
    desc = st.HeadDesc.of(wl)
    desc.grouped = 1 if grouped else 0
    heads = wl.n if grouped else 1
    feats = [WL.make_features(wl, seed=wl.feat_seed + i) for i in range(3)]
    labs = [WL.make_labels(WL.small_variant(wl, label_seed=wl.label_seed + 10 * i)) for i in range(3)]
    p_np = np.stack([WL.make_head_params(wl, seed=wl.init_seed + 17 * i) for i in range(heads)]).astype(np.float32)
    if not grouped:
        p_np = p_np[0]
    stream = torch.cuda.Stream()
    ws = st.new_workspace(desc)
    # fixed buffers: the graph is tied to their addresses, their contents change
    f = to_dev_features(wl, feats[0]).clone()
    lab = torch.from_numpy(labs[0]).cuda()
    p = torch.from_numpy(p_np).cuda()
    s1, s2 = torch.zeros_like(p), torch.zeros_like(p)
    steps = 3
    losses = torch.zeros((steps + 1, heads) if grouped else (steps + 1,), dtype=torch.float32, device="cuda")
    mious = torch.zeros((steps + 1, wl.n), dtype=torch.float64, device="cuda")
    conf = torch.zeros((wl.n, wl.n_classes, wl.n_classes), dtype=torch.int64, device="cuda")
    pred = torch.zeros((wl.n, wl.H, wl.W), dtype=torch.uint8, device="cuda")

    def call(graph):
        kw = dict(losses=losses, mious=mious, confusion=conf, pred=pred, workspace=ws, stream=stream, graph=graph)
        if mode == "adam":
            kw["adam"] = dict(m=s1, v=s2, t0=0)
        elif mode == "momentum":
            kw.update(momentum=0.9, velocity=s1)
        with torch.cuda.stream(stream):
            taken, _ = st.st_partial_distill(desc, f, lab, p, steps, wl.lr, **kw)
        assert taken == steps
        return outputs([p, s1, s2, losses, mious, conf, pred])

    def load(i):
        torch.cuda.synchronize()
        f.copy_(to_dev_features(wl, feats[i]))
        lab.copy_(torch.from_numpy(labs[i]).cuda())
        p.copy_(torch.from_numpy(p_np).cuda())
        s1.zero_(); s2.zero_()
        for b in (losses, mious, conf, pred):
            b.zero_()
        torch.cuda.synchronize()

    st.st_graph_cache_clear()
    want = []
    for i in range(3):
        load(i)
        want.append(call(False))
    assert st.st_graph_cache_size() == 0
    assert not np.array_equal(want[0][0], want[1][0])          # the inputs do differ
    scratch = torch.randn(1 << 20, device="cuda")
    for rep in range(2):
        for i in range(3):
            load(i)
            scratch = scratch * 1.0001 + 1.0                    # unrelated eager work between the launches
            got = call(True)
            torch.cuda.synchronize()
            for a, b in zip(got, want[i]):
                np.testing.assert_array_equal(a, b)
            assert st.st_graph_cache_size() == 1               # recorded once, replayed afterwards
    # a different call (another step count) gets a graph of its own
    load(0)
    with torch.cuda.stream(stream):
        st.st_partial_distill(desc, f, lab, p, 1, wl.lr, losses=losses, mious=mious, workspace=ws, stream=stream, graph=True)
    torch.cuda.synchronize()
    assert st.st_graph_cache_size() == 2
    st.st_graph_cache_clear()
    assert st.st_graph_cache_size() == 0


def test_graph_mode_falls_back_where_it_cannot_apply():
    wl = WL.small_variant(WL.WORKLOADS["720p"], steps=2, n=1, c_in=64, h=6, w=10, c1=64, c2=64, n_classes=4, n_sites=5)
    desc = st.HeadDesc.of(wl)
    f = to_dev_features(wl, WL.make_features(wl))
    lab = torch.from_numpy(WL.make_labels(wl)).cuda()
    p0 = torch.from_numpy(WL.make_head_params(wl)).cuda()
    st.st_graph_cache_clear()
    # early exit decides on the host: never recorded
    p = p0.clone()
    stream = torch.cuda.Stream()
    with torch.cuda.stream(stream):
        taken, best = st.st_partial_distill(desc, f, lab, p, 2, wl.lr, threshold=2.0, stream=stream, graph=True)
    torch.cuda.synchronize()
    assert taken == 2 and st.st_graph_cache_size() == 0
    ref = p.cpu().numpy()
    # the same through the plain path
    q = p0.clone()
    st.st_partial_distill(desc, f, lab, q, 2, wl.lr, threshold=2.0)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(q.cpu().numpy(), ref)


@pytest.mark.parametrize("graph", [False, True])
def test_clients_on_streams_of_their_own_do_not_disturb_each_other(graph):
    """Three clients (own key frame, head, workspace, stream) whose calls are issued back to back
    with no synchronisation in between must each get, bit for bit, what a call on its own gets."""
    wl0 = WL.small_variant(WL.WORKLOADS["720p"], steps=3, lr=0.02, n_sites=9, c_in=64, h=17, w=35, c1=64, c2=64,
                           n_classes=6)
    desc = st.HeadDesc.of(wl0)
    clients = []
    for i in range(3):
        wl = WL.small_variant(wl0, feat_seed=wl0.feat_seed + i, label_seed=wl0.label_seed + 10 * i)
        p0 = torch.from_numpy(WL.make_head_params(wl, seed=wl.init_seed + 17 * i)).cuda()
        clients.append(dict(f=to_dev_features(wl, WL.make_features(wl)), lab=torch.from_numpy(WL.make_labels(wl)).cuda(),
                            p0=p0, p=p0.clone(), ws=st.new_workspace(desc), s=torch.cuda.Stream(),
                            losses=torch.zeros(4, dtype=torch.float32, device="cuda"),
                            mious=torch.zeros((4, 1), dtype=torch.float64, device="cuda")))

    def call(c):
        st.st_partial_distill(desc, c["f"], c["lab"], c["p"], 3, wl0.lr, losses=c["losses"], mious=c["mious"],
                              workspace=c["ws"], stream=c["s"], graph=graph)

    alone = []
    for c in clients:                      # each on its own, the device idle around it
        torch.cuda.synchronize()
        call(c)
        alone.append(outputs([c["p"], c["losses"], c["mious"]]))
    for _ in range(3):                     # all together, several rounds in flight at once
        torch.cuda.synchronize()
        for c in clients:
            c["p"].copy_(c["p0"])
        torch.cuda.synchronize()
        for _ in range(4):
            for c in clients:
                call(c)                    # (round r continues from the parameters of round r - 1)
        torch.cuda.synchronize()
    # the same four rounds one client at a time
    for c, first in zip(clients, alone):
        together = outputs([c["p"], c["losses"], c["mious"]])
        c["p"].copy_(c["p0"])
        for r in range(4):
            torch.cuda.synchronize()
            call(c)
            if r == 0:
                for a, b in zip(outputs([c["p"], c["losses"], c["mious"]]), first):
                    np.testing.assert_array_equal(a, b)
        for a, b in zip(outputs([c["p"], c["losses"], c["mious"]]), together):
            np.testing.assert_array_equal(a, b)
    st.st_graph_cache_clear()


def test_two_host_threads_run_the_early_exit_form_side_by_side():
    """Algorithm 1 with its per-iteration read-back, called from two host threads at once (own
    stream, workspace and head each): every thread gets what it gets alone."""
    import threading
    wl0 = WL.small_variant(WL.WORKLOADS["720p"], steps=4, lr=0.02, n_sites=9, c_in=64, h=13, w=35, c1=64, c2=64,
                           n_classes=6)
    desc = st.HeadDesc.of(wl0)
    clients = []
    for i in range(2):
        wl = WL.small_variant(wl0, feat_seed=wl0.feat_seed + i, label_seed=wl0.label_seed + 10 * i)
        p0 = torch.from_numpy(WL.make_head_params(wl, seed=wl.init_seed + 17 * i)).cuda()
        clients.append(dict(f=to_dev_features(wl, WL.make_features(wl)), lab=torch.from_numpy(WL.make_labels(wl)).cuda(),
                            p0=p0, p=p0.clone(), ws=st.new_workspace(desc), s=torch.cuda.Stream(),
                            mious=torch.zeros((5, 1), dtype=torch.float64, device="cuda"), out=[]))

    def work(c, rounds):
        for _ in range(rounds):
            r = st.st_partial_distill(desc, c["f"], c["lab"], c["p"], 4, wl0.lr, threshold=1.5, return_best=True,
                                      mious=c["mious"], workspace=c["ws"], stream=c["s"])
            c["out"].append((tuple(r), r.first_metric))

    torch.cuda.synchronize()
    for c in clients:                                   # one after the other
        work(c, 3)
    torch.cuda.synchronize()
    alone = [(c["p"].cpu().numpy().copy(), list(c["out"])) for c in clients]
    for c in clients:
        c["p"].copy_(c["p0"])
        c["out"].clear()
    torch.cuda.synchronize()
    threads = [threading.Thread(target=work, args=(c, 3)) for c in clients]
    for t in threads:
        t.start()
    for t in threads:
        t.join()
    torch.cuda.synchronize()
    for c, (p_alone, out_alone) in zip(clients, alone):
        assert c["out"] == out_alone
        assert all(o[0][0] == 4 for o in c["out"])      # the threshold is out of reach: all four updates
        np.testing.assert_array_equal(c["p"].cpu().numpy(), p_alone)


def test_two_host_threads_record_and_launch_graphs_side_by_side():
    """Two host threads (own stream, workspace and head each) whose first graph-mode calls -- the
    ones that record -- and later launches happen at the same time: every thread gets what it gets
    alone, and the cache ends up with one graph per distinct call."""
    import threading
    st.st_graph_cache_clear()
    wl0 = WL.small_variant(WL.WORKLOADS["720p"], steps=3, lr=0.02, n_sites=9, c_in=64, h=13, w=35, c1=64, c2=64,
                           n_classes=6)
    desc = st.HeadDesc.of(wl0)
    clients = []
    for i in range(2):
        wl = WL.small_variant(wl0, feat_seed=wl0.feat_seed + i, label_seed=wl0.label_seed + 10 * i)
        p0 = torch.from_numpy(WL.make_head_params(wl, seed=wl.init_seed + 17 * i)).cuda()
        clients.append(dict(f=to_dev_features(wl, WL.make_features(wl)), lab=torch.from_numpy(WL.make_labels(wl)).cuda(),
                            p0=p0, p=p0.clone(), ws=st.new_workspace(desc), s=torch.cuda.Stream(),
                            losses=torch.zeros(4, dtype=torch.float32, device="cuda")))

    def work(c, rounds, graph):
        for _ in range(rounds):
            st.st_partial_distill(desc, c["f"], c["lab"], c["p"], 3, wl0.lr, losses=c["losses"], workspace=c["ws"],
                                  stream=c["s"], graph=graph)

    torch.cuda.synchronize()
    for c in clients:                                   # one after the other, plain launches
        work(c, 4, False)
    torch.cuda.synchronize()
    alone = [outputs([c["p"], c["losses"]]) for c in clients]
    for c in clients:
        c["p"].copy_(c["p0"])
    torch.cuda.synchronize()
    threads = [threading.Thread(target=work, args=(c, 4, True)) for c in clients]
    for t in threads:
        t.start()
    for t in threads:
        t.join()
    torch.cuda.synchronize()
    for c, ref in zip(clients, alone):
        for a, b in zip(outputs([c["p"], c["losses"]]), ref):
            np.testing.assert_array_equal(a, b)
    assert st.st_graph_cache_size() == 2
    st.st_graph_cache_clear()
