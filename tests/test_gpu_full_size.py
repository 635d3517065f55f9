"""GPU parity at the full workload sizes, in the launch configuration the benchmark times.
The CPU oracle finishes these in seconds to a few tens of seconds, so whole tensors are
compared (losses per step, every updated weight), plus the bit-exact staged check of the class
map, confusion counts and mean IoU."""
import numpy as np
import pytest

import workloads as WL
from gpu_util import (check_pred_against_oracle, check_staged_bit_exact, live_oracle, load_golden, progress, rel_err,
                      run_gpu, run_oracle, update_err)

pytestmark = pytest.mark.gpu


# Bar on the update (trained minus initial parameters) against the bf16-operand oracle at the
# full sizes: five times what is measured there (2e-5 .. 2e-4; the parameters themselves are
# dominated by their initial values and say little).  Small grids cannot carry a bar this tight:
# there a single activation whose sign the order of additions decides switches a ReLU mask
# element, which alone moves a gradient entry by about 1 / positions (up to 2e-2 on a few hundred
# positions, seen on the random shapes), so they keep 3e-2.  What the bar cannot tell at these
# sizes is a single misplaced rounding point of the bf16 path: planted in the oracle, one moves
# the 720p update error from 1.9e-4 to 2.4e-4 .. 7.3e-4 (on a few hundred positions: 2e-3 ..
# 1e-2).  The activations and back-propagated gradients are rounded by being stored as bfloat16.
FULL_SIZE_UPDATE_BAR = 1e-3


def compare_bf16(wl, steps, tight=5e-4):
    f, lab, p = WL.make_features(wl), WL.make_labels(wl), WL.make_head_params(wl)
    gpu = run_gpu(wl, f, lab, p, steps=steps)
    print(wl.name, "gpu losses", gpu["losses"], "mIoU", gpu["mious"][-1])
    check_staged_bit_exact(wl, gpu, lab)
    ora = run_oracle(wl, f, lab, p, steps=steps, bf16_operands=False, report=wl.name + " exact")
    print(wl.name, "oracle losses", ora["losses"])
    assert rel_err(gpu["losses"], ora["losses"]) < 2e-2          # bf16 GEMM inputs: 2e-2 relative
    assert rel_err(gpu["params"], ora["params"]) < 2e-2
    orq = run_oracle(wl, f, lab, p, steps=steps, bf16_operands=True, report=wl.name + " bf16 operands")
    progress("%s %d steps: against the exact oracle losses %.3g weights %.3g; against the bf16-operand oracle losses %.3g "
             "weights %.3g update %.3g" % (wl.name, len(gpu["losses"]) - 1, rel_err(gpu["losses"], ora["losses"]),
                                          rel_err(gpu["params"], ora["params"]), rel_err(gpu["losses"], orq["losses"]),
                                          rel_err(gpu["params"], orq["params"]), rel_err(gpu["params"] - p, orq["params"] - p)))
    # same rounding points on both sides: what is left is accumulation order
    assert rel_err(gpu["losses"], orq["losses"]) < tight
    assert rel_err(gpu["params"], orq["params"]) < tight
    assert update_err(wl.name, gpu["params"] - p, orq["params"] - p) < FULL_SIZE_UPDATE_BAR
    if wl.momentum:
        assert rel_err(gpu["velocity"], orq["velocity"]) < 3e-2
    np.testing.assert_allclose(gpu["mious"], orq["mious"], atol=5e-3)
    n_bad = check_pred_against_oracle(wl, gpu, orq, f, logit_tol=2e-2)
    print(wl.name, "class-map pixels differing from the oracle's own map:", n_bad)
    return gpu, ora, orq


def test_720p_key_frame_all_steps():
    compare_bf16(WL.WORKLOADS["720p"], steps=None)


@pytest.mark.timeout(600)
def test_1080p_ignore_and_momentum_all_steps():
    """The 1920x1080 key frame at its own length: eight steps with momentum 0.9, 5 % of the
    pixels ignored."""
    compare_bf16(WL.WORKLOADS["1080p"], steps=None)


@pytest.mark.timeout(600)
def test_2160p_beyond_the_measured_sizes():
    """A 3840x2160 key frame (nine times the benchmark's frame: every kernel's grid runs several
    rounds of blocks, the loss kernel 4 050 tiles), two steps with momentum and ignored pixels,
    against the oracle's bf16-operand mode."""
    wl = WL.small_variant(WL.WORKLOADS["1080p"], h=270, w=480, n_sites=120, steps=2)
    f, lab, p = WL.make_features(wl), WL.make_labels(wl), WL.make_head_params(wl)
    gpu = run_gpu(wl, f, lab, p, steps=2)
    check_staged_bit_exact(wl, gpu, lab)
    orq = run_oracle(wl, f, lab, p, steps=2, bf16_operands=True, report="2160p bf16 operands")
    progress("2160p 2 steps against the bf16-operand oracle: losses %.3g weights %.3g update %.3g" % (
        rel_err(gpu["losses"], orq["losses"]), rel_err(gpu["params"], orq["params"]),
        rel_err(gpu["params"] - p, orq["params"] - p)))
    assert rel_err(gpu["losses"], orq["losses"]) < 5e-4
    assert rel_err(gpu["params"], orq["params"]) < 5e-4
    assert update_err("2160p", gpu["params"] - p, orq["params"] - p) < FULL_SIZE_UPDATE_BAR
    assert rel_err(gpu["velocity"], orq["velocity"]) < 3e-2
    np.testing.assert_allclose(gpu["mious"], orq["mious"], atol=5e-3)


@pytest.mark.timeout(1500)
def test_batch4_shared_head_all_steps():
    """Four frames, one shared head 320 -> 256 -> 256 -> 21, at its own length: sixteen steps.
    The oracle needs minutes for that, so its result is read from tests/golden/ (written by the
    committed script there, from the oracle alone; ST_LIVE_ORACLE=1 runs it here instead): losses
    and per-frame mean IoU of all 17 passes, the trained parameters at every 13th index and all
    biases.  One step is also run live in both oracle modes and compared element by element; its
    two losses must equal the stored ones bit for bit, which ties the file to this oracle and
    these inputs."""
    wl = WL.WORKLOADS["batch4"]
    if live_oracle():
        compare_bf16(wl, steps=None)
        return
    gold = load_golden("batch4")
    assert int(gold["steps"]) == wl.steps == 16
    gpu1, ora1, orq1 = compare_bf16(wl, steps=1)
    np.testing.assert_array_equal(ora1["losses"], gold["exact_losses"][:2])
    np.testing.assert_array_equal(orq1["losses"], gold["bf16_losses"][:2])
    f, lab, p = WL.make_features(wl), WL.make_labels(wl), WL.make_head_params(wl)
    gpu = run_gpu(wl, f, lab, p)
    progress("batch4 16 steps: gpu losses %s" % np.round(gpu["losses"], 5).tolist())
    assert gpu["steps_taken"] == 16
    check_staged_bit_exact(wl, gpu, lab)
    idx = gold["index"]
    for tag, tol, tol_upd in (("bf16", 5e-4, FULL_SIZE_UPDATE_BAR), ("exact", 2e-2, 1e-1)):
        e_loss = rel_err(gpu["losses"], gold[tag + "_losses"])
        e_par = float(np.abs(gpu["params"][idx] - gold[tag + "_params"]).max() / gold[tag + "_max_abs_param"])
        e_upd = float(np.abs((gpu["params"][idx] - p[idx]) - (gold[tag + "_params"] - p[idx])).max()
                      / gold[tag + "_max_abs_update"])
        progress(f"batch4 16 steps against the {tag} oracle: losses {e_loss:.3g} weights {e_par:.3g} update {e_upd:.3g}")
        assert e_loss < tol and e_par < tol and e_upd < tol_upd
        np.testing.assert_allclose(gpu["mious"], gold[tag + "_mious"], atol=5e-3 if tag == "bf16" else 2e-2)


def test_720p_adam_all_steps():
    """The paper's optimiser (Section 5.2: Adam, learning rate 0.01) at the benchmark's shape and
    the paper's MAX_UPDATES = 8; see check_adam for why the weights are compared where the first
    gradient is not tiny."""
    from test_gpu_parity import check_adam
    wl = WL.WORKLOADS["720p"]
    f, lab, p = WL.make_features(wl), WL.make_labels(wl), WL.make_head_params(wl)
    check_adam(wl, f, lab, p, wl.steps, True, 2e-3, 2e-2)


def test_720p_paper_recipe_all_steps():
    """Adam at learning rate 0.01 on the cross-entropy weighted x5 within 4 pixels of an object
    (Section 5.2: the optimiser and the loss of the paper's experiments), the weight map made by
    st_object_weights, at the benchmark's shape for all eight steps."""
    from test_gpu_parity import check_adam
    wl = WL.WORKLOADS["720p"]
    f, lab, p = WL.make_features(wl), WL.make_labels(wl), WL.make_head_params(wl)
    check_adam(wl, f, lab, p, wl.steps, True, 2e-3, 2e-2, object_radius=4)


def test_720p_weighted_loss_all_steps():
    """Per-pixel loss weights (Section 5.2) at the benchmark's shape, all eight steps."""
    from test_gpu_parity import check_weighted
    check_weighted(WL.WORKLOADS["720p"], WL.WORKLOADS["720p"].steps, True, 5e-4)


def test_720p_feature_gradient():
    """The full backward pass (what partial distillation leaves out) at the benchmark's shape."""
    from test_gpu_parity import check_feature_grad
    check_feature_grad(WL.WORKLOADS["720p"], True, 5e-3)


def test_720p_four_clients_grouped():
    """Four clients' key frames and heads in one call, in the launch configuration the benchmark
    times for the grouped form, all eight steps; every head against its own single-frame oracle run."""
    import oracle as O
    from test_gpu_grouped import SGD, check_against_oracle, inputs, run_grouped
    wl = WL.small_variant(WL.WORKLOADS["720p"], n=4)
    f, lab, p = inputs(wl)
    g = run_grouped(wl, f, lab, p, wl.steps)
    o = O.partial_distill_grouped(O.desc_of(wl, True), WL.features_as_f64(wl, f), lab, p.astype(np.float64), wl.steps, SGD(wl))
    print("grouped losses", g["losses"].T, "oracle", o["losses"].T)
    check_against_oracle(wl, g, o, p)


def test_720p_graph_launch_equals_the_plain_call():
    """The benchmark's headline is timed through the cached launch graph on a stream of its own:
    at the full size, all eight steps, first launch and a replay, it must give bit for bit what
    the plain call gives (which the test above holds against the oracle)."""
    import torch
    import paper_2003_10735_amd as st
    from gpu_util import to_dev_features
    wl = WL.WORKLOADS["720p"]
    f, lab, p = WL.make_features(wl), WL.make_labels(wl), WL.make_head_params(wl)
    desc = st.HeadDesc.of(wl)
    fd, labd = to_dev_features(wl, f), torch.from_numpy(lab).cuda()
    stream = torch.cuda.Stream()
    ws = st.new_workspace(desc)
    pt = torch.from_numpy(p).cuda()
    losses = torch.zeros(wl.steps + 1, dtype=torch.float32, device="cuda")
    mious = torch.zeros((wl.steps + 1, 1), dtype=torch.float64, device="cuda")
    conf = torch.zeros((1, wl.n_classes, wl.n_classes), dtype=torch.int64, device="cuda")
    pred = torch.zeros((1, wl.H, wl.W), dtype=torch.uint8, device="cuda")

    def run(graph):
        torch.cuda.synchronize()
        pt.copy_(torch.from_numpy(p))
        torch.cuda.synchronize()
        st.st_partial_distill(desc, fd, labd, pt, wl.steps, wl.lr, losses=losses, mious=mious, confusion=conf,
                              pred=pred, workspace=ws, stream=stream, graph=graph)
        torch.cuda.synchronize()
        return [t.cpu().numpy().copy() for t in (pt, losses, mious, conf, pred)]

    plain = run(False)
    for _ in range(2):
        for a, b in zip(run(True), plain):
            np.testing.assert_array_equal(a, b)
    assert st.st_graph_cache_size() >= 1
    st.st_graph_cache_clear()
