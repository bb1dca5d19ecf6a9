"""GPU parity of cg_train_step (forward, backward in inverse layer order, per-layer gradient
aggregation + update on the second stream) against the oracle's iteration, and the schedule
invariant: the overlapped two-stream step is bit-identical to the serial one-stream step."""
import numpy as np
import pytest
import torch

import cg_synth
import paper_1706_00095_amd as cg
from gpu_util import host, max_abs_rel
from net_util import GpuNet
from oracle import net as onet
from test_oracle_net import _small_alexnet_like

pytestmark = pytest.mark.gpu
TOL = 1e-3
SGD = (0.01, 0.9, 5e-4, 1.0)

NETS = {
    "tiny_cnn_cfg1": lambda: cg_synth.tiny_cnn_layers() + (10, 8, 4, "xavier", 1e-2, 0),
    "alexnet_like": lambda: _small_alexnet_like() + (7, 6, 4, "fan_in", 1e-3, 4),
    "inception": lambda: cg_synth.inception_layers(modules=2, cin=12, hw=6, num_classes=9) + (9, 5, 8, "fan_in", 1e-3, 5),
}


def _build(name):
    layers, in_shape, ncls, B, K, init, pstd, seed = NETS[name]()
    t = cg_synth.net_tensors(layers, in_shape, B, K, seed=seed, num_classes=ncls, init=init, peer_std=pstd)
    return layers, in_shape, B, t


@pytest.mark.parametrize("name", list(NETS))
def test_one_iteration_matches_oracle(orc32, name):
    layers, in_shape, B, t = _build(name)
    gn = GpuNet(layers, in_shape, B, t)
    gn.step(SGD)
    gn.sync()
    # oracle: same inputs
    buckets = {k: v.copy() for k, v in t["buckets"].items()}
    hist = {k: np.zeros_like(v) for k, v in buckets.items()}
    loss, acts, aux = onet.forward(orc32, layers, t["x"], buckets, t["labels"], t["masks"])
    grads, dact, _ = onet.backward(orc32, layers, t["x"], buckets, t["masks"], acts, aux)
    assert abs(float(host(gn.loss)[0]) - float(loss)) <= TOL * max(1.0, abs(float(loss)))
    for li in range(len(layers) - 1):
        if gn.fused(li):
            continue        # not materialised: the rectifier's output, checked at its own index, stands for it
        assert max_abs_rel(host(gn.act(li)), acts[li].ravel()) <= TOL, ("activation", li, layers[li]["kind"])
    # the library skips gradients that reach no parameter (e.g. a pool applied to the net input)
    needs = []
    for ly in layers:
        needs.append(ly["kind"] in ("conv", "fc") or any(i >= 0 and needs[i] for i in ly["inputs"]))
    for li, dref in dact.items():
        if li == len(layers) - 1 or not needs[li] or gn.grad_folded(li):
            continue
        assert max_abs_rel(host(gn.act(li, 1)), dref.ravel()) <= TOL, ("gradient", li, layers[li]["kind"])
    for li in grads:
        assert max_abs_rel(host(gn.g[li]), grads[li]) <= TOL, ("g_local", li)
        # the update applied to the GPU's own local gradient is bit-exact (Eq. 1, fixed order) ...
        w, v = t["buckets"][li].copy(), np.zeros_like(t["buckets"][li])
        orc32.grad_reduce_sgd(w, v, host(gn.g[li]), t["peers"][li], *SGD)
        assert host(gn.w[li]).tobytes() == w.tobytes() and host(gn.v[li]).tobytes() == v.tobytes()
        # ... and the whole iteration's model agrees with the oracle's to the conv tolerance
        orc32.grad_reduce_sgd(buckets[li], hist[li], grads[li], t["peers"][li], *SGD)
        step_ref = buckets[li] - t["buckets"][li]
        step_got = host(gn.w[li]) - t["buckets"][li]
        assert max_abs_rel(step_got, step_ref) <= TOL


@pytest.mark.parametrize("name", list(NETS))
def test_overlapped_schedule_is_bit_identical_to_serial(name):
    """Strictly synchronous semantics (section 2.2): overlapping the per-layer updates with
    the rest of backward must not change a single bit, over consecutive iterations (the
    second one exercises the per-layer wait of forward on the previous update)."""
    layers, in_shape, B, t = _build(name)
    a, b = GpuNet(layers, in_shape, B, t), GpuNet(layers, in_shape, B, t)
    for _ in range(3):
        a.step(SGD, cg.CG_STEP_OVERLAP)
        b.step(SGD, cg.CG_STEP_SERIAL)
    a.sync(); b.sync()
    assert torch.equal(a.loss[:1], b.loss[:1])
    for li in a.w:
        assert torch.equal(a.w[li], b.w[li]) and torch.equal(a.v[li], b.v[li]) and torch.equal(a.g[li], b.g[li])
    # and it moved: three steps change the model
    assert not torch.equal(a.w[max(a.w)], GpuNet(layers, in_shape, B, t).w[max(a.w)])


@pytest.mark.parametrize("name", ["alexnet_like", "inception"])
def test_joined_step_recorded_into_a_hip_graph_replays_bit_identically(name):
    """CG_STEP_JOIN leaves nothing on a stream the caller did not pass and depends on no event of the
    call before, so stream capture on the compute stream records the whole iteration (three streams,
    their events) into one HIP graph.  Every replay, with eager work and synchronisation between
    replays, must give the bits of the eager iteration with the same number."""
    layers, in_shape, B, t = _build(name)
    a, b = GpuNet(layers, in_shape, B, t), GpuNet(layers, in_shape, B, t)
    ref = []
    for _ in range(5):
        a.step(SGD, cg.CG_STEP_JOIN)
        a.sync()
        ref.append((a.loss[:1].clone(), {li: (a.w[li].clone(), a.v[li].clone(), a.g[li].clone()) for li in a.w}))
    # and the joined form itself changes nothing against the plain overlapped schedule
    c = GpuNet(layers, in_shape, B, t)
    for _ in range(5):
        c.step(SGD, cg.CG_STEP_OVERLAP)
    c.sync()
    assert all(torch.equal(c.w[li], a.w[li]) and torch.equal(c.v[li], a.v[li]) for li in a.w)

    def same(k):
        loss, state = ref[k]
        assert torch.equal(b.loss[:1], loss), k
        for li, (w, v, g) in state.items():
            assert torch.equal(b.w[li], w) and torch.equal(b.v[li], v) and torch.equal(b.g[li], g), (k, li)

    b.step(SGD, cg.CG_STEP_JOIN)          # iteration 0 eagerly: the captured call follows a joined one
    b.sync()
    same(0)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=b.s0):
        b.step(SGD, cg.CG_STEP_JOIN)      # recorded, not run
    b.sync()
    same(0)
    for k in range(1, 5):
        with torch.cuda.stream(b.s0):
            graph.replay()
        b.sync()
        same(k)
        junk = torch.randn(1 << 16, device="cuda")       # eager work between replays
        assert bool(torch.isfinite(junk.sum()))
        torch.cuda.synchronize()


@pytest.mark.parametrize("flags", [cg.CG_STEP_TREE_SUM, cg.CG_STEP_TREE_SUM | cg.CG_STEP_SERIAL])
def test_step_with_tree_ordered_gradient_sum(orc32, flags):
    """CG_STEP_TREE_SUM: every layer's update is the tree-order oracle's, bit for bit, on the local
    gradient the step produced (K = 8 peers, where the two associations differ); the local
    gradients themselves are those of the plain step."""
    layers, in_shape, B, t = _build("inception")
    a, b = GpuNet(layers, in_shape, B, t), GpuNet(layers, in_shape, B, t)
    a.step(SGD, flags)
    b.step(SGD, flags & cg.CG_STEP_SERIAL)
    a.sync(); b.sync()
    differs = False
    for li in a.w:
        assert torch.equal(a.g[li], b.g[li])
        w, v = t["buckets"][li].copy(), np.zeros_like(t["buckets"][li])
        orc32.grad_reduce_sgd(w, v, host(a.g[li]), t["peers"][li], *SGD, order="tree")
        assert host(a.w[li]).tobytes() == w.tobytes() and host(a.v[li]).tobytes() == v.tobytes(), li
        differs = differs or not torch.equal(a.v[li], b.v[li])
    assert differs


@pytest.mark.parametrize("name", ["alexnet_like", "inception"])
def test_schedules_mixed_from_call_to_call_agree_with_the_serial_one(name):
    """Overlapped, joined and one-stream calls in any succession: each call waits for exactly what
    the call before left pending, so five mixed iterations give the bits of five serial ones."""
    layers, in_shape, B, t = _build(name)
    a, b = GpuNet(layers, in_shape, B, t), GpuNet(layers, in_shape, B, t)
    for flags in (cg.CG_STEP_OVERLAP, cg.CG_STEP_JOIN, cg.CG_STEP_SERIAL, cg.CG_STEP_OVERLAP, cg.CG_STEP_JOIN):
        a.step(SGD, flags)
        b.step(SGD, cg.CG_STEP_SERIAL)
    a.sync(); b.sync()
    assert torch.equal(a.loss[:1], b.loss[:1])
    for li in a.w:
        assert torch.equal(a.w[li], b.w[li]) and torch.equal(a.v[li], b.v[li]) and torch.equal(a.g[li], b.g[li])


def test_launch_counter_counts_the_kernels_of_a_step():
    """cg_debug_launch_count grows by one per kernel the library launches: by the same amount for every step
    of a net (the launch sequence depends on shapes only), and by exactly one for the calibration copy."""
    layers, in_shape, B, t = _build("inception")
    gn = GpuNet(layers, in_shape, B, t)
    counts = []
    for _ in range(3):
        c0 = cg.cg_debug_launch_count()
        gn.step(SGD)
        counts.append(cg.cg_debug_launch_count() - c0)
    gn.sync()
    assert counts[0] == counts[1] == counts[2] and counts[0] >= len(layers), counts
    a = torch.zeros(1024, device="cuda")
    b = torch.empty_like(a)
    c0 = cg.cg_debug_launch_count()
    cg.cg_debug_copy(b, a, a.numel() * 4)
    assert cg.cg_debug_launch_count() - c0 == 1
    torch.cuda.synchronize()


def test_loss_decreases_over_iterations_on_fixed_batch():
    layers, in_shape, B, t = _build("tiny_cnn_cfg1")
    for li in t["peers"]:
        t["peers"][li] = []        # single worker: plain SGD on one batch must reduce its loss
    gn = GpuNet(layers, in_shape, B, t)
    losses = []
    for _ in range(30):
        gn.step((0.05, 0.9, 0.0, 1.0))
        gn.sync()
        losses.append(float(host(gn.loss)[0]))
    assert losses[-1] < losses[0] - 0.3 and all(np.isfinite(losses))


def test_errors(orc32):
    layers, in_shape, B, t = _build("tiny_cnn_cfg1")
    gn = GpuNet(layers, in_shape, B, t)
    small = torch.empty(64, dtype=torch.uint8, device="cuda")
    with pytest.raises(cg.CgError) as e:
        cg.cg_train_step(gn.net, gn.x, gn.labels, None, cg.cg_sgd(*SGD), small, gn.s0, gn.s1, gn.loss, 0)
    assert e.value.code == cg.CG_ENOSPC
    with pytest.raises(cg.CgError) as e:      # both streams equal without the serial flag
        cg.cg_train_step(gn.net, gn.x, gn.labels, None, cg.cg_sgd(*SGD), gn.ws, gn.s0, gn.s0, gn.loss, 0)
    assert e.value.code == cg.CG_EINVAL
    bad = [dict(kind="relu", inputs=[-1])]
    with pytest.raises(cg.CgError):
        cg.Net(bad, 2, (3, 4, 4))            # no loss layer
