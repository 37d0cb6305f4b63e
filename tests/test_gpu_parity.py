"""HIP library vs the fp64 oracle, element by element, through the C ABI.

Tolerances (per tensor, max|x - y| / max|y|): 1e-4 on logits, values and
probabilities; 1e-3 on returns, head gradients, every parameter tensor's
gradient and the updated theta and g.  Sampling is exact given the library's
own fp32 probabilities, and equal to the oracle's away from CDF edges.
"""
import numpy as np
import pytest

import ga3c_synth as synth
import oracle as orc

pytestmark = pytest.mark.gpu

TOL_FWD = 1e-4
TOL_BWD = 1e-3
# math = 1 (operands of every contraction rounded to bfloat16 on both sides): the two sides round the same real
# numbers, computed in fp32 here and in fp64 there.  Nearly always the roundings agree and the results differ by fp32
# accumulation only (1e-6); but a value within ~1e-7 of a rounding boundary goes to different bfloat16 neighbours on
# the two sides, which changes one term of a later sum by up to 2^-7 of itself, and the sums of these layers cancel
# (sum |t| is 10-20 times |sum t|), so a single such operand can move an output by a fraction of a percent.  The bound
# is therefore set by the format, two bfloat16 units in the last place, not by the accumulation.
TOL_FWD_BF16 = 2.0 ** -6
TOL_BWD_BF16 = 2.0 ** -6


def rel_err(x, y):
    x = np.asarray(x, np.float64); y = np.asarray(y, np.float64)
    return np.abs(x - y).max() / max(np.abs(y).max(), 1e-12)


def med_err(x, y):
    """Median absolute difference over the tensor, relative to its largest reference value."""
    x = np.asarray(x, np.float64); y = np.asarray(y, np.float64)
    return np.median(np.abs(x - y)) / max(np.abs(y).max(), 1e-12)


# math = 1: the max-error bound above has to leave room for the rare operand that rounds differently on the two sides.
# Forward: the typical element must still agree as closely as fp32 accumulation allows (an operand left unrounded on
# one side moves the median logit by 7e-4 or more).  Backward: the whole-network statistics cannot separate a correct
# kernel from one that forgot a rounding (tests/test_oracle_pins.py shows both facts), so every layer is also compared
# on its own, from the inputs the library itself used (check_layers): then both sides round the same numbers, only
# fp32 accumulation is left, and the bound is STAGE_TOL_BF16, a twentieth of what any unrounded operand class causes.
MED_FWD_BF16 = 2e-5
MED_BWD_BF16 = 1e-3
STAGE_TOL_BF16 = 1e-5          # observed on the GPU: 4e-7 at most, over every layer of every math = 1 test


@pytest.fixture(scope="module")
def G():
    import torch
    import paper_1611_06256_amd as g
    assert torch.cuda.is_available()
    return g


def to_orc(desc):
    return orc.Net(in_c=desc.in_c, in_h=desc.in_h, in_w=desc.in_w, conv=tuple(desc.conv),
                   fc_units=desc.fc_units, n_actions=desc.n_actions, math=desc.math)


def tols(desc):
    """(forward, backward, distance from a CDF edge beyond which the draws must agree) for the net's arithmetic."""
    return (TOL_FWD, TOL_BWD, 1e-5) if desc.math == 0 else (TOL_FWD_BF16, TOL_BWD_BF16, 5e-4)


GENERIC = False     # set by the fixture below: run every test on both kernel families


@pytest.fixture(autouse=True, params=["shape-specific", "generic"])
def kernel_family(request):
    global GENERIC
    GENERIC = request.param == "generic"
    yield


def make(G, desc, max_pred, max_train, seed):
    import torch
    net = G.Ga3c(desc, max_pred, max_train)
    net.use_generic_kernels(GENERIC)
    onet = to_orc(desc)
    assert net.n_params == orc.param_count(onet)
    assert net.offsets() == orc.offsets(onet)
    theta = synth.perturbed_theta(seed, net.offsets(), net.n_params)
    net.params_set(torch.from_numpy(theta).cuda(), 0)
    return net, onet, theta


def run_predict(G, net, frames, uniforms=None):
    import torch
    B, A = frames.shape[0], net.n_actions
    fr = torch.from_numpy(frames).cuda()
    logits = torch.full((B, A), float("nan"), device="cuda"); values = torch.full((B,), float("nan"), device="cuda")
    probs = torch.full((B, A), float("nan"), device="cuda")
    actions = torch.full((B,), -1, dtype=torch.int32, device="cuda") if uniforms is not None else None
    u = torch.from_numpy(uniforms).cuda() if uniforms is not None else None
    print(f"predict B={B} A={A}", flush=True)
    net.predict(fr, uniforms=u, logits=logits, values=values, probs=probs, actions=actions)
    torch.cuda.synchronize()
    return (logits.cpu().numpy(), values.cpu().numpy(), probs.cpu().numpy(),
            actions.cpu().numpy() if actions is not None else None)


def check_predict(G, desc, B, seed, frames=None):
    net, onet, theta = make(G, desc, max(B, 1), 0, seed)
    if frames is None:
        frames = synth.uniform_frames(seed + 1, (B, desc.in_c, desc.in_h, desc.in_w))
    u = synth.uniforms(seed + 2, B)
    lg, vl, pr, ac = run_predict(G, net, frames, u)
    ref = orc.forward(onet, theta, frames)
    tf, _, edge = tols(desc)
    assert rel_err(lg, ref["logits"]) <= tf
    assert rel_err(vl, ref["values"]) <= tf
    assert rel_err(pr, ref["probs"]) <= tf
    if desc.math == 1:
        assert med_err(lg, ref["logits"]) <= MED_FWD_BF16 and med_err(pr, ref["probs"]) <= MED_FWD_BF16
    np.testing.assert_allclose(pr.sum(1), 1.0, atol=2e-6)
    # (i) exact w.r.t. the library's own fp32 probabilities, summed left to right in fp32
    A = desc.n_actions
    want = np.full(B, A - 1, np.int32)
    for b in range(B):
        c = np.float32(0)
        for j in range(A):
            c = np.float32(c + pr[b, j])
            if c > u[b]:
                want[b] = j
                break
    np.testing.assert_array_equal(ac, want)
    # (ii) equal to the oracle's sample wherever u is not within 1e-5 of a CDF edge
    oa = orc.sample(ref["probs"], u.astype(np.float64))
    cdf = np.cumsum(ref["probs"], 1)
    far = (np.abs(cdf - u[:, None].astype(np.float64)) > edge).all(1)
    np.testing.assert_array_equal(ac[far], oa[far])
    assert far.mean() > (0.99 if desc.math == 0 else 0.85)
    net.close()
    return frames


TINY = dict(in_c=2, in_h=12, in_w=12, conv=((3, 4, 2), (4, 2, 1)), fc_units=5, n_actions=3)
TINY3 = dict(in_c=1, in_h=15, in_w=13, conv=((2, 5, 2), (3, 3, 1), (2, 2, 1)), fc_units=4, n_actions=4)
ODD = dict(in_c=3, in_h=23, in_w=19, conv=((5, 5, 3), (7, 3, 2)), fc_units=33, n_actions=7)


def test_predict_config0(G):
    # small net of Sec. 3.2, 6 actions, B = 8, uniform bytes
    check_predict(G, G.SMALL_NET(6), 8, synth.BASE_SEED)


@pytest.mark.parametrize("B", [1, 3, 70])
def test_predict_small18_ragged_batches(G, B):
    check_predict(G, G.SMALL_NET(18), B, synth.BASE_SEED + 10 + B,
                  frames=synth.rectangle_frames(synth.BASE_SEED + 1, B))


@pytest.mark.parametrize("shape", [TINY, TINY3, ODD])
def test_predict_odd_shapes(G, shape):
    check_predict(G, G.NetDesc(**shape), 37, 500)


def test_predict_large_net(G):
    check_predict(G, G.LARGE_NET(18), 19, synth.BASE_SEED + 3)


def test_predict_subset_of_outputs_and_empty(G):
    import torch
    net, onet, theta = make(G, G.SMALL_NET(6), 8, 0, 7)
    frames = synth.uniform_frames(8, (4, 4, 84, 84))
    values = torch.zeros(4, device="cuda")
    net.predict(torch.from_numpy(frames).cuda(), values=values)      # only values asked for
    torch.cuda.synchronize()
    assert rel_err(values.cpu().numpy(), orc.forward(onet, theta, frames)["values"]) <= TOL_FWD
    net.predict(torch.empty((0, 4, 84, 84), dtype=torch.uint8, device="cuda"))   # B = 0: no-op
    with pytest.raises(G.Ga3cError):
        net.predict(torch.zeros((9, 4, 84, 84), dtype=torch.uint8, device="cuda"))   # above capacity
    with pytest.raises(G.Ga3cError):
        net.predict(torch.from_numpy(frames).cuda(), actions=torch.zeros(4, dtype=torch.int32, device="cuda"))
    net.close()


def run_train(G, desc, N, T, seed, hp_kw, frames=None, g0_scale=0.0, steps=1, seg=None):
    """One or more updates on both sides, compared step by step.  seg = None: N segments of T frames; otherwise the
    dict of synth.ragged_segments (N segments of unequal length, T unused), which goes through the ragged entry
    point and the oracle's ragged update."""
    import torch
    from paper_1611_06256_amd.binding import stats_from_tensor
    nfr = N * T if seg is None else int(seg["seg_start"][-1])
    net, onet, theta = make(G, desc, N, nfr, seed)
    if frames is None:
        shape = (N, T) if seg is None else (nfr,)
        frames = synth.uniform_frames(seed + 1, shape + (desc.in_c, desc.in_h, desc.in_w))
    tr = synth.trajectories(seed + 2, N, T, desc.n_actions) if seg is None else seg
    # bootstrap value from the net itself, on N more frames, with the pre-update theta
    bf = synth.uniform_frames(seed + 3, (N, desc.in_c, desc.in_h, desc.in_w))
    boot_t = torch.zeros(N, device="cuda")
    net.predict(torch.from_numpy(bf).cuda(), values=boot_t)
    torch.cuda.synchronize()
    boot = boot_t.cpu().numpy()
    TF, TB, _ = tols(desc)
    assert rel_err(boot, orc.forward(onet, theta, bf)["values"]) <= TF
    g0 = (np.abs(synth.rng(seed + 4).standard_normal(net.n_params)) * g0_scale).astype(np.float32)
    net.params_set(torch.from_numpy(g0).cuda(), 1)
    hp = G.HParams(**hp_kw); ohp = orc.HParams(**hp_kw)
    stats_t = torch.zeros(8, dtype=torch.float32, device="cuda")
    d = dict(frames=torch.from_numpy(frames).cuda(), actions=torch.from_numpy(tr["actions"]).cuda(),
             rewards=torch.from_numpy(tr["rewards"]).cuda(), dones=torch.from_numpy(tr["dones"]).cuda())
    th_ref, g_ref = theta.astype(np.float64), g0.astype(np.float64)
    for step in range(steps):
        print(f"train N={N} T={T if seg is None else 'ragged'} frames={nfr} A={desc.n_actions} step={step}", flush=True)
        if seg is None:
            net.train_step(d["frames"], d["actions"], d["rewards"], d["dones"], boot_t, hp, stats=stats_t)
        else:
            net.train_step_ragged(d["frames"], d["actions"], d["rewards"], d["dones"],
                                  torch.from_numpy(seg["seg_start"]).cuda(), boot_t, hp, stats=stats_t)
        torch.cuda.synchronize()
        # the oracle starts each step from the library's own state, so that one
        # step's rounding does not compound into the next comparison
        if seg is None:
            ref = orc.train_step(onet, th_ref, g_ref, frames, tr["actions"], tr["rewards"], tr["dones"],
                                 boot.astype(np.float64), ohp)
        else:
            ref = orc.train_step_ragged(onet, th_ref, g_ref, frames, tr["actions"], tr["rewards"], tr["dones"],
                                        seg["seg_start"], boot.astype(np.float64), ohp)
        B, A = nfr, desc.n_actions
        R = net.train_debug_get(0, torch.empty(B, device="cuda")).cpu().numpy()
        lg = net.train_debug_get(1, torch.empty(B * A, device="cuda")).cpu().numpy().reshape(B, A)
        vl = net.train_debug_get(2, torch.empty(B, device="cuda")).cpu().numpy()
        dzv = net.train_debug_get(3, torch.empty(B * (A + 1), device="cuda")).cpu().numpy().reshape(B, A + 1)
        grad = net.params_get(2).cpu().numpy()
        th1 = net.params_get(0).cpu().numpy(); g1 = net.params_get(1).cpu().numpy()
        st = stats_from_tensor(stats_t)
        assert rel_err(R, ref["R"].reshape(-1)) <= TB
        assert rel_err(lg, ref["logits"]) <= TF
        assert rel_err(vl, ref["values"]) <= TF
        if desc.math == 1:
            assert med_err(lg, ref["logits"]) <= MED_FWD_BF16 and med_err(dzv[:, :A], ref["dZ"]) <= MED_BWD_BF16
        assert rel_err(dzv[:, :A], ref["dZ"]) <= TB
        assert rel_err(dzv[:, A], ref["dV"]) <= TB
        for name, (o, shape) in net.offsets().items():
            n = int(np.prod(shape))
            e = rel_err(grad[o:o + n], ref["grad"][o:o + n])
            assert e <= TB, (name, e)
            if desc.math == 1 and n >= 16:
                assert med_err(grad[o:o + n], ref["grad"][o:o + n]) <= MED_BWD_BF16, name
        assert rel_err(th1, ref["theta"]) <= TB
        # the update itself, not only theta (whose change is ~lr): compare the step taken
        assert rel_err(th1.astype(np.float64) - th_ref, ref["theta"] - th_ref) <= 2 * TB
        assert rel_err(g1, ref["g"]) <= TB
        for k in ("policy_loss", "value_loss", "entropy", "grad_norm", "clip_scale"):
            assert abs(st[k] - ref["stats"][k]) <= TB * max(abs(ref["stats"][k]), 1e-3), (k, st[k], ref["stats"][k])
        assert st["nonfinite"] == 0
        check_layers(net, onet, th_ref, frames, nfr)
        th_ref, g_ref = th1.astype(np.float64), g1.astype(np.float64)
    net.close()
    return ref


def check_layers(net, onet, theta, frames, B):
    """Every layer of the last update on its own: the oracle's single-layer functions get the inputs the library
    itself used (its stored activations and gradients), so an error is charged to the layer that made it, and with
    math = 1 both sides round identical numbers.  Bounds: the fp32 ones for math = 0, STAGE_TOL_BF16 for math = 1."""
    import torch
    m = onet.math
    tf, tb = (TOL_FWD, TOL_BWD) if m == 0 else (STAGE_TOL_BF16, STAGE_TOL_BF16)
    A, F = onet.n_actions, onet.fc_units
    v = orc.views(onet, theta.astype(np.float64))
    shapes = [(onet.in_c, onet.in_h, onet.in_w)]
    for (oc, k, s) in onet.conv:
        shapes.append((oc, (shapes[-1][1] - k) // s + 1, (shapes[-1][2] - k) // s + 1))

    def get(which, shape):
        n = int(np.prod(shape))
        return net.train_debug_get(which, torch.empty(n, device="cuda")).cpu().numpy().astype(np.float64).reshape(shape)

    nl = len(onet.conv)
    act = [frames.reshape((B,) + shapes[0]).astype(np.float64) / 255.0] + [get(4 + l, (B,) + shapes[l + 1]) for l in range(nl)]
    dact = [get(10 + l, (B,) + shapes[l + 1]) for l in range(nl)]
    h = get(8, (B, F)); dh = get(9, (B, F))
    zv = np.concatenate([get(1, (B, A)), get(2, (B, 1))], 1)
    dzv = get(3, (B, A + 1))
    grad = orc.views(onet, net.params_get(2).cpu().numpy().astype(np.float64))
    worst = {}

    def close(tag, got, want, tol):
        e = rel_err(got, want)
        worst[tag] = e
        assert e <= tol, (tag, e, tol)

    for l, (oc, k, s) in enumerate(onet.conv):
        close(f"conv{l + 1} out", act[l + 1],
              orc.conv_layer_forward(act[l], v[f"conv{l + 1}.W"], v[f"conv{l + 1}.b"], s, m, 255.0 if l == 0 else 1.0), tf)
    flat = act[nl].reshape(B, -1)
    close("fc out", h, orc.dense_forward(flat, v["fc.W"], v["fc.b"], True, m), tf)
    Wh = np.concatenate([v["policy.W"], v["value.W"]], 0); bh = np.concatenate([v["policy.b"], v["value.b"]])
    close("heads out", zv, orc.dense_forward(h, Wh, bh, False, m), tf)
    gW, gb, dx = orc.dense_backward(h, Wh, dzv, m)
    close("policy.W", grad["policy.W"], gW[:A], tb); close("policy.b", grad["policy.b"], gb[:A], tb)
    close("value.W", grad["value.W"], gW[A:], tb); close("value.b", grad["value.b"], gb[A:], tb)
    close("dh", dh, dx * (h > 0), tb)
    gW, gb, dx = orc.dense_backward(flat, v["fc.W"], dh, m)
    close("fc.W", grad["fc.W"], gW, tb); close("fc.b", grad["fc.b"], gb, tb)
    close(f"d conv{nl}", dact[nl - 1].reshape(B, -1), dx * (flat > 0), tb)
    for l in reversed(range(nl)):
        oc, k, s = onet.conv[l]
        gW, gb, dx = orc.conv_layer_backward(act[l], v[f"conv{l + 1}.W"], s, act[l + 1], dact[l], m, 255.0 if l == 0 else 1.0,
                                             want_dx=l > 0)
        close(f"conv{l + 1}.W", grad[f"conv{l + 1}.W"], gW, tb); close(f"conv{l + 1}.b", grad[f"conv{l + 1}.b"], gb, tb)
        if l > 0:
            close(f"d conv{l}", dact[l - 1], dx * (act[l] > 0), tb)
    print("layer by layer, math", m, " ".join(f"{k}:{e:.1e}" for k, e in worst.items()), flush=True)


def test_train_config0(G):
    # 8 agents x t_max = 5, 6 actions, gamma .99, beta .01, lr 3e-4, decay .99, eps .1, no clip
    run_train(G, G.SMALL_NET(6), 8, 5, synth.BASE_SEED, dict(), g0_scale=0.0)


def test_train_config2_clip_two_steps(G):
    # 18 actions, clip 40, rectangle frames, non-zero RMSProp state, two consecutive updates
    N, T = 32, 5
    frames = synth.rectangle_frames(synth.BASE_SEED + 2, N * T).reshape(N, T, 4, 84, 84)
    ref = run_train(G, G.SMALL_NET(18), N, T, synth.BASE_SEED + 2, dict(clip_norm=40.0), frames=frames,
                    g0_scale=1e-3, steps=2)
    assert ref["stats"]["grad_norm"] > 0


def test_a_large_update_keeps_the_derived_filter_fragments_current(G):
    # the kernel that updates the parameters also rewrites the split filter fragments that the fused forward kernel and
    # the conv2 input-gradient kernel read; with a learning rate this large a fragment left behind by one update shows
    # in the next step's layer-by-layer comparison (conv outputs, d conv1), which uses the parameters of that step
    # (a third update of this size drives probabilities to zero and the comparison into 0 * inf)
    ref = run_train(G, G.SMALL_NET(6), 8, 5, 4300, dict(lr=0.02), steps=2)
    assert ref["stats"]["grad_norm"] > 0


def test_train_clip_active(G):
    ref = run_train(G, G.SMALL_NET(6), 6, 5, 900, dict(clip_norm=0.5, lr=1e-3))
    assert ref["stats"]["clip_scale"] < 1.0


def test_predict_follows_a_large_update(G):
    # whatever the library derives from the parameters (split filter fragments) must follow an update, an explicit
    # params_set and a re-initialisation: a large learning rate makes a stale copy show
    import torch
    N, T, A = 16, 5, 6
    desc = G.SMALL_NET(A)
    net, onet, theta = make(G, desc, N * T, N * T, 4242)
    frames = synth.rectangle_frames(4243, N * T).reshape(N, T, 4, 84, 84)
    tr = synth.trajectories(4244, N, T, A)
    boot = torch.zeros(N, device="cuda")
    flat = frames.reshape(N * T, 4, 84, 84)

    def check(th):
        lg, vl, pr, _ = run_predict(G, net, flat)
        ref = orc.forward(onet, th.astype(np.float64), flat)
        assert rel_err(lg, ref["logits"]) <= TOL_FWD
        assert rel_err(vl, ref["values"]) <= TOL_FWD

    for step in range(2):
        net.train_step(torch.from_numpy(frames).cuda(), torch.from_numpy(tr["actions"]).cuda(),
                       torch.from_numpy(tr["rewards"]).cuda(), torch.from_numpy(tr["dones"]).cuda(), boot,
                       G.HParams(lr=0.02))
        th1 = net.params_get(0).cpu().numpy()
        assert rel_err(th1, theta) > 1e-2          # the update moved the parameters visibly
        check(th1)
    th2 = synth.perturbed_theta(4245, net.offsets(), net.n_params)
    net.params_set(torch.from_numpy(th2).cuda(), 0)
    check(th2)
    net.params_init(77)
    check(net.params_get(0).cpu().numpy())
    net.close()


@pytest.mark.parametrize("PB", [64, 8])
def test_predictions_on_one_stream_while_training_on_another(G, PB):
    # the way the benchmark and the scheduler submit work (Sec. 4.1: predictors and trainers share the GPU): every
    # prediction must see one whole parameter set, the one before or the one after the update, never a mixture,
    # and the update itself must not be disturbed by the predictions reading next to it.  PB frames per prediction:
    # 64 go through the three-kernel path, 8 through the one-launch kernel (which reads the filter fragments that
    # the update's last kernel rewrites).
    import torch
    N, T, A = 64, 5, 18
    desc = G.SMALL_NET(A)
    net, onet, theta = make(G, desc, N, N * T, 5150)
    frames = synth.rectangle_frames(5151, N * T).reshape(N, T, 4, 84, 84)
    tr = synth.trajectories(5152, N, T, A)
    boot = synth.rng(5153).standard_normal(N).astype(np.float32)
    hp_kw = dict(lr=0.02)               # large, so that the two parameter sets give visibly different outputs
    ref = orc.train_step(onet, theta.astype(np.float64), np.zeros(net.n_params), frames, tr["actions"], tr["rewards"],
                         tr["dones"], boot.astype(np.float64), orc.HParams(**hp_kw))
    pf = [frames[:PB, t] for t in range(T)]
    want = [(orc.forward(onet, theta.astype(np.float64), f)["logits"], orc.forward(onet, ref["theta"], f)["logits"])
            for f in pf]
    assert all(rel_err(a, b) > 1e-2 for a, b in want)
    d = dict(frames=torch.from_numpy(frames).cuda(), actions=torch.from_numpy(tr["actions"]).cuda(),
             rewards=torch.from_numpy(tr["rewards"]).cuda(), dones=torch.from_numpy(tr["dones"]).cuda())
    boot_t = torch.from_numpy(boot).cuda()
    pft = [torch.from_numpy(np.ascontiguousarray(f)).cuda() for f in pf]
    outs = [torch.full((PB, A), float("nan"), device="cuda") for _ in range(3 * T)]
    sp, st = torch.cuda.Stream(), torch.cuda.Stream()
    torch.cuda.synchronize()
    print("predictions and a training step on two streams", flush=True)
    for k in range(T):
        net.predict(pft[k], logits=outs[k], stream=sp)
    net.train_step(d["frames"], d["actions"], d["rewards"], d["dones"], boot_t, G.HParams(**hp_kw), stream=st)
    for k in range(T, 3 * T):
        net.predict(pft[k % T], logits=outs[k], stream=sp)
    torch.cuda.synchronize()
    th1 = net.params_get(0).cpu().numpy()
    assert rel_err(th1, ref["theta"]) <= TOL_BWD
    assert rel_err(th1.astype(np.float64) - theta, ref["theta"] - theta) <= 2 * TOL_BWD
    seen_new = False
    for k in range(3 * T):
        lg = outs[k].cpu().numpy()
        e_old, e_new = rel_err(lg, want[k % T][0]), rel_err(lg, want[k % T][1])
        assert min(e_old, e_new) <= TOL_FWD, (k, e_old, e_new)
        assert not (seen_new and e_new > TOL_FWD), f"prediction {k} went back to the old parameters"
        seen_new = seen_new or e_new <= TOL_FWD
    lg, _, _, _ = run_predict(G, net, pf[0])       # after everything has finished: the new parameters
    assert rel_err(lg, want[0][1]) <= TOL_FWD
    net.close()


@pytest.mark.parametrize("shape,N,T", [(TINY, 13, 5), (TINY3, 9, 3), (ODD, 11, 4)])
def test_train_odd_shapes(G, shape, N, T):
    run_train(G, G.NetDesc(**shape), N, T, 600, dict(beta=0.05, value_coef=0.5, gamma=0.9), g0_scale=1e-2)


def test_train_eps_variant(G):
    # Eq. 5 with epsilon > 0
    run_train(G, G.NetDesc(**ODD), 11, 4, 700, dict(beta=0.05, log_eps=1e-3))
    run_train(G, G.SMALL_NET(6), 4, 5, 701, dict(log_eps=1e-6))


def test_eps_variant_silences_a_near_zero_probability_sample(G):
    # Eq. 5 discussion: with pi(a) ~ 0 the factor d log(pi + eps) / d pi = 1 / (pi + eps) is bounded, and the
    # policy-gradient term of such a sample, (pi / (pi + eps)) * advantage, vanishes; with eps = 0 it is a full
    # -advantage on the logit of the action taken.  Policy bias of action 0 pushed to -60, every sample took action 0.
    import torch
    from paper_1611_06256_amd.binding import stats_from_tensor
    N, T, A = 6, 5, 6
    desc = G.SMALL_NET(A)
    norms = {}
    for eps in (0.0, 1e-2):
        net, onet, theta = make(G, desc, N * T, N * T, 7300)
        ob, _ = net.offsets()["policy.b"]
        theta = theta.copy(); theta[ob] = -60.0
        net.params_set(torch.from_numpy(theta).cuda(), 0)
        frames = synth.rectangle_frames(7301, N * T).reshape(N, T, 4, 84, 84)
        tr = synth.trajectories(7302, N, T, A)
        acts = np.zeros_like(tr["actions"])
        boot = np.zeros(N, np.float32)
        kw = dict(beta=0.0, value_coef=0.0, log_eps=eps)
        stats_t = torch.zeros(8, device="cuda")
        print(f"train eps={eps} with pi(a) ~ e^-60", flush=True)
        net.train_step(torch.from_numpy(frames).cuda(), torch.from_numpy(acts).cuda(), torch.from_numpy(tr["rewards"]).cuda(),
                       torch.from_numpy(tr["dones"]).cuda(), torch.from_numpy(boot).cuda(), G.HParams(**kw), stats=stats_t)
        torch.cuda.synchronize()
        ref = orc.train_step(onet, theta.astype(np.float64), np.zeros(net.n_params), frames, acts, tr["rewards"], tr["dones"],
                             boot.astype(np.float64), orc.HParams(**kw))
        grad = net.params_get(2).cpu().numpy()
        st = stats_from_tensor(stats_t)
        assert st["nonfinite"] == 0 and np.isfinite(st["policy_loss"])
        scale = max(np.abs(ref["grad"]).max(), 1e-30)
        if eps == 0.0:
            assert np.abs(grad - ref["grad"]).max() <= TOL_BWD * scale
        else:
            assert np.abs(grad).max() < 1e-20 and np.abs(ref["grad"]).max() < 1e-20
        norms[eps] = float(np.linalg.norm(grad))
        net.close()
    assert norms[0.0] > 1e-2 and norms[1e-2] < 1e-20 * norms[0.0] + 1e-20


def paper_family_net(G, stride, n_actions=18):
    # Sec. 5 (GPU utilization and DNN size), footnote: 32 filters in the first layer, a third convolution of 64
    # filters of 4x4 with stride 2, first-layer stride 4, 3, 2 or 1; the stride-1 member has a 4 times larger fully
    # connected layer.  VALID arithmetic gives 84 -> 20/26/39/77 -> 9/12/18/37 -> 3/5/8/17.
    return G.NetDesc(in_c=4, in_h=84, in_w=84, conv=((32, 8, stride), (32, 4, 2), (64, 4, 2)),
                     fc_units=1024 if stride == 1 else 256, n_actions=n_actions)


@pytest.mark.parametrize("stride,B,N,T", [(4, 5, 2, 3), (3, 5, 2, 3), (2, 4, 2, 2), (1, 3, 1, 2)])
def test_predict_and_train_paper_family_net(G, stride, B, N, T):
    # the four members of the paper's larger-network family; but for the stride-4 member's first layer and the
    # backward pass of its second one (a 4x4 stride-2 layer on 20x20 maps, which the conv2 backward kernels take),
    # every layer runs on the any-shape kernels
    desc = paper_family_net(G, stride)
    check_predict(G, desc, B, 7400 + stride, frames=synth.rectangle_frames(7401 + stride, B))
    run_train(G, desc, N, T, 7410 + stride, dict(clip_norm=40.0),
              frames=synth.rectangle_frames(7420 + stride, N * T).reshape(N, T, 4, 84, 84))


def test_predict_and_train_forty_actions(G):
    # more than 31 actions: the heads, the loss and the heads' backward pass run as separate kernels in training
    # (the fused kernel gives a thread to every (frame, output) pair of 8 frames)
    desc = G.SMALL_NET(40)
    check_predict(G, desc, 9, 7500, frames=synth.rectangle_frames(7501, 9))
    run_train(G, desc, 5, 5, 7510, dict(clip_norm=40.0), frames=synth.rectangle_frames(7511, 25).reshape(5, 5, 4, 84, 84))


@pytest.mark.parametrize("A,F", [(1, 5), (2, 8), (21, 12), (31, 16), (32, 16), (63, 64)])
def test_action_count_edges(G, A, F):
    # one action (softmax of a single logit), the counts around which the head kernels change their thread layout
    # (20/21 in predictions, 31/32 in training) and the largest count the interface takes
    shape = dict(TINY, fc_units=F, n_actions=A)
    check_predict(G, G.NetDesc(**shape), 11, 7600 + A)
    if A > 1:
        run_train(G, G.NetDesc(**shape), 7, 3, 7700 + A, dict(beta=0.05, value_coef=0.5, gamma=0.9), g0_scale=1e-2)
        return
    # one action: pi = 1, so the policy and entropy terms and their gradients are exactly zero in exact arithmetic
    # (relative errors against a zero reference mean nothing); the value path must still match
    import torch
    N, T = 7, 3
    desc = G.NetDesc(**shape)
    net, onet, theta = make(G, desc, N, N * T, 7700)
    frames = synth.uniform_frames(7701, (N, T, desc.in_c, desc.in_h, desc.in_w))
    tr = synth.trajectories(7702, N, T, A)
    boot = synth.rng(7703).standard_normal(N).astype(np.float32)
    kw = dict(beta=0.05, value_coef=0.5, gamma=0.9)
    print("train with a single action", flush=True)
    net.train_step(torch.from_numpy(frames).cuda(), torch.from_numpy(tr["actions"]).cuda(), torch.from_numpy(tr["rewards"]).cuda(),
                   torch.from_numpy(tr["dones"]).cuda(), torch.from_numpy(boot).cuda(), G.HParams(**kw))
    torch.cuda.synchronize()
    ref = orc.train_step(onet, theta.astype(np.float64), np.zeros(net.n_params), frames, tr["actions"], tr["rewards"],
                         tr["dones"], boot.astype(np.float64), orc.HParams(**kw))
    grad = net.params_get(2).cpu().numpy()
    scale = np.abs(ref["grad"]).max()
    assert scale > 1e-3
    assert np.abs(grad - ref["grad"]).max() <= TOL_BWD * scale
    for name in ("policy.W", "policy.b"):
        o, shp = net.offsets()[name]
        assert np.abs(grad[o:o + int(np.prod(shp))]).max() <= 1e-6 * scale
    assert rel_err(net.params_get(0).cpu().numpy(), ref["theta"]) <= TOL_BWD
    net.close()


def test_small_net_most_actions(G):
    # the interface's largest action count on the small network
    desc = G.SMALL_NET(63)
    check_predict(G, desc, 6, 7800, frames=synth.rectangle_frames(7801, 6))
    run_train(G, desc, 2, 5, 7810, dict(clip_norm=40.0), frames=synth.rectangle_frames(7811, 10).reshape(2, 5, 4, 84, 84))


def test_wide_fc_most_actions_that_fit(G):
    # the heads keep both weight matrices in LDS: (n_actions + 5) * (fc_units + 16) <= 40960 floats, i.e. at most
    # 34 actions with 1024 hidden units; the three head kernels then take more than 64 KB of LDS each
    shape = dict(TINY, fc_units=1024)
    check_predict(G, G.NetDesc(**dict(shape, n_actions=34)), 9, 7820)
    run_train(G, G.NetDesc(**dict(shape, n_actions=34)), 5, 3, 7830, dict(beta=0.05, value_coef=0.5, gamma=0.9), g0_scale=1e-2)
    with pytest.raises(G.Ga3cError):
        G.Ga3c(G.NetDesc(**dict(shape, n_actions=35)), 4, 0)


@pytest.mark.parametrize("N,T", [(1, 1), (3, 1), (1, 7), (2, 150)])
def test_segment_length_edges(G, N, T):
    # one-step segments, a single agent, and segments so long that the rewards of a block's agents do not fit the
    # training heads kernel's LDS copy (it then reads them from global memory)
    run_train(G, G.NetDesc(**TINY), N, T, 7900 + 10 * N + T, dict(beta=0.02, value_coef=0.5, gamma=0.97), g0_scale=1e-2)


@pytest.mark.parametrize("nseg,t_max,A", [(13, 5, 18), (40, 5, 6), (3, 1, 4), (1, 9, 3), (7, 40, 40)])
def test_train_ragged_segments(G, nseg, t_max, A):
    # Sec. 4.1: agents hand in fewer than t_max experiences when the episode ends.  Segments of mixed length through
    # the fused heads kernel (A <= 31) and through the separate loss kernel (A = 40), on the small net for the first
    # case and a tiny net otherwise; t_max = 1 makes every segment one frame, nseg = 1 a single segment.
    seg = synth.ragged_segments(8100 + nseg, nseg, t_max, A, p_short=0.5)
    if nseg == 13:
        F = int(seg["seg_start"][-1])
        run_train(G, G.SMALL_NET(A), nseg, t_max, 8110, dict(clip_norm=40.0), frames=synth.rectangle_frames(8111, F), seg=seg)
    else:
        run_train(G, G.NetDesc(**dict(TINY, fc_units=12, n_actions=A)), nseg, t_max, 8120 + nseg,
                  dict(beta=0.02, value_coef=0.5, gamma=0.97, lr=1e-2), g0_scale=1e-2, seg=seg, steps=2 if nseg == 40 else 1)
        # (lr = 1e-2: with a handful of frames the default step is a few fp32 units in the last place of theta, too
        # coarse for the comparison of the step taken)


def test_ragged_with_equal_lengths_is_the_rectangular_update_bit_for_bit(G):
    # the two entry points differ only in how a frame finds its segment; an empty segment in the table changes nothing
    import torch
    N, T, A = 9, 5, 6
    desc = G.NetDesc(**dict(TINY, n_actions=A))
    frames = torch.from_numpy(synth.uniform_frames(8201, (N, T, desc.in_c, desc.in_h, desc.in_w))).cuda()
    tr = synth.trajectories(8202, N, T, A)
    ac, rw, dn = (torch.from_numpy(tr[k]).cuda() for k in ("actions", "rewards", "dones"))
    boot = torch.from_numpy(synth.rng(8203).standard_normal(N).astype(np.float32)).cuda()
    hp = G.HParams(clip_norm=1.0, gamma=0.9)
    out = []
    for mode in ("rect", "ragged", "ragged_with_empty"):
        net = G.Ga3c(desc, 4, N * T)
        net.use_generic_kernels(GENERIC)
        net.params_init(77)
        print("mode", mode, flush=True)
        if mode == "rect":
            net.train_step(frames, ac, rw, dn, boot, hp)
        else:
            start = np.arange(N + 1, dtype=np.int32) * T
            b = boot
            if mode == "ragged_with_empty":
                start = np.concatenate([start[:4], start[3:4], start[4:]]).astype(np.int32)
                b = torch.cat([boot[:3], torch.full((1,), 123.0, device="cuda"), boot[3:]])
            net.train_step_ragged(frames.reshape(N * T, *frames.shape[2:]), ac.reshape(-1), rw.reshape(-1), dn.reshape(-1),
                                  torch.from_numpy(start).cuda(), b, hp)
        torch.cuda.synchronize()
        out.append((net.params_get(0).cpu().numpy(), net.params_get(2).cpu().numpy(),
                    net.train_debug_get(0, torch.empty(N * T, device="cuda")).cpu().numpy()))
        net.close()
    for o in out[1:]:
        for x, y in zip(o, out[0]):
            np.testing.assert_array_equal(x, y)


def test_ragged_argument_errors(G):
    import torch
    desc = G.NetDesc(**TINY)
    net = G.Ga3c(desc, 4, 10)
    fr = torch.zeros(12, desc.in_c, desc.in_h, desc.in_w, dtype=torch.uint8, device="cuda")
    z = lambda n, dt: torch.zeros(n, dtype=dt, device="cuda")
    hp = G.HParams()
    with pytest.raises(G.Ga3cError):      # above capacity
        net.train_step_ragged(fr, z(12, torch.int32), z(12, torch.float32), z(12, torch.uint8),
                              torch.tensor([0, 12], dtype=torch.int32, device="cuda"), None, hp)
    with pytest.raises(G.Ga3cError):      # frames but no segment
        net.train_step_ragged(fr[:4], z(4, torch.int32), z(4, torch.float32), z(4, torch.uint8),
                              torch.tensor([0], dtype=torch.int32, device="cuda"), None, hp)
    with pytest.raises(G.Ga3cError):      # array sizes do not match
        net.train_step_ragged(fr[:4], z(3, torch.int32), z(4, torch.float32), z(4, torch.uint8),
                              torch.tensor([0, 4], dtype=torch.int32, device="cuda"), None, hp)
    # no frames: a no-op
    net.train_step_ragged(fr[:0], z(0, torch.int32), z(0, torch.float32), z(0, torch.uint8),
                          torch.tensor([0], dtype=torch.int32, device="cuda"), None, hp)
    torch.cuda.synchronize()
    net.close()


@pytest.mark.parametrize("math", [0, 1])
def test_handful_of_frames_in_one_launch(G, math):
    # up to 64 frames of the small net go out as one kernel (convolutions, fc, heads, draw; 32 blocks per frame up to
    # 8 frames, 16 up to 16, 8 up to 32, 4 up to 64); more frames take the three-kernel path.  Both compute the same
    # numbers up to summation order, call after call (the kernel's ticket counters must be back at zero after every
    # launch), in any order of batch sizes.
    import torch
    import dataclasses
    desc = dataclasses.replace(G.SMALL_NET(18), math=math)
    net = G.Ga3c(desc, 96, 0)
    net.use_generic_kernels(GENERIC)
    net.params_init(31)
    fr = torch.from_numpy(synth.rectangle_frames(8301, 96)).cuda()
    u = torch.from_numpy(synth.uniforms(8302, 96)).cuda()
    def run(B):
        lg = torch.empty(B, 18, device="cuda"); vl = torch.empty(B, device="cuda"); pr = torch.empty(B, 18, device="cuda")
        ac = torch.empty(B, dtype=torch.int32, device="cuda")
        net.predict(fr[:B].contiguous(), uniforms=u[:B].contiguous(), logits=lg, values=vl, probs=pr, actions=ac)
        torch.cuda.synchronize()
        return lg.cpu().numpy(), vl.cpu().numpy(), pr.cpu().numpy(), ac.cpu().numpy()
    ref = run(96)
    tol = 1e-5 if math == 0 else TOL_FWD_BF16
    first = {}
    for B in (3, 8, 1, 16, 5, 8, 9, 2, 7, 12, 4, 6, 16, 1, 3, 9, 17, 64, 32, 33, 40, 5, 64, 17, 31, 33, 63):
        print("frames", B, flush=True)
        lg, vl, pr, ac = run(B)
        assert rel_err(lg, ref[0][:B]) <= tol and rel_err(vl, ref[1][:B]) <= tol and rel_err(pr, ref[2][:B]) <= tol
        cdf = np.cumsum(pr.astype(np.float64), 1)
        clear = (np.abs(cdf - u[:B].cpu().numpy()[:, None]) > 1e-4).all(1)
        if math == 0:
            np.testing.assert_array_equal(ac[clear], ref[3][:B][clear])
        assert ((ac >= 0) & (ac < 18)).all()
        if B in first:            # the same call again: the same bits
            for x, y in zip((lg, vl, pr, ac), first[B]):
                np.testing.assert_array_equal(x, y)
        first[B] = (lg, vl, pr, ac)
    net.close()


@pytest.mark.parametrize("math", [0, 1])
@pytest.mark.parametrize("B", [17, 32, 33, 64])
def test_one_launch_prediction_17_to_64_frames_against_the_oracle(G, B, math):
    # the batch sizes that used to take three launches, element by element against the oracle
    import dataclasses
    check_predict(G, dataclasses.replace(G.SMALL_NET(18), math=math), B, 8400 + B, frames=synth.rectangle_frames(8400 + B, B))


def test_one_launch_prediction_is_stable_next_to_a_training_step(G):
    # The block that finishes a frame last reads what the other blocks of the launch wrote, with no device-wide fence
    # (see predict_small_kernel).  20 000 calls of 1 .. 64 frames while training steps run on a second stream: every
    # result must equal, bit for bit, the first result for that batch size.  Parameters are held fixed (lr = 0).
    import torch
    if GENERIC:
        pytest.skip("the general kernels have no one-launch path")
    net = G.Ga3c(G.SMALL_NET(18), 64, 640)
    net.params_init(41)
    fr = torch.from_numpy(synth.rectangle_frames(8501, 64)).cuda()
    u = torch.from_numpy(synth.uniforms(8502, 64)).cuda()
    tf = torch.from_numpy(synth.rectangle_frames_tiled(8503, 640).reshape(128, 5, 4, 84, 84)).cuda()
    tr = synth.trajectories(8504, 128, 5, 18)
    ta, trw, td = (torch.from_numpy(tr[k]).cuda() for k in ("actions", "rewards", "dones"))
    hp = G.HParams(lr=0.0)
    s_pred, s_train = torch.cuda.Stream(), torch.cuda.Stream()
    sizes = [1, 2, 5, 8, 9, 16, 17, 31, 32, 33, 48, 64]
    outs = {B: [torch.empty(B, 18, device="cuda"), torch.empty(B, device="cuda"), torch.empty(B, dtype=torch.int32, device="cuda")]
            for B in sizes}
    want = {}
    for B in sizes:
        net.predict(fr[:B], uniforms=u[:B], logits=outs[B][0], values=outs[B][1], actions=outs[B][2], stream=s_pred)
        s_pred.synchronize()
        want[B] = [t.clone() for t in outs[B]]
    rng = synth.rng(8505)
    order = rng.integers(0, len(sizes), 20000)
    bad = torch.zeros(1, dtype=torch.int32, device="cuda")
    for i, k in enumerate(order):
        B = sizes[int(k)]
        if i % 8 == 0:
            net.train_step(tf, ta, trw, td, None, hp, stream=s_train)
        net.predict(fr[:B], uniforms=u[:B], logits=outs[B][0], values=outs[B][1], actions=outs[B][2], stream=s_pred)
        with torch.cuda.stream(s_pred):
            for got, w in zip(outs[B], want[B]):
                bad += (got != w).any().to(torch.int32)
        if i % 2000 == 1999:
            torch.cuda.synchronize()
            print("calls", i + 1, "mismatches", int(bad.item()), flush=True)
            assert int(bad.item()) == 0
    torch.cuda.synchronize()
    assert int(bad.item()) == 0
    net.close()


def test_train_large_net(G):
    run_train(G, G.LARGE_NET(18), 5, 5, synth.BASE_SEED + 3, dict(clip_norm=40.0))


def test_a_large_update_keeps_the_larger_net_filter_fragments_current(G):
    # the larger net's conv2 / conv3 kernels read their filters as fragments that are rebuilt after every update; two
    # updates with a learning rate seven times the usual (larger ones saturate this net in one step): the second one's forward pass and input gradients (checked layer by layer
    # against that step's parameters) would show fragments left behind by the first
    ref = run_train(G, G.LARGE_NET(6), 4, 5, 4400, dict(lr=0.002), steps=2)
    assert ref["stats"]["grad_norm"] > 0


def test_train_degenerate_inputs(G):
    import torch
    net, onet, theta = make(G, G.SMALL_NET(6), 0, 10, 5)
    hp = G.HParams()
    z = lambda *s, dt=torch.float32: torch.zeros(s, dtype=dt, device="cuda")
    # N*T = 0 is a no-op; above capacity is refused; theta untouched in both cases
    net.train_step(z(0, 5, 4, 84, 84, dt=torch.uint8), z(0, 5, dt=torch.int32), z(0, 5), z(0, 5, dt=torch.uint8), None, hp)
    with pytest.raises(G.Ga3cError):
        net.train_step(z(3, 5, 4, 84, 84, dt=torch.uint8), z(3, 5, dt=torch.int32), z(3, 5), z(3, 5, dt=torch.uint8), None, hp)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(net.params_get(0).cpu().numpy(), theta)
    # one agent, one step, NULL bootstrap, terminal step
    frames = synth.uniform_frames(6, (1, 1, 4, 84, 84))
    a = np.array([[2]], np.int32); r = np.array([[1.0]], np.float32); d = np.array([[1]], np.uint8)
    net.train_step(torch.from_numpy(frames).cuda(), torch.from_numpy(a).cuda(), torch.from_numpy(r).cuda(),
                   torch.from_numpy(d).cuda(), None, hp)
    torch.cuda.synchronize()
    ref = orc.train_step(onet, theta, np.zeros_like(theta), frames, a, r, d, None, orc.HParams())
    assert rel_err(net.params_get(2).cpu().numpy(), ref["grad"]) <= TOL_BWD
    assert rel_err(net.params_get(0).cpu().numpy().astype(np.float64) - theta, ref["theta"] - theta) <= 2e-3
    net.close()


def test_predict_full_size_sweep_end(G):
    # largest batch of the prediction sweep (1024 frames, 18 actions, game-like frames), every frame checked
    frames = synth.rectangle_frames_tiled(synth.BASE_SEED + 1, 1024)
    check_predict(G, G.SMALL_NET(18), 1024, synth.BASE_SEED + 1, frames=frames)


@pytest.mark.parametrize("B", [255, 257, 513])
def test_predict_around_one_frame_per_compute_unit(G, B):
    # the fused convolution kernel gives every compute unit (256) a queue of frames: one short of a full round,
    # one over, and one over two rounds
    frames = synth.rectangle_frames_tiled(synth.BASE_SEED + 5, B)
    check_predict(G, G.SMALL_NET(18), B, synth.BASE_SEED + 5 + B, frames=frames)


def test_train_just_over_the_benchmark_size(G):
    # 513 agents x 5: the last blocks of every kernel carry a ragged tail
    N, T = 513, 5
    frames = synth.rectangle_frames_tiled(synth.BASE_SEED + 6, N * T).reshape(N, T, 4, 84, 84)
    run_train(G, G.SMALL_NET(18), N, T, synth.BASE_SEED + 6, dict(clip_norm=40.0), frames=frames, g0_scale=1e-3)


def test_train_full_size_512_agents(G):
    # largest training step of the sweep, in the configuration the benchmark times: 512 agents x 5, clip 40
    N, T = 512, 5
    frames = synth.rectangle_frames_tiled(synth.BASE_SEED + 2, N * T).reshape(N, T, 4, 84, 84)
    run_train(G, G.SMALL_NET(18), N, T, synth.BASE_SEED + 2, dict(clip_norm=40.0), frames=frames, g0_scale=1e-3)


def test_large_net_full_size(G):
    # larger CNN: predict 256, train 256 agents x 5
    frames = synth.rectangle_frames_tiled(synth.BASE_SEED + 3, 256)
    check_predict(G, G.LARGE_NET(18), 256, synth.BASE_SEED + 3, frames=frames)
    tf = synth.rectangle_frames_tiled(synth.BASE_SEED + 4, 1280).reshape(256, 5, 4, 84, 84)
    run_train(G, G.LARGE_NET(18), 256, 5, synth.BASE_SEED + 4, dict(clip_norm=40.0), frames=tf)


# ---- math = 1: operands of every contraction rounded to bfloat16 (the reduced-precision variant) ----

def bf16(desc):
    import dataclasses
    return dataclasses.replace(desc, math=1)


@pytest.mark.parametrize("which,B", [("small", 37), ("large", 9), ("odd", 11)])
def test_bf16_variant_predict(G, which, B):
    desc = {"small": G.SMALL_NET(18), "large": G.LARGE_NET(18), "odd": G.NetDesc(**ODD)}[which]
    frames = None if which == "odd" else synth.rectangle_frames(77, B)
    check_predict(G, bf16(desc), B, 7700 + B, frames=frames)


@pytest.mark.parametrize("which,N,T", [("small", 8, 5), ("small", 67, 5), ("large", 5, 5), ("odd", 11, 4), ("tiny3", 9, 3)])
def test_bf16_variant_train(G, which, N, T):
    desc = {"small": G.SMALL_NET(6), "large": G.LARGE_NET(18), "odd": G.NetDesc(**ODD), "tiny3": G.NetDesc(**TINY3)}[which]
    run_train(G, bf16(desc), N, T, 7800 + N, dict(clip_norm=40.0), g0_scale=1e-3, steps=2)


@pytest.mark.parametrize("A,F", [(21, 12), (40, 24), (63, 64)])
def test_bf16_variant_many_actions(G, A, F):
    shape = dict(TINY, fc_units=F, n_actions=A)
    check_predict(G, bf16(G.NetDesc(**shape)), 11, 8100 + A)
    run_train(G, bf16(G.NetDesc(**shape)), 7, 3, 8200 + A, dict(beta=0.05, value_coef=0.5, gamma=0.9), g0_scale=1e-2)


def test_bf16_variant_full_size_step(G):
    # the benchmark's training step with operands rounded to bfloat16
    N, T = 512, 5
    frames = synth.rectangle_frames_tiled(synth.BASE_SEED + 7, N * T).reshape(N, T, 4, 84, 84)
    run_train(G, bf16(G.SMALL_NET(18)), N, T, synth.BASE_SEED + 7, dict(clip_norm=40.0), frames=frames, g0_scale=1e-3)


def test_bf16_variant_differs_from_fp32(G):
    # the switch does something: the same parameters and frames give visibly different logits
    import torch
    desc = G.SMALL_NET(6)
    frames = synth.rectangle_frames(79, 16)
    outs = []
    for d in (desc, bf16(desc)):
        net, onet, theta = make(G, d, 16, 0, 7900)
        lg, _, _, _ = run_predict(G, net, frames)
        outs.append(lg)
        net.close()
    e = rel_err(outs[1], outs[0])
    assert 1e-5 < e < 3e-2


def test_params_init_statistics_and_determinism(G):
    import torch
    net = G.Ga3c(G.SMALL_NET(18), 1, 0)
    net.params_init(1234)
    t1 = net.params_get(0).cpu().numpy()
    net.params_init(1234)
    t2 = net.params_get(0).cpu().numpy()
    net.params_init(1235)
    t3 = net.params_get(0).cpu().numpy()
    torch.cuda.synchronize()
    np.testing.assert_array_equal(t1, t2)
    assert (t1 != t3).mean() > 0.9
    for name, (o, shape) in net.offsets().items():
        n = int(np.prod(shape)); x = t1[o:o + n]
        if name.endswith(".b"):
            assert (x == 0).all()
            continue
        std = np.sqrt(2.0 / np.prod(shape[1:]))
        assert abs(x.mean()) < 4 * std / np.sqrt(n), name
        assert abs(x.std() / std - 1) < 4 / np.sqrt(2 * n) + 1e-3, name
        if n > 10000:     # tails of a normal: P(|x| > 3 sigma) = 0.0027
            assert abs((np.abs(x) > 3 * std).mean() - 0.0027) < 0.001, name
    assert (net.params_get(1).cpu().numpy() == 0).all()
    net.close()


def test_rmsprop_flat(G):
    import torch
    n = 1_000_003
    r = synth.rng(321)
    th = r.standard_normal(n).astype(np.float32); g = np.abs(r.standard_normal(n)).astype(np.float32)
    d = r.standard_normal(n).astype(np.float32)
    tt, gt, dt = (torch.from_numpy(x).cuda() for x in (th, g, d))
    G.rmsprop_flat(tt, gt, dt, 0.5, 3e-4, 0.99, 0.1)
    torch.cuda.synchronize()
    t_ref, g_ref = orc.rmsprop(th, g, d, 0.5, 3e-4, 0.99, 0.1)
    assert rel_err(gt.cpu().numpy(), g_ref) <= 1e-6
    assert rel_err(tt.cpu().numpy().astype(np.float64) - th, t_ref - th) <= 1e-3


def test_stage_timer_changes_no_result_and_reports_every_stage(G):
    # While the stage timer is on, every kernel goes out through another launch call of the runtime (one that stamps
    # an event pair at the dispatch's own start and end): the numbers must be the same bit for bit, every stage of
    # the two calls must be reported with its call count, and a stage's time must be a kernel's, not a launch gap's.
    import torch
    desc = G.SMALL_NET(18)
    B, N, T = 64 + 5, 16, 5
    frames = synth.rectangle_frames(9901, N * T).reshape(N, T, 4, 84, 84)
    tr = synth.trajectories(9902, N, T, 18)
    pf = torch.from_numpy(synth.rectangle_frames(9903, B)).cuda()
    results = []
    for timed in (False, True):
        net, _, _ = make(G, desc, B, N * T, 9900)
        net.profile_enable(timed)
        lg = torch.empty(B, 18, device="cuda"); vl = torch.empty(B, device="cuda")
        net.predict(pf, logits=lg, values=vl)
        net.train_step(torch.from_numpy(frames).cuda(), torch.from_numpy(tr["actions"]).cuda(), torch.from_numpy(tr["rewards"]).cuda(),
                       torch.from_numpy(tr["dones"]).cuda(), torch.zeros(N, device="cuda"), G.HParams(clip_norm=40.0))
        torch.cuda.synchronize()
        if timed:
            st = net.profile_read()
            net.profile_enable(False)
            want = {"fc_fwd": 2, "wgrad_reduce": 1, "rmsprop": 1, "fc_dgrad": 1}
            want.update({"conv1_fwd": 2, "conv2_fwd": 2, "conv1_wgrad": 1, "conv2_wgrad": 1, "conv2_dgrad": 1} if GENERIC
                        else {"conv12_fwd": 2, "heads_fwd": 1, "heads_train": 1, "conv1_wgrad": 1, "conv2_wgrad": 1, "conv2_dgrad": 1})
            for name, calls in want.items():
                assert name in st and st[name]["calls"] == calls, (name, st.get(name))
                assert 0.0005 < st[name]["ms"] / calls < 5.0, (name, st[name])      # between half a microsecond and 5 ms
        results.append((lg.cpu().numpy(), vl.cpu().numpy(), net.params_get(0).cpu().numpy(), net.params_get(2).cpu().numpy()))
        net.close()
    for a, b in zip(*results):
        np.testing.assert_array_equal(a, b)
