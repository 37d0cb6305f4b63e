"""ga3c_predict_static (prediction without device allocation) against ga3c_predict, through the C ABI.

Both run the same kernels on the same parameters, so the outputs must be equal bit for bit; ga3c_predict itself is
compared with the oracle in tests/test_gpu_parity.py, and once more here.  Two calls in a row share the library's
scratch array, the second with a smaller batch: stale contents of the first must not leak into it.
"""
import numpy as np
import pytest

import ga3c_synth as synth
import oracle as orc

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("math", [0, 1])
def test_predict_static_equals_predict_on_two_calls_in_a_row(math):
    import dataclasses
    import torch
    import paper_1611_06256_amd as G
    A = 18
    desc = dataclasses.replace(G.SMALL_NET(A), math=math)
    net = G.Ga3c(desc, G.STATIC_MAX_FRAMES, 0)
    theta = synth.perturbed_theta(4100 + math, net.offsets(), net.n_params)
    th_t = torch.from_numpy(theta).cuda()
    net.params_set(th_t, 0)
    onet = orc.Net(n_actions=A, math=math)

    def outputs(B):
        return dict(logits=torch.full((B, A), float("nan"), device="cuda"), values=torch.full((B,), float("nan"), device="cuda"),
                    probs=torch.full((B, A), float("nan"), device="cuda"),
                    actions=torch.full((B,), -1, dtype=torch.int32, device="cuda"))

    # 200 frames (three launches), then 37 (fewer frames in the same scratch), then 5 and 16 (one launch: tickets), then 256
    for i, B in enumerate([200, 37, 5, 16, G.STATIC_MAX_FRAMES, 1]):
        frames = synth.rectangle_frames(4200 + i, B)
        fr = torch.from_numpy(frames).cuda()
        u = torch.from_numpy(synth.uniforms(4300 + i, B)).cuda()
        want, got = outputs(B), outputs(B)
        print(f"predict_static math={math} B={B}", flush=True)
        net.predict(fr, uniforms=u, **want)
        G.predict_static(A, math, th_t, fr, uniforms=u, **got)
        torch.cuda.synchronize()
        for k in want:
            np.testing.assert_array_equal(got[k].cpu().numpy(), want[k].cpu().numpy(), err_msg=f"{k} B={B}")
        ref = orc.forward(onet, theta, frames)
        tol = 1e-4 if math == 0 else 2.0 ** -6
        lg = got["logits"].cpu().numpy()
        assert np.abs(lg - ref["logits"]).max() <= tol * np.abs(ref["logits"]).max()
    # subset of outputs, empty batch, errors
    vals = torch.zeros(3, device="cuda")
    G.predict_static(A, math, th_t, fr[:1].expand(3, -1, -1, -1).contiguous(), values=vals)
    G.predict_static(A, math, th_t, torch.empty((0, 4, 84, 84), dtype=torch.uint8, device="cuda"))
    torch.cuda.synchronize()
    assert torch.all(vals == got["values"][0])
    with pytest.raises(G.Ga3cError, match="outside"):
        G.predict_static(A, math, th_t, torch.zeros((G.STATIC_MAX_FRAMES + 1, 4, 84, 84), dtype=torch.uint8, device="cuda"))
    with pytest.raises(G.Ga3cError):
        G.predict_static(0, math, th_t, fr)
    with pytest.raises(G.Ga3cError):
        G.predict_static(A, math, th_t, fr, actions=torch.zeros(1, dtype=torch.int32, device="cuda"))
    net.close()
