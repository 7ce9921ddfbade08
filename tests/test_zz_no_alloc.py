"""The entry point that allocates nothing (gae_compute_static) against gae_compute on a buffer binding of the same
arrays: identical kernels, so identical bits.  Two calls in a row on one device, the second on a smaller input (the
entry point's fixed partial-sum array keeps the first call's contents)."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu


def _case(g, inst, T, N, ld, normalize, seed):
    from paper_2206_08482_amd.runner import RolloutBuffers
    rng = np.random.default_rng(seed)
    dev = torch.device("cuda:0")
    rb = RolloutBuffers(T, ld, 3, 2, dev)
    rb.rew.copy_(torch.tensor(rng.standard_normal((T, ld)).astype(np.float32)))
    rb.val.copy_(torch.tensor(rng.standard_normal((T, ld)).astype(np.float32)))
    rb.done.copy_(torch.tensor((rng.random((T, ld)) < 0.1).astype(np.uint8)))
    last = torch.tensor(rng.standard_normal(N).astype(np.float32), device=dev)
    adv2 = torch.full((T, ld), 7.0, device=dev)
    ret2 = torch.full((T, ld), 7.0, device=dev)
    torch.cuda.synchronize()
    hb = g.gmi_buffer_bind(inst, rb.desc(0, N))
    g.gae_compute(inst, hb, last, 0.99, 0.95, normalize)
    g.gae_compute_static(inst, T, N, ld, rb.rew, rb.val, rb.done, last, 0.99, 0.95, normalize, adv2, ret2)
    g.gmi_sync(inst)
    a1, r1 = rb.adv.cpu().numpy(), rb.ret.cpu().numpy()
    a2, r2 = adv2.cpu().numpy(), ret2.cpu().numpy()
    assert np.array_equal(a1[:, :N], a2[:, :N]) and np.array_equal(r1[:, :N], r2[:, :N])
    assert np.isfinite(a2[:, :N]).all()
    assert (a2[:, N:] == 7.0).all() and (r2[:, N:] == 7.0).all()          # columns past N are not touched
    # and against the oracle, to the bar of the existing entry point's own test
    from oracle import ppo as oppo
    o_adv, o_ret = oppo.gae(rb.rew.cpu().numpy()[:, :N], rb.val.cpu().numpy()[:, :N], rb.done.cpu().numpy()[:, :N],
                            last.cpu().numpy(), 0.99, 0.95, normalize)
    assert np.linalg.norm(a2[:, :N] - o_adv) <= 1e-5 * np.linalg.norm(o_adv)
    assert np.linalg.norm(r2[:, :N] - o_ret) <= 1e-5 * np.linalg.norm(o_ret)
    g.gmi_buffer_destroy(hb)


def test_gae_compute_static_equals_gae_compute_twice_in_a_row():
    import paper_2206_08482_amd as g
    inst = g.gmi_create()
    _case(g, inst, 16, 5000, 5120, True, 0)       # 20 workgroups' partials
    _case(g, inst, 7, 300, 300, True, 1)          # smaller: 2 workgroups' partials, the rest keeps the first call's
    _case(g, inst, 3, 77, 80, False, 2)
    # sizes beyond the fixed array are refused before anything runs
    with pytest.raises(g.GmiError):
        g.gae_compute_static(inst, 1, 256 * 16384 + 1, 256 * 16384 + 1, None, None, None, None, 0.99, 0.95, True,
                             None, None)
    g.gae_compute_static(inst, 0, 0, 0, None, None, None, None, 0.99, 0.95, True, None, None)     # empty: nothing to do
    g.gmi_destroy(inst)
