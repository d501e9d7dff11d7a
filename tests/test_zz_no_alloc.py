"""sasgd_applyUpdateNoAlloc (the server update for callers that cannot allocate) against sasgd_applyUpdate.

The same inputs go through a context (pushGradientExternal / sumGradients / applyUpdate) and through the context-free
entry point; both run the same kernels, so theta, v and the bf16 copy must come out bit-identical.  Two calls in a row
share the library's static buffer of partial sums: a long window over a vector of several stretches with a ragged tail,
then a smaller one.
"""
import numpy as np
import pytest

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu


def _case(P, c, seed, lr_mode, momentum, wd, alpha0=0.01, warm=3):
    from paper_1511_05950_amd import binding
    rng = np.random.default_rng(seed)
    theta0 = torch.from_numpy((rng.standard_normal(P) * 0.01).astype(np.float32)).cuda()
    grads = [torch.from_numpy((rng.standard_normal(P) * 1e-3).astype(np.float32)).cuda() for _ in range(c)]
    ctx = binding.Sasgd(c, 0, 1, 1, net=None, num_params=P, lr_mode=lr_mode, alpha0=alpha0, momentum=momentum, weight_decay=wd,
                        init_weights=theta0)
    for _ in range(warm):                                  # move the timestamp and fill the momentum
        i = ctx.timestamp()
        for l in range(c):
            ctx.pushGradientExternal(grads[(l + 1) % c], i)
        ctx.sumGradients()
        ctx.applyUpdate()
    i = ctx.timestamp()
    th_in = torch.from_numpy(ctx.copyWeights()).cuda()
    v_in = torch.from_numpy(ctx.copyMomentum()).cuda()
    taus = [int(t) for t in rng.integers(0, i + 1, size=c)]
    for l in range(c):
        assert ctx.pushGradientExternal(grads[l], i - taus[l]) == taus[l]
    ctx.sumGradients()
    ctx.applyUpdate()
    th_ref, v_ref = ctx.copyWeights(), ctx.copyMomentum()
    ctx.destroy()
    return th_in, v_in, grads, taus, th_ref, v_ref


def _bf16_rne(a):
    u = a.view(np.uint32).astype(np.uint64)
    u = (u + 0x7FFF + ((u >> 16) & 1)) >> 16
    return u.astype(np.uint16)


def test_no_alloc_update_matches_context_update_twice_in_a_row():
    from paper_1511_05950_amd import binding
    # (P, c): first the two-launch form over 2 full stretches + a ragged one + a scalar tail, then a smaller vector
    # (one stretch and a bit) with another window length, then a short window that takes the single launch
    for (P, c, mode) in [(2 * (1 << 21) + 300_001, 30, "per_gradient"), ((1 << 21) + 4_099, 26, "mean_staleness"),
                         (70_001, 3, "per_gradient")]:
        print("case P=%d c=%d %s" % (P, c, mode), flush=True)
        th_in, v_in, grads, taus, th_ref, v_ref = _case(P, c, seed=P % 1000 + c, lr_mode=mode, momentum=0.9, wd=5e-4)
        th_out = torch.empty_like(th_in)
        shadow = torch.zeros(P, dtype=torch.int16, device="cuda")
        v = v_in.clone()
        torch.cuda.synchronize()
        free_before = torch.cuda.mem_get_info()[0]          # the driver's figure: it moves only when somebody calls hipMalloc / hipFree
        binding.applyUpdateNoAlloc(th_in, th_out, v, grads, taus, lr_mode=mode, alpha0=0.01, momentum=0.9, weight_decay=5e-4,
                                   shadow_out_dev=shadow)
        torch.cuda.synchronize()
        assert torch.cuda.mem_get_info()[0] == free_before
        got_th, got_v = th_out.cpu().numpy(), v.cpu().numpy()
        assert np.array_equal(got_th.view(np.uint32), th_ref.view(np.uint32))
        assert np.array_equal(got_v.view(np.uint32), v_ref.view(np.uint32))
        assert np.array_equal(shadow.cpu().numpy().view(np.uint16), _bf16_rne(th_ref))
        # in place, as the context does it
        th2, v2 = th_in.clone(), v_in.clone()
        binding.applyUpdateNoAlloc(th2, th2, v2, grads, taus, lr_mode=mode, alpha0=0.01, momentum=0.9, weight_decay=5e-4)
        torch.cuda.synchronize()
        assert np.array_equal(th2.cpu().numpy().view(np.uint32), th_ref.view(np.uint32))
        assert np.array_equal(v2.cpu().numpy().view(np.uint32), v_ref.view(np.uint32))


def test_no_alloc_update_refuses_sizes_beyond_its_limits():
    from paper_1511_05950_amd import binding
    th = torch.zeros(64, device="cuda")
    g = torch.zeros(64, device="cuda")
    with pytest.raises(binding.SasgdError) as e:
        binding.applyUpdateNoAlloc(th, th, th.clone(), [g] * 65, [0] * 65)
    assert e.value.code == binding.EINVAL and "1..64" in str(e.value)
    with pytest.raises(binding.SasgdError) as e:
        binding.applyUpdateNoAlloc(th, th, th.clone(), [g], [0], num_params=(1 << 32) + 1)
    assert e.value.code == binding.EINVAL and "num_params" in str(e.value)
    with pytest.raises(binding.SasgdError) as e:
        binding.applyUpdateNoAlloc(th, th, th.clone(), [g], [-1])
    assert e.value.code == binding.EINVAL
    with pytest.raises(binding.SasgdError) as e:
        binding.applyUpdateNoAlloc(th, th, th.clone(), [], [])
    assert e.value.code == binding.EINVAL
