"""The entry point that allocates nothing, pier_inner_adamw_clipped_static, against the entry
point it is a variant of, pier_inner_adamw_clipped: same inputs, through the C ABI, two calls
in a row on the GPU's one static scratch array, the second with a smaller model; bit for bit
(theta, m, v, bf16 working copy, norm, coefficient), and both within the parity bar of the
oracle's clipped step.  (Named to be collected after every other test file.)"""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

HP = dict(lr=3e-4, beta1=0.9, beta2=0.95, eps=1e-8, weight_decay=0.1)


def _state(numels, seed, bf16):
    """One replica's buffers (theta, m, v, grad, bf16 working copy) with seeded contents."""
    rng = np.random.default_rng(seed)
    gdt = torch.bfloat16 if bf16 else torch.float32
    out = []
    for n in numels:
        p = torch.from_numpy(rng.normal(0, 0.02, n).astype(np.float32)).cuda()
        m = torch.from_numpy(rng.normal(0, 1e-3, n).astype(np.float32)).cuda()
        v = torch.from_numpy(rng.uniform(0, 1e-6, n).astype(np.float32)).cuda()
        g = torch.from_numpy(rng.normal(0, 1e-3, n).astype(np.float32)).cuda().to(gdt)
        w = torch.zeros(n, dtype=torch.bfloat16, device="cuda")
        out.append((p, m, v, g, w))
    return [list(col) for col in zip(*out)] if out else [[], [], [], [], []]


def _ctx(numels, cols, bf16, fold=None):
    import paper_2511_17849_amd as pier
    ctx = pier.pier_ctx_create(numels, 1)
    if fold is not None:
        pier.pier_ctx_set_norm_fold(ctx, fold)
    P, M, V, G, W = cols
    pier.pier_bind_replica(ctx, 0, P, M, V, G, bf16)
    pier.pier_bind_shadow(ctx, 0, W)
    return ctx


def _bits(t):
    t = t.detach().cpu()
    return t.view(torch.int16).numpy() if t.dtype == torch.bfloat16 else t.numpy().view(np.uint32)


def _compare(numels, seed, bf16, max_norm, step, stream):
    """Runs both entry points on twin states; returns the static call's (norm, coef)."""
    import paper_2511_17849_amd as pier
    from oracle import pier_oracle as O
    print("[no-alloc] case numels=%s seed=%d bf16=%d max_norm=%g" % (numels, seed, bf16, max_norm), flush=True)
    a, b = _state(numels, seed, bf16), _state(numels, seed, bf16)
    ca, cb = _ctx(numels, a, bf16), _ctx(numels, b, bf16)
    # oracle's clipped step on a host copy of the same inputs
    host = [[t.cpu() for t in col] for col in a]
    torch.cuda.synchronize()
    pier.pier_inner_adamw_clipped_static(ca, 0, step=step, max_norm=max_norm, stream=stream, **HP)
    got = pier.pier_grad_norm_last(ca, 0, stream=stream)
    pier.pier_inner_adamw_clipped(cb, 0, step=step, max_norm=max_norm, stream=stream, **HP)
    ref = pier.pier_grad_norm_last(cb, 0, stream=stream)
    torch.cuda.synchronize()
    assert got == ref, (got, ref)
    for k in range(5):
        if k == 3:
            continue                                       # gradients are inputs
        for x, y in zip(a[k], b[k]):
            assert np.array_equal(_bits(x), _bits(y)), "buffer kind %d differs" % k
    # and against the oracle: sum of squares over the tensor list in order, then the step
    ss = 0.0
    for g in host[3]:
        gg = g.view(torch.int16).numpy().view(np.uint16) if bf16 else g.numpy()
        ss = O.sumsq(np.ascontiguousarray(gg), ss)
    coef = O.clip_coef(ss, max_norm)
    assert abs(got[0] - np.sqrt(ss)) <= 1e-11 * np.sqrt(ss) and abs(got[1] - coef) <= 6e-8 * coef
    for i, n in enumerate(numels):
        if n == 0:
            continue
        p, m, v = (host[k][i].numpy().copy() for k in range(3))
        g = host[3][i]
        g = np.ascontiguousarray(g.view(torch.int16).numpy().view(np.uint16)) if bf16 else g.numpy()
        O.adamw(p, m, v, g, step=step, grad_scale=coef, **HP)         # the oracle's own coefficient
        for name, want, have in (("theta", p, a[0][i]), ("m", m, a[1][i]), ("v", v, a[2][i])):
            have = have.cpu().numpy()
            assert np.all(np.abs(have.astype(np.float64) - want) <= 1e-6 * np.maximum(1.0, np.abs(want))), name
            if np.float32(got[1]) == np.float32(coef):                # same fp32 coefficient: same bits
                assert np.array_equal(have, want), name
        if np.float32(got[1]) == np.float32(coef):
            assert np.array_equal(O.to_bf16(p), a[4][i].cpu().view(torch.int16).numpy().view(np.uint16))
    return got


def test_static_scratch_entry_point_matches_the_allocating_one_twice_in_a_row():
    import paper_2511_17849_amd as pier
    stream = torch.cuda.Stream()
    # The call allocates and frees nothing: the device's free memory is the same before and after.
    # (First launches of a process load code, and the runtime may grow one of its own pools at any
    # launch, so a few calls are taken and one with no change at all is asked for.)
    warm = _state([70_000], 70, False)
    wc = _ctx([70_000], warm, False)
    pier.pier_inner_adamw_clipped_static(wc, 0, step=1, max_norm=1.0, stream=stream, **HP)
    pier.pier_inner_adamw_clipped(wc, 0, step=2, max_norm=1.0, stream=stream, **HP)
    torch.cuda.synchronize()
    deltas = []
    for k in range(4):
        before = torch.cuda.mem_get_info()[0]
        pier.pier_inner_adamw_clipped_static(wc, 0, step=3 + k, max_norm=1.0, stream=stream, **HP)
        torch.cuda.synchronize()
        deltas.append(torch.cuda.mem_get_info()[0] - before)
    assert 0 in deltas, deltas
    big = [300_000, 1025, 7, 0, 4096 * 5, 3]               # 318 chunks' worth of partial sums
    small = [5000, 3, 1024]                                # fewer partial sums than the call before left behind
    n1 = _compare(big, 71, False, 0.05, 3, stream)
    n2 = _compare(small, 72, True, 0.01, 9, stream)
    assert n1[1] < 1.0 and n2[1] < 1.0 and n1 != n2         # clipping active both times
    n3 = _compare(big, 73, False, 5.0, 4, stream)          # larger again, threshold above the norm
    assert n3[1] == 1.0
    _compare([0, 0], 74, False, 1.0, 1, stream)            # empty model: norm 0, coefficient 1, no launch over data


def test_static_scratch_entry_point_rejects_what_the_array_cannot_hold():
    import paper_2511_17849_amd as pier
    numels = [1024 * 20_000]                               # 20 000 chunks
    cols = _state(numels, 75, False)
    before = [_bits(col[0]).copy() for col in cols[:3]]
    ok = _ctx(numels, cols, False)                         # default fold: 16 384 partial sums, fits
    pier.pier_inner_adamw_clipped_static(ok, 0, step=1, max_norm=1.0, **HP)
    torch.cuda.synchronize()
    assert not np.array_equal(_bits(cols[0][0]), before[0])
    before = [_bits(col[0]).copy() for col in cols[:3]]
    wide = _ctx(numels, cols, False, fold=20_000)          # 20 000 partial sums: 160 256 bytes > 131 328
    with pytest.raises(pier.PierError, match="PIER_ERR_INVALID_ARG") as e:
        pier.pier_inner_adamw_clipped_static(wide, 0, step=2, max_norm=1.0, **HP)
    assert "static scratch holds" in str(e.value)
    torch.cuda.synchronize()
    for col, b in zip(cols[:3], before):
        assert np.array_equal(_bits(col[0]), b)            # nothing was launched
    pier.pier_inner_adamw_clipped(wide, 0, step=2, max_norm=1.0, **HP)    # the allocating entry point takes it
    torch.cuda.synchronize()
    with pytest.raises(pier.PierError, match="PIER_ERR_INVALID_ARG"):
        pier.pier_ctx_set_norm_fold(pier.pier_ctx_create([4], 1), (1 << 20) + 1)
    with pytest.raises(pier.PierError, match="PIER_ERR_STATE"):
        pier.pier_ctx_set_norm_fold(ok, 64)                # after the first bind
