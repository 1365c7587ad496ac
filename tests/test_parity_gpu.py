"""GPU parity: the HIP library, called through its C ABI (ctypes binding), against the
CPU oracle on identical seeded inputs.  Bar: |err| <= 1e-6 * max(1, |x|) per fp32
element for every buffer (theta_g, m_g, v_g, anchor, M), plus a relative 1e-5 bar on
the small-magnitude state.  Small cases compare every element; the full-size
configurations compare a deterministic sample of element indices."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

WARMUP, PIER = 0, 1
RAGGED = [1, 3, 5, 1023, 1025, 4096 + 7, 0, 70001, 16384, 16388, 2]


def _harness():
    import pier_harness
    return pier_harness


def _log(msg):
    print("[pier-parity] " + msg, flush=True)


# ------------------------------------------------------------------ config 1

def test_config1_tiny_every_element():
    H_ = _harness()
    from pier_inputs import shapes
    w = shapes.workloads()["tiny"]
    _log("config 1: N=%d G=%d H=%d" % (w.N, w.G, w.H))
    r = H_.Run(w.numels, w.G, seed=w.seed)
    r.inner_steps(w.H)
    rep = r.check("after inner")
    lr, mu = w.fixed_outer
    r.outer(mu=mu, lr=lr, phase=PIER)
    rep = r.check("after outer")
    _log("config 1: %s" % rep)
    # every replica holds the new anchor
    st = r.device_state()
    for g in range(w.G):
        assert np.array_equal(st["P%d" % g], st["A"])
    assert np.abs(st["Mo"]).max() > 1e-5      # something actually happened


# ------------------------------------------------------------------ ragged shapes, edge cases

@pytest.mark.parametrize("G", [1, 2, 3, 4, 5, 8])
@pytest.mark.parametrize("pad", [0, 1])
def test_ragged_tensor_list_all_elements(G, pad):
    """Odd sizes, an empty tensor, tensors that start off a 16-byte boundary (pad=1),
    group counts with and without a specialised kernel; two rounds: lazy start then Pier."""
    H_ = _harness()
    _log("ragged G=%d pad=%d" % (G, pad))
    r = H_.Run(RAGGED, G, pad=pad, seed=3, launch=dict(chunk_elems=4096))
    r.inner_steps(3, shared_stream=True)
    r.outer(mu=0.9, lr=0.0, phase=WARMUP)
    r.check("warmup round")
    st = r.device_state()
    for g in range(G):
        # the anchor IS the model, bit for bit, for every group count; replicas untouched
        assert np.array_equal(st["P%d" % g].view(np.uint32), st["A"].view(np.uint32))
    r.inner_steps(3)
    r.outer(mu=0.99, lr=0.4, phase=PIER)
    rep = r.check("pier round")
    _log("ragged G=%d pad=%d: %s" % (G, pad, rep))


@pytest.mark.parametrize("launch", [
    dict(chunk_elems=1024, unroll=1), dict(chunk_elems=1024, unroll=4),
    dict(chunk_elems=2048, unroll=2, nontemporal=0), dict(chunk_elems=65536, unroll=4, max_grid=3),
    dict(chunk_elems=16384, unroll=2, max_grid=7, nontemporal=0),
    dict(wg_threads=256, lds_bytes=0), dict(wg_threads=64, lds_bytes=0), dict(wg_threads=64, lds_bytes=65536),
    dict(wg_threads=256, lds_bytes=40960, unroll=2), dict(chunk_elems=4096, max_grid=5, wg_threads=64, lds_bytes=13312),
])
def test_result_does_not_depend_on_launch_shape(launch):
    H_ = _harness()
    _log("launch shape %s" % launch)
    outs = []
    for L in (launch, None):
        r = H_.Run(RAGGED + [300_000], 4, seed=5, launch=L)
        r.inner_steps(2)
        r.outer(mu=0.95, lr=0.8, phase=PIER)
        r.inner_steps(1)
        if L is launch:
            r.check(str(launch))
        outs.append(r.device_state())
    for k in outs[0]:
        assert np.array_equal(outs[0][k], outs[1][k]), k


def test_bf16_gradients():
    H_ = _harness()
    _log("bf16 grads")
    r = H_.Run(RAGGED + [200_000], 2, grad_bf16=True, seed=7)
    r.inner_steps(4)
    r.outer(mu=0.9, lr=1.1, phase=PIER)
    rep = r.check("bf16")
    _log("bf16: %s" % rep)
    r2 = H_.Run(RAGGED, 2, grad_bf16=True, seed=7, pad=1)      # 2-byte aligned gradient tensors
    r2.inner_steps(2)
    r2.check("bf16 misaligned")


def test_grad_scale_and_other_hyperparameters():
    H_ = _harness()
    _log("grad_scale / Table I betas")
    hp = dict(lr=1.5e-4, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.1, grad_scale=0.37)
    r = H_.Run([50_000, 77], 1, hp=hp, seed=11)
    r.inner_steps(5)
    r.outer(mu=0.0, lr=1.0, phase=PIER)
    r.check("grad_scale")
    # late in training the bias corrections are exactly 1 (beta^t underflows against 1)
    r.t = 999_999
    r.inner_steps(2)
    rep = r.check("step one million")
    assert rep["bit_exact"], rep


@pytest.mark.parametrize("case", range(64))
def test_randomised_small_cases(case):
    """Seeded random tensor lists (odd sizes, empty tensors, sizes around chunk multiples), group
    counts 1..16, launch shapes, gradient dtype, padding, phase sequence and scalars."""
    H_ = _harness()
    rng = np.random.default_rng(1000 + case)
    nt = int(rng.integers(1, 12))
    pool = [0, 1, 2, 3, 4, 5, 255, 256, 1023, 1024, 1025, 4095, 4096, 4100, 12289, 65536 + 3]
    numels = [int(rng.choice(pool)) if rng.random() < 0.7 else int(rng.integers(1, 200_000)) for _ in range(nt)]
    if sum(numels) == 0:
        numels.append(17)
    G = int(rng.choice([1, 2, 3, 4, 6, 7, 8, 9, 16]))
    launch = dict(chunk_elems=int(rng.choice([1024, 2048, 4096, 16384])), unroll=int(rng.choice([1, 2, 4])),
                  max_grid=int(rng.choice([0, 0, 5, 64])), nontemporal=int(rng.choice([0, 1])),
                  wg_threads=int(rng.choice([0, 64, 256])), lds_bytes=int(rng.choice([-1, 0, 13312])))
    bf16 = bool(rng.integers(0, 2))
    pad = int(rng.integers(0, 2))
    shadow = bool(rng.integers(0, 2))
    hp = dict(lr=float(rng.choice([1e-4, 3e-4, 1e-3])), beta1=0.9, beta2=float(rng.choice([0.95, 0.999])),
              eps=1e-8, weight_decay=float(rng.choice([0.0, 0.1])))
    _log("random case %d: numels=%s G=%d launch=%s bf16=%d pad=%d shadow=%d" % (case, numels, G, launch, bf16, pad, shadow))
    r = H_.Run(numels, G, grad_bf16=bf16, hp=hp, pad=pad, launch=launch, seed=case, shadow=shadow)
    for _ in range(int(rng.integers(1, 4))):
        phase = int(rng.integers(0, 2))
        r.inner_steps(int(rng.integers(1, 4)), shared_stream=(phase == WARMUP),
                      clip=float(rng.choice([0.02, 0.5])) if rng.random() < 0.5 else None)
        r.outer(mu=float(rng.choice([0.0, 0.9, 0.95, 0.99])), lr=float(rng.choice([0.25, 0.7, 1.0, 1.1])), phase=phase)
        rep = r.check("random case %d" % case)
    assert rep["bit_exact"]


# ------------------------------------------------------------------ bf16 working weights

@pytest.mark.parametrize("G,pad", [(1, 0), (2, 1), (3, 0), (8, 0)])
def test_bf16_working_copies(G, pad):
    """The bfloat16 copy of theta written by the AdamW step and by the Pier outer step
    (not by the lazy-start step), bit for bit; odd sizes and 2-byte aligned tensors too."""
    H_ = _harness()
    _log("bf16 working copies G=%d pad=%d" % (G, pad))
    r = H_.Run(RAGGED + [150_000], G, pad=pad, seed=29, shadow=True)
    r.inner_steps(2, shared_stream=True)
    r.outer(mu=0.9, lr=0.0, phase=WARMUP)
    r.check("shadow warmup")                       # working copies still those of the last inner step
    r.inner_steps(2, clip=0.05)
    r.outer(mu=0.95, lr=0.8, phase=PIER)
    rep = r.check("shadow pier")
    st = r.device_state()
    for g in range(1, G):
        assert np.array_equal(st["W0"], st["W%d" % g])
    assert np.abs((st["W0"].astype(np.uint32) << 16).view(np.float32) - st["P0"]).max() <= 2.0 ** -8 * np.abs(st["P0"]).max()
    _log("bf16 working copies: %s" % rep)


def test_bf16_working_copies_offload_and_partial_binding():
    import paper_2511_17849_amd as pier
    H_ = _harness()
    numels = [70_000, 1024, 4, 0, 300_000]
    res = H_.Run(numels, 2, seed=31, shadow=True)
    off = H_.Run(numels, 2, seed=31, shadow=True, offload=True, chunk_bytes=262144)
    for r in (res, off):
        r.inner_steps(2)
        r.outer(mu=0.9, lr=1.1, phase=PIER)
    off.check("shadow offload")
    a, b = res.device_state(), off.device_state()
    for k in a:
        assert np.array_equal(a[k], b[k]), k
    pier.pier_bind_shadow(res.ctx, 1, None)        # one replica without a working copy
    with pytest.raises(pier.PierError, match="PIER_ERR_STATE"):
        pier.pier_outer_step(res.ctx, outer_lr=0.7, mu=0.9, phase=PIER)
    pier.pier_bind_shadow(res.ctx, 0, None)        # none: plain path again
    before = res.device_state()
    old_w, res.W, res.oW = res.W, None, None
    res.inner_steps(1)
    res.outer(mu=0.9, lr=0.7, phase=PIER)
    res.check("shadow unbound")
    assert np.array_equal(before["W0"], res._take(old_w[0].flat))      # no longer written


# ------------------------------------------------------------------ whole schedule

@pytest.mark.parametrize("diloco,offload", [(False, False), (True, False), (False, True)])
def test_train_step_runs_the_whole_schedule(diloco, offload):
    """T = 40 iterations, r = 4: lazy start (t <= 4), mu 0.99 (t = 4 is lazy; 8 would be 0.9 ...) -
    every phase of the schedule through pier_train_step, with clipping, cosine inner learning
    rate and bf16 working copies, against the oracle's step-by-step mirror."""
    H_ = _harness()
    _log("train_step diloco=%d offload=%d" % (diloco, offload))
    numels = [4096, 1000, 36, 0, 70_000] if offload else RAGGED + [50_000]
    r = H_.Run(numels, 2, seed=37, shadow=True, offload=offload, chunk_bytes=65536 if offload else None)
    T = 40
    r.train_steps(T, T=T, r=4, diloco=diloco, lr_max=3e-4, lr_min=3e-5, warmup_frac=0.1, clip=0.1)
    rep = r.check("train_step")
    phases = [(t, ph, mu) for t, ph, mu, _ in r.sync_log]
    if diloco:
        assert all(ph == PIER and mu == 0.9 and lr == 0.7 for _, ph, mu, lr in r.sync_log)
    else:
        assert phases[:5] == [(4, WARMUP, 0.9), (8, PIER, 0.9), (12, PIER, 0.9), (16, PIER, 0.9), (20, PIER, 0.9)]
        assert [lr for *_, lr in r.sync_log][1:4] == pytest.approx([1.1, 1.1, 1.1])
        assert r.sync_log[-1][3] == pytest.approx(0.9)          # last 20 %
    _log("train_step: %s" % rep)


def test_train_step_mu_bands():
    """T = 400, r = 10: synchronisations at t = 40 (lazy start), 50 (mu 0.99, lr 0.25), 60 (0.95, 0.5),
    70 (0.95, 0.75), 80 (0.9, 1.1): the momentum-decay bands and the outer-lr ramp."""
    H_ = _harness()
    r = H_.Run([5000, 24, 3], 2, seed=41)
    r.train_steps(80, T=400, r=10, lr_max=4e-4, lr_min=4e-5)
    r.check("mu bands")
    got = [(t, ph, mu, round(lr, 4)) for t, ph, mu, lr in r.sync_log]
    assert got == [(10, WARMUP, 0.9, 0.0), (20, WARMUP, 0.9, 0.0), (30, WARMUP, 0.9, 0.0), (40, WARMUP, 0.9, 0.0),
                   (50, PIER, 0.99, 0.25), (60, PIER, 0.95, 0.5), (70, PIER, 0.95, 0.75), (80, PIER, 0.9, 1.1)]


# ------------------------------------------------------------------ gradient clipping

def _check_clip_log(r, expect_active):
    assert r.clip_log
    for norm_o, coef_o, norm_d, coef_d in r.clip_log:
        assert abs(norm_d - norm_o) <= 1e-11 * norm_o            # double sums, different fold order
        assert abs(coef_d - coef_o) <= 6e-8 * coef_o              # equal up to the last fp32 bit
        assert (coef_o < 1.0) == expect_active


@pytest.mark.parametrize("pad,bf16", [(0, False), (1, False), (0, True), (1, True)])
def test_clipped_adamw_all_elements(pad, bf16):
    """Global-norm clipping in front of the AdamW step: norm, coefficient and the step."""
    H_ = _harness()
    _log("clipped adamw pad=%d bf16=%d" % (pad, bf16))
    r = H_.Run(RAGGED + [300_000], 2, pad=pad, grad_bf16=bf16, seed=23)
    r.inner_steps(3, clip=0.1)                     # norm ~ 0.64: clipping active
    _check_clip_log(r, True)
    rep = r.check("clip active")
    r.inner_steps(2, clip=5.0)                     # threshold above the norm: coefficient 1
    _check_clip_log(r, False)
    r.outer(mu=0.9, lr=0.7, phase=PIER)
    rep = r.check("clip inactive")
    _log("clipped: %s" % rep)
    import paper_2511_17849_amd as pier
    with pytest.raises(pier.PierError, match="PIER_ERR_INVALID_ARG"):
        pier.pier_inner_adamw_clipped(r.ctx, 0, step=9, max_norm=0.0, **r.hp)
    with pytest.raises(pier.PierError, match="PIER_ERR_INVALID_ARG"):
        pier.pier_inner_adamw_clipped(r.ctx, 0, step=9, max_norm=float("nan"), **r.hp)


def test_clipped_norm_is_reproducible_and_tiny_config():
    """Config 1's shapes with the paper's clip threshold 1: N(0, 1e-3) gradients over 3.9 M
    parameters have norm ~ 1.98, so every step is clipped."""
    H_ = _harness()
    from pier_inputs import shapes
    w = shapes.workloads()["tiny"]
    logs = []
    for _ in range(2):
        r = H_.Run(w.numels, w.G, seed=w.seed)
        r.inner_steps(2, clip=1.0)
        _check_clip_log(r, True)
        r.check("tiny clipped")
        logs.append([(n_d, c_d) for _, _, n_d, c_d in r.clip_log])
    assert logs[0] == logs[1]                      # bit-identical norms run to run
    assert abs(logs[0][0][0] - 1e-3 * np.sqrt(w.N)) < 0.01


def test_runs_are_deterministic():
    H_ = _harness()
    _log("determinism")
    outs = []
    for _ in range(2):
        r = H_.Run(RAGGED + [500_000], 8, seed=13)
        r.inner_steps(2)
        r.outer(mu=0.9, lr=1.1, phase=PIER)
        outs.append(r.device_state())
    for k in outs[0]:
        assert np.array_equal(outs[0][k], outs[1][k]), k


# ------------------------------------------------------------------ host offload

@pytest.mark.parametrize("chunk_bytes", [1 << 20, 1_000_016, 1 << 30, 4096])
@pytest.mark.parametrize("phase", [WARMUP, PIER])
def test_offload_is_bit_identical_to_resident(chunk_bytes, phase):
    H_ = _harness()
    numels = [300_000, 1023 * 4, 4, 0, 1_200_000, 20, 64]
    if chunk_bytes == 4096:
        numels = [3000, 1024, 4, 0, 5000, 20]          # many tiny pieces
    _log("offload chunk_bytes=%d phase=%d" % (chunk_bytes, phase))
    res = H_.Run(numels, 4, seed=17)
    off = H_.Run(numels, 4, seed=17, offload=True, chunk_bytes=chunk_bytes)
    for r in (res, off):
        r.inner_steps(2, shared_stream=(phase == WARMUP))
        r.outer(mu=0.95, lr=0.6, phase=phase)
        r.inner_steps(1)
        r.outer(mu=0.9, lr=1.1, phase=phase)                   # second call re-uses plan, slots, events
    off.check("offload")
    a, b = res.device_state(), off.device_state()
    for k in a:
        assert np.array_equal(a[k], b[k]), k
    st = off.stats
    assert st.n_pieces >= 1 and 1 <= st.n_slots <= 4
    assert st.h2d_bytes == 8.0 * sum(numels) and st.d2h_bytes == st.h2d_bytes
    assert st.wall_ms > 0 and st.kernel_ms > 0
    _log("offload stats pieces=%d slots=%d wall=%.3f ms" % (st.n_pieces, st.n_slots, st.wall_ms))


@pytest.mark.parametrize("slots", [2, 9])
def test_offload_with_trailing_write_back(slots):
    """Trailing mode: the compute stream does not wait for the copy-back, so the next inner steps
    are enqueued (and may run) while anchor and M are still on their way to the host; the next
    offload call orders itself behind the previous copy-back.  Same numbers as the resident step."""
    import paper_2511_17849_amd as pier
    H_ = _harness()
    numels = [300_000, 4096, 4, 0, 1_200_000, 20, 64]
    chunk = 1 << 19
    _log("offload, trailing write-back, %d slots" % slots)
    res = H_.Run(numels, 4, seed=23)
    off = H_.Run(numels, 4, seed=23, offload=True, chunk_bytes=chunk)
    off.workspace = torch.empty(2 * chunk * slots, dtype=torch.uint8, device="cuda")
    off.want_stats = False
    pier.pier_ctx_set_offload_writeback(off.ctx, 1)
    with pytest.raises(pier.PierError, match="PIER_ERR_INVALID_ARG"):
        pier.pier_ctx_set_offload_writeback(off.ctx, 2)
    for r in (res, off):
        r.inner_steps(2, shared_stream=True)
        r.outer(mu=0.9, lr=0.0, phase=WARMUP)
        r.inner_steps(1)
        r.outer(mu=0.99, lr=0.6, phase=PIER)
        r.outer(mu=0.95, lr=1.1, phase=PIER)        # back to back: waits for the previous copy-back itself
        r.inner_steps(1)
    rep = off.check("trailing")                    # synchronises the device, hence every stream
    assert rep["bit_exact"], rep
    a, b = res.device_state(), off.device_state()
    for k in a:
        assert np.array_equal(a[k], b[k]), k
    pier.pier_ctx_set_offload_writeback(off.ctx, 0)
    off.want_stats = True
    off.outer(mu=0.9, lr=1.1, phase=PIER)
    res.outer(mu=0.9, lr=1.1, phase=PIER)
    assert off.stats.n_slots == min(slots, off.stats.n_pieces) and 0 < off.stats.compute_ms <= off.stats.wall_ms
    a, b = res.device_state(), off.device_state()
    for k in a:
        assert np.array_equal(a[k], b[k]), k


def test_offload_with_odd_sized_tensors():
    """Flat host arrays pack tensors back to back, so odd sizes put later tensors off
    the 16-byte grid: the kernel must take its scalar path there, same numbers."""
    H_ = _harness()
    numels = [1001, 3, 70_001, 2, 5000]
    _log("offload odd sizes")
    res = H_.Run(numels, 2, seed=19)
    off = H_.Run(numels, 2, seed=19, offload=True, chunk_bytes=65536)
    for r in (res, off):
        r.inner_steps(2)
        r.outer(mu=0.9, lr=0.7, phase=PIER)
    off.check("offload odd")
    a, b = res.device_state(), off.device_state()
    for k in a:
        assert np.array_equal(a[k], b[k]), k


@pytest.mark.parametrize("G", [3, 6, 9, 16, 33, 64])
def test_group_counts_without_a_specialised_kernel(G):
    """Group counts other than 1, 2, 4, 8 (the paper runs 8, 32 and 64 groups) go through the
    kernel that walks the replicas in a run-time loop: vector path on aligned tensors, scalar
    path on misaligned ones and on tails, resident and offloaded, with bf16 working copies."""
    H_ = _harness()
    numels = [4096 * 3, 1025, 7, 0, 20_000, 1024, 3]
    _log("any-G outer step, G=%d" % G)
    res = H_.Run(numels, G, seed=100 + G, shadow=(G % 2 == 1))
    off = H_.Run(numels, G, seed=100 + G, offload=True, chunk_bytes=40_000, shadow=(G % 2 == 1))
    pad = H_.Run(numels, G, seed=100 + G, pad=1, launch=dict(wg_threads=256, lds_bytes=0))
    for r in (res, off, pad):
        r.inner_steps(1, shared_stream=True)
        m_before = r.device_state()["Mo"]
        r.outer(mu=0.9, lr=0.0, phase=WARMUP)
        st = r.device_state()
        assert all(np.array_equal(st["P%d" % g], st["A"]) for g in range(G))     # anchor == model, any G
        assert np.array_equal(m_before, np.zeros_like(m_before)) and np.abs(st["Mo"]).max() > 0
        r.inner_steps(2)
        r.outer(mu=0.99, lr=0.8, phase=PIER)
        rep = r.check("G=%d" % G)
        assert rep["bit_exact"], rep
    a, b = res.device_state(), off.device_state()
    for k in a:
        assert np.array_equal(a[k], b[k]), k


# ------------------------------------------------------------------ error paths (host-side checks)

def test_argument_errors_are_reported_not_launched():
    import paper_2511_17849_amd as pier
    _log("argument errors")
    n = [1000, 24]
    ctx = pier.pier_ctx_create(n, 2)
    dev_t = [torch.zeros(k, device="cuda") for k in n]
    host_t = [torch.zeros(k) for k in n]
    with pytest.raises(pier.PierError, match="PIER_ERR_STATE"):
        pier.pier_inner_adamw(ctx, 0, lr=1e-3, beta1=0.9, beta2=0.95, eps=1e-8, weight_decay=0.1, step=1)
    with pytest.raises(pier.PierError, match="PIER_ERR_INVALID_ARG"):
        pier.pier_bind_replica(ctx, 0, host_t, dev_t, dev_t, dev_t)            # host memory
    with pytest.raises(pier.PierError, match="PIER_ERR_INVALID_ARG"):
        pier.pier_bind_replica(ctx, 5, dev_t, dev_t, dev_t, dev_t)             # no such replica
    big = torch.zeros(1000 + 64, device="cuda")
    with pytest.raises(pier.PierError, match="PIER_ERR_ALIGNMENT"):
        pier.pier_bind_replica(ctx, 0, [big.data_ptr() + 2, dev_t[1]], dev_t, dev_t, dev_t)
    with pytest.raises(pier.PierError, match="PIER_ERR_INVALID_ARG"):
        pier.pier_bind_replica(ctx, 0, [None, dev_t[1]], dev_t, dev_t, dev_t)  # NULL for a non-empty tensor
    P = [[torch.zeros(k, device="cuda") for k in n] for _ in range(4)]
    pier.pier_bind_replica(ctx, 0, *P)
    with pytest.raises(pier.PierError, match="PIER_ERR_INVALID_ARG"):
        pier.pier_inner_adamw(ctx, 0, lr=1e-3, beta1=0.9, beta2=0.95, eps=1e-8, weight_decay=0.1, step=0)
    with pytest.raises(pier.PierError, match="PIER_ERR_INVALID_ARG"):
        pier.pier_inner_adamw(ctx, 0, lr=1e-3, beta1=1.0, beta2=0.95, eps=1e-8, weight_decay=0.1, step=1)
    with pytest.raises(pier.PierError, match="PIER_ERR_STATE"):
        pier.pier_grad_norm_last(ctx, 0)                                       # no clipped step yet
    with pytest.raises(pier.PierError, match="PIER_ERR_STATE"):
        pier.pier_outer_step(ctx, outer_lr=0.7, mu=0.9, phase=PIER)           # replica 1 unbound
    pier.pier_bind_replica(ctx, 1, *P)
    with pytest.raises(pier.PierError, match="PIER_ERR_STATE"):
        pier.pier_outer_step(ctx, outer_lr=0.7, mu=0.9, phase=PIER)           # outer state unbound
    pier.pier_bind_outer(ctx, pier.PIER_LOC_DEVICE, dev_t, dev_t)
    with pytest.raises(pier.PierError, match="PIER_ERR_INVALID_ARG"):
        pier.pier_outer_step(ctx, outer_lr=0.7, mu=0.9, phase=7)
    with pytest.raises(pier.PierError, match="PIER_ERR_STATE"):
        pier.pier_offload_stream(ctx, outer_lr=0.7, mu=0.9, phase=PIER, chunk_bytes=1 << 20,
                                 workspace=torch.zeros(1 << 22, dtype=torch.uint8, device="cuda"))
    with pytest.raises(pier.PierError, match="PIER_ERR_INVALID_ARG"):
        pier.pier_bind_outer(ctx, pier.PIER_LOC_HOST_PINNED, torch.zeros(1024), torch.zeros(1024))  # not pinned
    pa, pm = torch.zeros(1024, pin_memory=True), torch.zeros(1024, pin_memory=True)
    pier.pier_bind_outer(ctx, pier.PIER_LOC_HOST_PINNED, pa, pm)
    with pytest.raises(pier.PierError, match="PIER_ERR_INVALID_ARG"):
        pier.pier_offload_stream(ctx, outer_lr=0.7, mu=0.9, phase=PIER, chunk_bytes=1000,     # not /16
                                 workspace=torch.zeros(1 << 22, dtype=torch.uint8, device="cuda"))
    with pytest.raises(pier.PierError, match="PIER_ERR_INVALID_ARG"):
        pier.pier_offload_stream(ctx, outer_lr=0.7, mu=0.9, phase=PIER, chunk_bytes=1 << 20,
                                 workspace=torch.zeros(64, dtype=torch.uint8, device="cuda"))  # too small
    torch.cuda.synchronize()
    # nothing above may have modified the buffers
    for lst in P:
        for t_ in lst:
            assert float(t_.abs().sum()) == 0.0


def test_bound_pointer_must_hold_numel_elements_of_its_allocation():
    """The extent check of the bind calls is made against the underlying allocation of each
    pointer: a hipMalloc'd block shorter than numel elements, or a pointer so far into a block
    that numel elements overrun it, is an error code at bind time, not a fault at launch time.
    (A torch tensor is a slice of a cached segment, so for torch callers the check bounds the
    segment, not the tensor.)"""
    import paper_2511_17849_amd as pier
    from pier_inputs import device as dev
    MiB = 1 << 20
    n = [MiB, 24]                                   # 4 MiB of floats: a size no allocator rounds
    ctx = pier.pier_ctx_create(n, 1)
    ok = [torch.zeros(k, device="cuda") for k in n]
    exact = dev.RawDeviceBlock(4 * MiB)             # exactly numel[0] floats
    short = dev.RawDeviceBlock(2 * MiB)             # half of them
    pier.pier_bind_replica(ctx, 0, [exact.ptr, ok[1]], ok, ok, ok)                    # fits exactly
    for bad in ([short.ptr, ok[1]], [exact.ptr + 4, ok[1]]):
        with pytest.raises(pier.PierError, match="PIER_ERR_INVALID_ARG") as e:
            pier.pier_bind_replica(ctx, 0, bad, ok, ok, ok)
        assert "do not fit its allocation" in str(e.value)
        for kind in range(1, 4):                     # the same for m, v, grad
            lists = [ok, ok, ok, ok]
            lists[kind] = bad
            with pytest.raises(pier.PierError, match="do not fit its allocation"):
                pier.pier_bind_replica(ctx, 0, *lists)
        with pytest.raises(pier.PierError, match="do not fit its allocation"):
            pier.pier_bind_outer(ctx, pier.PIER_LOC_DEVICE, bad, ok)
        with pytest.raises(pier.PierError, match="do not fit its allocation"):
            pier.pier_bind_outer(ctx, pier.PIER_LOC_DEVICE, ok, bad)
    short_w = dev.RawDeviceBlock(MiB)                # half the bytes of numel[0] bfloat16 values
    with pytest.raises(pier.PierError, match="do not fit its allocation"):
        pier.pier_bind_shadow(ctx, 0, [short_w.ptr, torch.zeros(24, dtype=torch.bfloat16, device="cuda")])
    # a bfloat16 gradient needs half the bytes: numel[0] of them fill the 2 MiB block exactly
    pier.pier_bind_replica(ctx, 0, ok, ok, ok, [short.ptr, ok[1].to(torch.bfloat16)], True)
    # the offload workspace is checked the same way
    pa, pm = torch.zeros(sum(n), pin_memory=True), torch.zeros(sum(n), pin_memory=True)
    pier.pier_bind_outer(ctx, pier.PIER_LOC_HOST_PINNED, pa, pm)
    ws = dev.RawDeviceBlock(2 * MiB)                 # one staging slot of 2 x 1 MiB
    with pytest.raises(pier.PierError, match="do not fit its allocation"):
        pier.pier_offload_stream(ctx, outer_lr=0.7, mu=0.9, phase=PIER, chunk_bytes=MiB,
                                 workspace=(ws.ptr, 4 * MiB))     # claims twice what the block holds
    pier.pier_offload_stream(ctx, outer_lr=0.7, mu=0.9, phase=PIER, chunk_bytes=MiB, workspace=(ws.ptr, 2 * MiB))
    torch.cuda.synchronize()
    pier.pier_ctx_destroy(ctx)


def _snapshot(r):
    torch.cuda.synchronize()
    bufs = [x.flat for g in range(r.G) for x in (r.P[g], r.M1[g], r.V[g])] + [r.A.flat, r.Mo.flat]
    if r.W is not None:
        bufs += [w.flat.view(torch.int16) for w in r.W]
    return [b.clone() for b in bufs], bufs


@pytest.mark.parametrize("offload", [False, True])
def test_train_step_that_is_refused_launches_nothing(offload):
    """On a synchronisation iteration everything the outer step could refuse - the offload piece
    size, a missing, too small, misaligned or overstated workspace, working copies bound for some
    replicas only - is checked before the first inner launch: the call returns the error and every
    buffer is bit-unchanged, so the caller can fix the argument and call again for the same t."""
    import paper_2511_17849_amd as pier
    H_ = _harness()
    numels = [4096, 1000, 36, 0, 70_000]
    r = H_.Run(numels, 2, seed=53, shadow=True, offload=offload, chunk_bytes=65536 if offload else None)
    cfg = dict(T=40, r=4, lr_max=3e-4, lr_min=3e-5, warmup_frac=0.1, clip=0.1)
    r.train_steps(3, **cfg)                                      # t = 1..3: no synchronisation
    hp = {k: r.hp[k] for k in ("beta1", "beta2", "eps", "weight_decay")}
    base = dict(T=40, r=4, lr_max=3e-4, lr_min=3e-5, warmup_frac=0.1, clip_norm=0.1, stream=r.stream, **hp)
    for g in range(r.G):                                         # gradients of iteration 4, as train_steps draws them
        r.Gd[g].fill_normal(seed=r.seed, stream=0, step=4, std=r.grad_std, hip_stream=r.stream)
    before, live = _snapshot(r)
    refused = []
    if offload:
        good = dict(workspace=r.workspace, chunk_bytes=r.chunk_bytes, h2d_stream=r.s_in, d2h_stream=r.s_out)
        small = torch.empty(100, dtype=torch.uint8, device="cuda")
        refused = [("PIER_ERR_INVALID_ARG", dict(good, workspace=None)),
                   ("PIER_ERR_INVALID_ARG", dict(good, workspace=small)),
                   ("PIER_ERR_INVALID_ARG", dict(good, chunk_bytes=1000)),
                   ("PIER_ERR_INVALID_ARG", dict(good, chunk_bytes=0))]
    else:
        good = {}
    for status, kw in refused:
        with pytest.raises(pier.PierError, match=status):
            pier.pier_train_step(r.ctx, 4, **base, **kw)
    if offload:
        # misaligned workspace: a pointer 4 bytes into a large enough block (raw pointer through the ABI)
        wb = r.workspace.numel()
        blk = torch.empty(wb + 64, dtype=torch.uint8, device="cuda")
        import ctypes
        L = pier.binding._load()
        cfgs = pier.TrainCfg(40, 4, pier.PIER_MODE_PIER, 3e-4, 3e-5, 0.1, hp["beta1"], hp["beta2"], hp["eps"],
                             hp["weight_decay"], 0.1, r.chunk_bytes, blk.data_ptr() + 4, wb,
                             r.s_in.cuda_stream or None, r.s_out.cuda_stream or None)
        assert L.pier_train_step(r.ctx.handle, ctypes.byref(cfgs), 4, r.stream.cuda_stream or None) == 2   # PIER_ERR_ALIGNMENT
    # working copies bound for one replica only: the outer step refuses, before anything ran
    kept = r.W[1].tensors
    pier.pier_bind_shadow(r.ctx, 1, None)
    with pytest.raises(pier.PierError, match="PIER_ERR_STATE"):
        pier.pier_train_step(r.ctx, 4, **base, **good)
    pier.pier_bind_shadow(r.ctx, 1, kept)
    torch.cuda.synchronize()
    for was, now in zip(before, live):
        assert torch.equal(was, now)
    # the same iteration with good arguments still works and matches the oracle
    r.t = 3
    r.train_steps(1, **cfg)
    rep = r.check("train_step after refused calls")
    assert rep["bit_exact"], rep
    assert [(t, ph) for t, ph, _, _ in r.sync_log] == [(4, WARMUP)]


def test_round_replays_from_a_hip_graph():
    """Nothing on the path synchronises, allocates or clears memory once a context is bound, so a
    caller can record a whole round - clipped inner steps through the entry point that allocates
    nothing, plain inner steps, lazy-start and Pier outer steps - into a HIP graph and replay it.
    Every replay (with eager work and synchronisations in between) must leave exactly what the
    same calls leave when issued eagerly."""
    import paper_2511_17849_amd as pier
    H_ = _harness()
    numels = [4096 * 3, 1025, 7, 0, 50_000]
    G = 3
    hp = dict(lr=3e-4, beta1=0.9, beta2=0.95, eps=1e-8, weight_decay=0.1)

    def make():
        r = H_.Run(numels, G, seed=61, shadow=True)
        for g in range(G):
            r.Gd[g].fill_normal(seed=61, stream=g, step=1, std=1e-3)
        torch.cuda.synchronize()
        return r

    def round_(r, stream):
        for step in (1, 2):
            for g in range(G):
                pier.pier_inner_adamw_clipped_static(r.ctx, g, step=step, max_norm=0.05, stream=stream, **hp)
        pier.pier_outer_step(r.ctx, outer_lr=0.0, mu=0.9, phase=WARMUP, stream=stream)
        for g in range(G):
            pier.pier_inner_adamw(r.ctx, g, step=3, stream=stream, **hp)
        pier.pier_outer_step(r.ctx, outer_lr=0.8, mu=0.95, phase=PIER, stream=stream)

    eager, graphed = make(), make()
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        round_(graphed, side)                      # warm-up outside the capture (first launches load code)
        side.synchronize()
        with torch.cuda.graph(graph, stream=side):
            round_(graphed, side)
    torch.cuda.synchronize()
    round_(eager, torch.cuda.current_stream())     # the warm-up round
    for replay in range(3):
        graph.replay()
        round_(eager, torch.cuda.current_stream())
        torch.cuda.synchronize()
        a, b = eager.device_state(), graphed.device_state()
        for k in a:
            assert np.array_equal(a[k], b[k]), (replay, k)
        scratch_user = H_.Run([3000], 1, seed=62)  # eager work between replays, sharing the static scratch
        scratch_user.Gd[0].fill_normal(seed=62, stream=0, step=1, std=1e-3)
        pier.pier_inner_adamw_clipped_static(scratch_user.ctx, 0, step=1, max_norm=0.01, **hp)
        torch.cuda.synchronize()
    assert np.abs(a["Mo"]).max() > 0


def test_two_threads_drive_two_contexts_at_once():
    """The threading rule of the ABI: different contexts may be used from different threads at the
    same time (each on its own stream); one thread's failing call does not disturb the other's
    error text.  Results equal those of the same work done alone."""
    import threading
    import paper_2511_17849_amd as pier
    H_ = _harness()
    numels = [200_000, 1025, 7, 0, 4096]
    hp = dict(lr=3e-4, beta1=0.9, beta2=0.95, eps=1e-8, weight_decay=0.1)

    def make(seed):
        r = H_.Run(numels, 2, seed=seed, stream=torch.cuda.Stream())
        for g in range(2):
            r.Gd[g].fill_normal(seed=seed, stream=g, step=1, std=1e-3)
        torch.cuda.synchronize()
        return r

    def work(r, errors, rounds=40):
        try:
            for k in range(rounds):
                for g in range(2):
                    pier.pier_inner_adamw_clipped(r.ctx, g, step=k + 1, max_norm=0.05, stream=r.stream, **hp)
                pier.pier_outer_step(r.ctx, outer_lr=0.7, mu=0.9, phase=PIER if k % 2 else WARMUP, stream=r.stream)
                try:                                   # a failing call on this thread, with its own message
                    pier.pier_inner_adamw(r.ctx, 5 + r.seed, step=1, stream=r.stream, **hp)
                except pier.PierError as e:
                    assert "replica = %d" % (5 + r.seed) in str(e), str(e)
            r.stream.synchronize()
        except Exception as e:                         # surfaced in the main thread below
            errors.append(e)

    alone = [make(71), make(72)]
    errs = []
    for r in alone:
        work(r, errs)
    together = [make(71), make(72)]
    threads = [threading.Thread(target=work, args=(r, errs)) for r in together]
    for t in threads:
        t.start()
    for t in threads:
        t.join(60)
    assert not errs, errs
    torch.cuda.synchronize()
    for a, b in zip(alone, together):
        sa, sb = a.device_state(), b.device_state()
        for k in sa:
            assert np.array_equal(sa[k], sb[k]), k


def test_plain_c_client_of_the_abi(tmp_path):
    """A client that uses nothing but the C ABI, hipMalloc'd tensors and HIP streams (no torch):
    inner steps, the resident outer step, then the host-offload outer step; every buffer it
    writes back is compared with the oracle run on the same case."""
    import os
    import subprocess
    from oracle import pier_oracle as O
    exe = os.path.join(os.path.dirname(__file__), "abi_client", "pier_client")
    if not os.path.exists(exe):
        from paper_2511_17849_amd import build as b
        b.build_abi_client()
    rng = np.random.default_rng(43)
    numel, G, H = [5000, 7, 0, 1025, 4096], 2, 3
    N = sum(numel)
    theta0 = rng.normal(0, 0.02, N).astype(np.float32)
    grads = rng.normal(0, 1e-3, (2, H, G, N)).astype(np.float32)
    case, result = tmp_path / "case.bin", tmp_path / "result.bin"
    with open(case, "wb") as f:
        np.array([len(numel), G, H], np.int32).tofile(f)
        np.array(numel, np.int64).tofile(f)
        theta0.tofile(f)
        grads.tofile(f)
    _log("running %s" % exe)
    out = subprocess.run([exe, str(case), str(result)], capture_output=True, text=True, timeout=100)
    assert out.returncode == 0, out.stderr
    got = np.fromfile(result, np.float32).reshape(3 * G + 2, N)
    hp = dict(lr=3e-4, beta1=0.9, beta2=0.95, eps=1e-8, weight_decay=0.1)
    P = [theta0.copy() for _ in range(G)]
    M1 = [np.zeros(N, np.float32) for _ in range(G)]
    V = [np.zeros(N, np.float32) for _ in range(G)]
    a, Mo = theta0.copy(), np.zeros(N, np.float32)
    t = 0
    for rnd, lr_o in ((0, 0.7), (1, 1.1)):
        for h in range(H):
            t += 1
            for g in range(G):
                O.adamw(P[g], M1[g], V[g], np.ascontiguousarray(grads[rnd, h, g]), step=t, **hp)
        O.outer(P, a, Mo, mu=0.9, lr=lr_o, phase=O.PIER)
    H_ = _harness()
    want = [x for g in range(G) for x in (P[g], M1[g], V[g])] + [a, Mo]
    for k, (g_, w_) in enumerate(zip(got, want)):
        assert H_.tol_ok(g_, w_).all(), k
        assert np.array_equal(g_, w_), k           # and in fact bit for bit


def _same_bits_or_both_nan(got, want):
    got, want = np.asarray(got), np.asarray(want)
    both_nan = np.isnan(got) & np.isnan(want)
    return both_nan | (got.view(np.uint32) == want.view(np.uint32))


def test_special_values_take_the_same_path_as_the_oracle():
    """Zeros of both signs, subnormals, the smallest and largest normals, infinities and NaN in
    every input: the kernels use IEEE division and square root with subnormals kept, so the
    result is the oracle's bit for bit (any NaN standing for any other NaN)."""
    import paper_2511_17849_amd as pier
    from oracle import pier_oracle as O
    tiny, big = np.float32(1.1754944e-38), np.float32(3.4028235e38)
    vals = np.array([0.0, -0.0, 1e-45, -1e-45, 3e-41, tiny, -tiny, 1e-30, 1e-20, -1e-12, 1e-3, -0.02, 1.0,
                     1e10, -1e19, 1e30, big, -big, np.inf, -np.inf, np.nan], dtype=np.float32)
    nonneg = np.array([0.0, 1e-45, 3e-41, tiny, 1e-30, 1e-12, 1e-6, 1.0, 1e19, big, np.inf, np.nan], dtype=np.float32)
    rng = np.random.default_rng(77)
    n = 1024 * 5 + 3                          # vector path, ragged tile and scalar tail
    pick = lambda pool: np.ascontiguousarray(rng.choice(pool, n))
    p, m, v, g = pick(vals), pick(vals), pick(nonneg), pick(vals)
    hp = dict(lr=3e-4, beta1=0.9, beta2=0.95, eps=1e-8, weight_decay=0.1)
    dp, dm, dv, dg = (torch.from_numpy(x.copy()).cuda() for x in (p, m, v, g))
    ctx = pier.pier_ctx_create([n], 2)
    th1 = torch.from_numpy(pick(vals)).cuda()
    pier.pier_bind_replica(ctx, 0, [dp], [dm], [dv], [dg])
    pier.pier_bind_replica(ctx, 1, [th1], [dm], [dv], [dg])
    with np.errstate(all="ignore"):
        for step in (1, 3):
            pier.pier_inner_adamw(ctx, 0, step=step, **hp)
            O.adamw(p, m, v, g, step=step, **hp)
            torch.cuda.synchronize()
            for name, d, h in (("theta", dp, p), ("m", dm, m), ("v", dv, v)):
                ok = _same_bits_or_both_nan(d.cpu().numpy(), h)
                assert ok.all(), (name, step, int((~ok).sum()), d.cpu().numpy()[~ok][:4], h[~ok][:4])
        # outer step, both phases, on the same menagerie
        a, M = pick(vals), pick(vals)
        da, dM = torch.from_numpy(a.copy()).cuda(), torch.from_numpy(M.copy()).cuda()
        pier.pier_bind_outer(ctx, pier.PIER_LOC_DEVICE, [da], [dM])
        th = [p, th1.cpu().numpy().copy()]
        for phase in (WARMUP, PIER):
            pier.pier_outer_step(ctx, outer_lr=1.1, mu=0.95, phase=phase)
            O.outer(th, a, M, mu=0.95, lr=1.1, phase=phase)
            torch.cuda.synchronize()
            for name, d, h in (("anchor", da, a), ("M", dM, M), ("theta0", dp, th[0]), ("theta1", th1, th[1])):
                ok = _same_bits_or_both_nan(d.cpu().numpy(), h)
                assert ok.all(), (name, phase, int((~ok).sum()), d.cpu().numpy()[~ok][:4], h[~ok][:4])
        # clipping with a non-finite norm: an infinite gradient gives coefficient 0 (and 0 * inf = NaN
        # for that element), a NaN gradient leaves the coefficient at 1; same on both sides
        for bad in (np.inf, np.nan):
            g2 = np.ascontiguousarray(rng.normal(0, 1e-3, n).astype(np.float32))
            g2[n // 2] = bad
            dg.copy_(torch.from_numpy(g2))
            pier.pier_inner_adamw_clipped(ctx, 0, step=4, max_norm=1.0, **hp)
            torch.cuda.synchronize()
            coef = O.clip_coef(O.sumsq(g2), 1.0)
            norm_d, coef_d = pier.pier_grad_norm_last(ctx, 0)
            assert coef_d == coef == (0.0 if bad == np.inf else 1.0)
            assert (np.isinf(norm_d) if bad == np.inf else np.isnan(norm_d))
            O.adamw(p, m, v, g2, step=4, grad_scale=coef, **hp)       # the oracle continues from its own state
            for name, d, h in (("theta", dp, p), ("m", dm, m), ("v", dv, v)):
                ok = _same_bits_or_both_nan(d.cpu().numpy(), h)
                assert ok.all(), (name, bad, int((~ok).sum()))
    pier.pier_ctx_destroy(ctx)


def test_all_empty_model_is_a_no_op():
    import paper_2511_17849_amd as pier
    ctx = pier.pier_ctx_create([0, 0], 1)
    e = [None, None]
    pier.pier_bind_replica(ctx, 0, e, e, e, e)
    pier.pier_bind_outer(ctx, pier.PIER_LOC_DEVICE, e, e)
    pier.pier_inner_adamw(ctx, 0, lr=1e-3, beta1=0.9, beta2=0.95, eps=1e-8, weight_decay=0.1, step=1)
    pier.pier_outer_step(ctx, outer_lr=0.7, mu=0.9, phase=PIER)
    torch.cuda.synchronize()


def test_device_generator_matches_host_generator():
    """The device input generator against its numpy twin: same Philox stream, normal
    transform equal to float rounding of log/sin/cos."""
    from pier_inputs import device as dev, generator as gen
    n = 100_003
    t = torch.empty(n, device="cuda")
    dev.fill_normal(t, seed=5, stream=3, step=9, std=1e-3)
    host = gen.normal(n, seed=5, stream=3, step=9, std=1e-3)
    d = t.cpu().numpy()
    assert np.max(np.abs(d - host)) < 5e-9                     # 5e-6 of one std
    assert abs(d.std() - 1e-3) < 2e-5
    tb = torch.empty(n, device="cuda", dtype=torch.bfloat16)
    dev.fill_normal(tb, seed=5, stream=3, step=9, std=1e-3)
    hb = gen.bf16_bits_to_f32(gen.to_bf16_bits(host))
    db = tb.float().cpu().numpy()
    assert np.mean(db != hb) < 1e-3                            # a rounding tie may flip a handful
    assert np.max(np.abs(db - hb)) <= 2.0 ** -8 * np.abs(hb).max()
    part = torch.empty(1000, device="cuda")
    dev.fill_normal(part, seed=5, stream=3, step=9, std=1e-3, first_elem=5000)
    assert torch.equal(part, t[5000:6000])
