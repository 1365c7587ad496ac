"""Host-only checks of the C ABI (no GPU, no compute): the library loads, exports every
function include/pier.h declares, its host-side helpers follow the paper's schedule
constants, and argument errors come back as status codes."""
import ctypes
import os
import re

import pytest

import paper_2511_17849_amd as pier
from test_oracle_pins import _golden_rows

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "pier.h")


def declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(pier_[a-z_0-9]+)\s*\(", text)))


def test_library_is_built_and_exports_every_declared_symbol():
    pier.pier_status_string(0)                 # loads the library (building it first if nothing is built)
    assert os.path.exists(pier.library_path())
    lib = ctypes.CDLL(pier.library_path())
    names = declared_functions()
    assert {"pier_inner_adamw", "pier_outer_step", "pier_offload_stream"} <= set(names)
    assert len(names) >= 15
    for n in names:
        assert hasattr(lib, n), "libpier.so does not export " + n


def test_header_is_plain_c(tmp_path):
    """include/pier.h compiles as C99 on its own (no C++, no HIP, no torch types)."""
    import subprocess
    src = tmp_path / "use_pier.c"
    src.write_text('#include "pier.h"\nint main(void) { pier_outer_hp hp; pier_train_cfg c; (void)hp; (void)c; '
                   'return pier_status_string(PIER_OK) == 0; }\n')
    subprocess.check_call(["gcc", "-std=c99", "-pedantic", "-Wall", "-Werror", "-I", os.path.join(ROOT, "include"),
                           "-c", str(src), "-o", str(tmp_path / "use_pier.o")])


def test_binding_covers_the_header():
    for n in declared_functions():
        assert hasattr(pier, n), "binding lacks " + n


@pytest.mark.parametrize("row", _golden_rows())
def test_schedule_helpers_follow_the_printed_constants(row):
    t, T, ph, mu, lr = row
    assert pier.pier_mu_schedule(t, T) == pytest.approx(mu, abs=1e-7)
    assert pier.pier_outer_lr_schedule(t, T) == pytest.approx(lr, abs=1e-7)
    hp = pier.pier_outer_schedule(t, T)
    assert hp.phase == ph
    if ph == pier.PIER_PHASE_WARMUP:
        assert hp.mu == pytest.approx(0.9, abs=1e-7) and hp.outer_lr == 0.0
    else:
        assert hp.mu == pytest.approx(mu, abs=1e-7) and hp.outer_lr == pytest.approx(lr, abs=1e-7)


def test_schedule_helpers_agree_with_the_oracle_everywhere():
    from oracle import pier_oracle as O
    for T in (10, 37, 1000, 1100, 1800):
        for t in range(1, T + 1):
            hp = pier.pier_outer_schedule(t, T)
            assert (hp.phase, hp.mu, hp.outer_lr) == O.outer_scalars(t, T), (t, T)
            assert pier.pier_mu_schedule(t, T) == O.mu(t, T)
            assert pier.pier_outer_lr_schedule(t, T) == O.outer_lr(t, T)


def test_inner_lr_helper_agrees_with_the_oracle():
    from oracle import pier_oracle as O
    for T, lr_max, lr_min, wf in ((100_000, 4e-4, 4e-5, 0.02), (40, 3e-4, 3e-5, 0.1), (1000, 1.5e-4, 1.5e-5, 0.0)):
        ts = range(1, T + 2) if T <= 1000 else list(range(1, 4000, 3)) + list(range(4000, T + 2, 331))
        for t in ts:
            assert pier.pier_inner_lr_schedule(t, T, lr_max, lr_min, wf) == O.inner_lr(t, T, lr_max, lr_min, wf), t
    assert pier.pier_inner_lr_schedule(2000, 100_000, 4e-4, 4e-5) == pytest.approx(4e-4, rel=1e-6)   # Table I


def test_host_side_argument_errors():
    with pytest.raises(pier.PierError, match="PIER_ERR_INVALID_ARG"):
        pier.pier_ctx_create([], 1)
    with pytest.raises(pier.PierError, match="PIER_ERR_INVALID_ARG"):
        pier.pier_ctx_create([4, -1], 1)
    with pytest.raises(pier.PierError, match="PIER_ERR_INVALID_ARG"):
        pier.pier_ctx_create([4], 0)
    with pytest.raises(pier.PierError, match="PIER_ERR_INVALID_ARG"):
        pier.pier_ctx_create([4], 65)
    with pytest.raises(pier.PierError, match="PIER_ERR_INVALID_ARG"):
        pier.pier_outer_schedule(0, 100)
    with pytest.raises(pier.PierError, match="PIER_ERR_INVALID_ARG"):
        pier.pier_outer_schedule(101, 100)
    ctx = pier.pier_ctx_create([10, 0, 6], 3)
    assert pier.pier_ctx_numel(ctx) == 16
    with pytest.raises(pier.PierError, match="PIER_ERR_INVALID_ARG"):
        pier.pier_ctx_set_launch(ctx, chunk_elems=1000)
    with pytest.raises(pier.PierError, match="PIER_ERR_INVALID_ARG"):
        pier.pier_ctx_set_launch(ctx, unroll=3)
    pier.pier_ctx_set_launch(ctx, chunk_elems=4096, unroll=2, max_grid=16, nontemporal=0)
    for bad in (dict(wg_threads=128), dict(wg_threads=32), dict(lds_bytes=65537), dict(lds_bytes=-2)):
        with pytest.raises(pier.PierError):
            pier.pier_ctx_set_occupancy(ctx, **bad)
    pier.pier_ctx_set_occupancy(ctx, wg_threads=64, lds_bytes=13312)
    pier.pier_ctx_set_occupancy(ctx)                    # back to each kernel's own choice
    for bad in (-1, (1 << 20) + 1):
        with pytest.raises(pier.PierError, match="PIER_ERR_INVALID_ARG"):
            pier.pier_ctx_set_norm_fold(ctx, bad)
    pier.pier_ctx_set_norm_fold(ctx, 4096)
    pier.pier_ctx_set_norm_fold(ctx, 0)                 # the default again
    with pytest.raises(pier.PierError, match="PIER_ERR_STATE"):      # the static-scratch step needs a bound replica too
        pier.pier_inner_adamw_clipped_static(ctx, 0, lr=1e-3, beta1=0.9, beta2=0.95, eps=1e-8, weight_decay=0.0,
                                             step=1, max_norm=1.0)
    with pytest.raises(pier.PierError, match="PIER_ERR_STATE"):
        pier.pier_inner_adamw(ctx, 0, lr=1e-3, beta1=0.9, beta2=0.95, eps=1e-8, weight_decay=0.0, step=1)
    with pytest.raises(pier.PierError, match="PIER_ERR_STATE"):
        pier.pier_outer_step(ctx, outer_lr=0.7, mu=0.9, phase=1)
    tc = dict(T=100, r=10, lr_max=1e-3, lr_min=1e-4, beta1=0.9, beta2=0.95, eps=1e-8, weight_decay=0.1)
    with pytest.raises(pier.PierError, match="PIER_ERR_STATE"):
        pier.pier_train_step(ctx, 1, **tc)                     # nothing bound
    with pytest.raises(pier.PierError, match="PIER_ERR_INVALID_ARG"):
        pier.pier_train_step(ctx, 0, **tc)
    with pytest.raises(pier.PierError, match="PIER_ERR_INVALID_ARG"):
        pier.pier_train_step(ctx, 1, **dict(tc, r=0))
    assert pier.pier_offload_workspace_bytes(ctx, 1 << 20) == 2 * 64      # 16 floats round up to one 64-byte piece
    with pytest.raises(pier.PierError, match="PIER_ERR_INVALID_ARG"):
        pier.pier_offload_workspace_bytes(ctx, 100)
    assert "replica" in pier.pier_last_error() or "chunk_bytes" in pier.pier_last_error()
    assert pier.pier_status_string(0) == "PIER_OK" and pier.pier_status_string(3) == "PIER_ERR_STATE"
    pier.pier_ctx_destroy(ctx)


def test_product_package_does_not_touch_the_oracle():
    """The HIP package must not import, link or read anything under oracle/."""
    pkg = os.path.join(ROOT, "paper_2511_17849_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h", ".cpp")):
                assert "oracle" not in open(os.path.join(dirpath, f)).read().lower(), f
    import subprocess
    needed = subprocess.run(["readelf", "-d", pier.library_path()], capture_output=True, text=True).stdout
    assert "oracle" not in needed
