"""Host-only checks of the C ABI: the library loads, exports every symbol the
header declares, validates arguments, and its RAE entry points match the
oracle.  No GPU work is issued here."""
import ctypes
import os
import re

import numpy as np
import pytest

from oracle.rae import RAE
from paper_2506_24119_amd import binding as sb
from paper_2506_24119_amd import inputs as si

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(sb.LIB_PATH):
        from paper_2506_24119_amd.build import build
        build(verbose=False)
    return sb.load_library()


def test_every_declared_symbol_is_exported(lib):
    header = open(os.path.join(ROOT, "include", "spiral.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(spiral_[a-z0-9_]+)\s*\(", header))
    assert declared == set(sb.EXPORTS), declared ^ set(sb.EXPORTS)
    for name in declared:
        assert hasattr(lib, name), name
    assert "gfx950" in sb.spiral_version()


def test_missing_library_fails_loudly(tmp_path):
    with pytest.raises(OSError):
        sb.load_library(str(tmp_path / "nope.so"))


def test_rae_matches_oracle_within_1e6(lib):
    gid, r0 = si.make_game_outcomes(3, 500, seed=7)          # TicTacToe / Kuhn Poker / Negotiation
    h = sb.spiral_rae_create(3, 0.95)
    ref = RAE(3, 0.95)
    for lo in range(0, 500, 128):                            # 128 trajectories per policy step
        adv = sb.spiral_rae_update(h, gid[lo:lo + 128], r0[lo:lo + 128])
        want = ref.update(gid[lo:lo + 128], r0[lo:lo + 128])
        assert np.abs(adv - want).max() <= 1e-6
        assert np.abs(sb.spiral_rae_get(h, 3) - ref.b).max() <= 1e-6
    # bit-identical in fact: same float64 operations in the same order
    assert np.array_equal(sb.spiral_rae_get(h, 3), ref.b)
    # snapshot / restore
    snap = sb.spiral_rae_get(h, 3)
    sb.spiral_rae_update(h, [0], [1.0])
    sb.spiral_rae_set(h, snap)
    assert np.array_equal(sb.spiral_rae_get(h, 3), snap)
    sb.spiral_rae_free(h)


def test_rae_rejects_bad_arguments_without_side_effects(lib):
    with pytest.raises(sb.SpiralError) as e:
        sb.spiral_rae_create(0, 0.95)
    assert e.value.code == sb.SPIRAL_ERR_INVALID_ARG
    with pytest.raises(sb.SpiralError):
        sb.spiral_rae_create(2, 1.5)
    h = sb.spiral_rae_create(2, 0.95)
    sb.spiral_rae_update(h, [0, 1], [1.0, -1.0])
    before = sb.spiral_rae_get(h, 2)
    for gid, r in (([0, 2], [1.0, 1.0]), ([0, -1], [1.0, 1.0]), ([0, 1], [1.0, float("nan")])):
        with pytest.raises(sb.SpiralError) as e:
            sb.spiral_rae_update(h, gid, r)
        assert e.value.code == sb.SPIRAL_ERR_INVALID_ARG
        assert np.array_equal(sb.spiral_rae_get(h, 2), before)     # nothing was applied
    assert "rae_update" in sb.spiral_last_error()
    sb.spiral_rae_free(h)


def test_model_load_validates_geometry(lib):
    g = si.GEOMETRIES["tiny"]
    n = 3 + sb.SPIRAL_LAYER_SLOTS * g.n_layers
    fake = [0x1000 * (i + 1) for i in range(n)]                     # never dereferenced by model_load
    for i in range(g.n_layers):
        for slot in (4, 5, 6, 7, 8):
            fake[3 + i * sb.SPIRAL_LAYER_SLOTS + slot] = None
    m = sb.spiral_model_load(sb.make_config(g), fake)
    assert sb.spiral_workspace_bytes(m, 4, 128) > 0
    assert sb.spiral_workspace_bytes(m, 0, 128) == 0
    assert sb.spiral_kv_pool_bytes(m, 10, 4, 8) > 10 * g.n_layers * g.n_kv_heads * 2 * 16 * g.head_dim * 2
    sb.spiral_model_free(m)

    def expect(code, **over):
        cfg = sb.make_config(si.ModelGeometry(**{**g.__dict__, **over}))
        with pytest.raises(sb.SpiralError) as e:
            sb.spiral_model_load(cfg, fake)
        assert e.value.code == code, sb.spiral_last_error()

    expect(sb.SPIRAL_ERR_SHAPE, head_dim=48)
    expect(sb.SPIRAL_ERR_SHAPE, n_q_heads=5)
    expect(sb.SPIRAL_ERR_SHAPE, kv_block_tokens=32)
    expect(sb.SPIRAL_ERR_INVALID_ARG, qk_norm=True)                 # q/k norm gains missing
    expect(sb.SPIRAL_ERR_INVALID_ARG, n_layers=3)                   # pointer table too short
    bad = list(fake)
    bad[0] = 0x1008                                                 # misaligned embedding
    with pytest.raises(sb.SpiralError):
        sb.spiral_model_load(sb.make_config(g), bad)


def test_sample_argument_checks_need_no_gpu(lib):
    with pytest.raises(sb.SpiralError) as e:
        sb.load_library()  # ensure loaded
        rc = lib.spiral_sample(None, 1, 8, 1.0, 0, None, None, None, None, None)
        sb._check(rc)
    assert e.value.code == sb.SPIRAL_ERR_INVALID_ARG


def test_new_entry_points_validate_arguments_without_a_gpu(lib):
    """Truncated sampler, scoring pass, objective and repack reject bad arguments before any GPU call."""
    def code(rc):
        with pytest.raises(sb.SpiralError) as e:
            sb._check(rc)
        return e.value.code

    fake = ctypes.c_void_p(0x10000)
    # top_p outside (0, 1]
    for bad_p in (0.0, -1.0, 1.5, float("nan")):
        assert code(lib.spiral_sample_truncated(fake, 1, 8, 1.0, 0, bad_p, 0, None, None, None, fake, None, None)) == sb.SPIRAL_ERR_INVALID_ARG
    # greedy decoding has no threshold to report
    assert code(lib.spiral_sample_truncated(fake, 1, 8, 0.0, 2, 0.9, 0, None, None, None, fake, fake, None)) == sb.SPIRAL_ERR_INVALID_ARG
    # generated noise needs sequence ids and steps
    assert code(lib.spiral_sample_truncated(fake, 1, 8, 1.0, 2, 0.9, 0, None, None, None, fake, None, None)) == sb.SPIRAL_ERR_INVALID_ARG
    assert code(lib.spiral_sample_truncated(None, 1, 8, 1.0, 2, 0.9, 0, None, None, None, fake, None, None)) == sb.SPIRAL_ERR_INVALID_ARG
    # workspace variant: null, misaligned or too small workspace; the size query answers 0 for a bad shape
    need = lib.spiral_sample_truncated_workspace_bytes(4, 50000)
    assert need > 0 and lib.spiral_sample_truncated_workspace_bytes(0, 50000) == 0 and lib.spiral_sample_truncated_workspace_bytes(4, 0) == 0
    one = (ctypes.c_int32 * 4)(0, 1, 2, 3)
    for ws, nbytes in ((None, need), (ctypes.c_void_p(0x10010), need), (fake, need - 1)):
        assert code(lib.spiral_sample_truncated_ws(fake, 4, 50000, 1.0, 2, 0.9, 0, one, one, None, fake, None, ws, nbytes, None)) == sb.SPIRAL_ERR_INVALID_ARG
    assert code(lib.spiral_sample_truncated_ws(fake, 4, 50000, 1.0, 2, 1.5, 0, one, one, None, fake, None, fake, need, None)) == sb.SPIRAL_ERR_INVALID_ARG
    # objective: null pointers, negative count, bad clip parameter
    assert code(lib.spiral_policy_objective(None, fake, fake, None, 4, 0.2, fake, None)) == sb.SPIRAL_ERR_INVALID_ARG
    assert code(lib.spiral_policy_objective(fake, fake, fake, None, -1, 0.2, fake, None)) == sb.SPIRAL_ERR_INVALID_ARG
    assert code(lib.spiral_policy_objective(fake, fake, fake, None, 4, -0.1, fake, None)) == sb.SPIRAL_ERR_INVALID_ARG
    # scoring and repack without a model
    assert code(lib.spiral_score(None, None, None, None, 1, fake, fake, fake, 1024, fake, None)) == sb.SPIRAL_ERR_NOT_LOADED
    assert code(lib.spiral_score(None, None, None, None, 1, fake, None, fake, 1024, fake, None)) == sb.SPIRAL_ERR_INVALID_ARG
    assert code(lib.spiral_model_repack(None, fake, 1 << 20, None)) == sb.SPIRAL_ERR_NOT_LOADED
    assert lib.spiral_model_repack_bytes(None) == 0


def test_repack_plan_and_buffer_checks(lib):
    """Repack sizes follow the geometry (every matrix padded to 32 rows, gate/up interleaved into one); a
    short or misaligned buffer is refused, and fp32 models cannot be repacked."""
    g = si.ModelGeometry("rp", 2, 256, 8, 2, 128, 640, 1000, 1e6, qk_norm=True)
    n = 3 + sb.SPIRAL_LAYER_SLOTS * g.n_layers
    fake = [0x100000 + 0x1000 * i for i in range(n)]
    cfg = sb.make_config(g)
    m = sb.spiral_model_load(cfg, fake)
    try:
        a256 = lambda x: (x + 255) // 256 * 256
        qw, kw, d, F = 8 * 128, 2 * 128, 256, 640
        per_layer = a256((qw + 2 * kw) * d * 2) + a256(d * qw * 2) + a256(2 * F * d * 2) + a256(d * F * 2)
        want = per_layer * 2 + a256(1024 * d * 2)                   # vocabulary 1000 padded to 1024 rows
        assert lib.spiral_model_repack_bytes(m) == want
        with pytest.raises(sb.SpiralError) as e:
            sb._check(lib.spiral_model_repack(m, ctypes.c_void_p(0x200000), want - 1, None))
        assert e.value.code == sb.SPIRAL_ERR_INVALID_ARG
        with pytest.raises(sb.SpiralError) as e:
            sb._check(lib.spiral_model_repack(m, ctypes.c_void_p(0x200010), want, None))
        assert e.value.code == sb.SPIRAL_ERR_INVALID_ARG
    finally:
        sb.spiral_model_free(m)
    g32 = si.ModelGeometry("rp32", 1, 128, 4, 2, 32, 512, 1024, 1e4, weight_dtype=0)
    n = 3 + sb.SPIRAL_LAYER_SLOTS
    m = sb.spiral_model_load(sb.make_config(g32), [0x100000 + 0x1000 * i for i in range(n)])
    try:
        assert lib.spiral_model_repack_bytes(m) == 0
    finally:
        sb.spiral_model_free(m)


def test_step_variants_and_hooks_validate_arguments_without_a_gpu(lib):
    """The fused decode + sample step, the static-workspace step, the tuning call and the streaming probe refuse bad
    arguments before any GPU call."""
    def code(rc):
        with pytest.raises(sb.SpiralError) as e:
            sb._check(rc)
        return e.value.code

    fake = ctypes.c_void_p(0x10000)
    assert code(lib.spiral_decode_sample_step(None, None, None, 1, fake, fake, 1 << 20, 1.0, 0, None, fake, None)) == sb.SPIRAL_ERR_NOT_LOADED
    assert code(lib.spiral_decode_step_static(None, None, None, 1, fake, fake, None)) == sb.SPIRAL_ERR_NOT_LOADED
    assert lib.spiral_static_workspace_bytes() == 16 << 20
    assert code(lib.spiral_model_tune(None, b"chunk=4")) == sb.SPIRAL_ERR_NOT_LOADED
    assert code(int(lib.spiral_kv_pool_status_offset(None))) == sb.SPIRAL_ERR_NOT_LOADED
    ms = ctypes.c_double(0.0)
    assert code(lib.spiral_probe_stream_read(None, 1 << 24, 1, ctypes.byref(ms), None)) == sb.SPIRAL_ERR_INVALID_ARG
    assert code(lib.spiral_probe_stream_read(fake, 1 << 10, 1, ctypes.byref(ms), None)) == sb.SPIRAL_ERR_INVALID_ARG
    assert code(lib.spiral_probe_stream_read(fake, 1 << 24, 0, ctypes.byref(ms), None)) == sb.SPIRAL_ERR_INVALID_ARG
    g = si.ModelGeometry("tn", 1, 128, 4, 2, 32, 512, 1024, 1e4)
    m = sb.spiral_model_load(sb.make_config(g), [0x100000 + 0x1000 * i for i in range(3 + sb.SPIRAL_LAYER_SLOTS)])
    try:
        sb.spiral_model_tune(m, "chunk=4,wgs=12,qkv=64:3,unknown=7,fail_after=0")      # unknown keys are ignored
        assert code(lib.spiral_model_tune(m, None)) == sb.SPIRAL_ERR_INVALID_ARG
        # pools of another model / null pools are refused by both step variants
        assert code(lib.spiral_decode_step_static(m, None, None, 1, fake, fake, None)) == sb.SPIRAL_ERR_NOT_LOADED
        assert code(lib.spiral_decode_sample_step(m, None, None, 1, fake, fake, 1 << 20, 1.0, 0, None, fake, None)) == sb.SPIRAL_ERR_NOT_LOADED
    finally:
        sb.spiral_model_free(m)
