"""Host-side checks of the C ABI (no GPU, no kernel launch): the library loads, exports every
function that include/fastclip.h declares, rejects bad arguments before touching the device,
sizes its workspace, and its gamma schedule agrees with the oracle's."""
import ctypes as C
import os
import re
import sys

import pytest

from oracle import gamma_cosine
from paper_2407_01445_amd import binding as fc

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def good_cfg(**over):
    kw = dict(version=fc.V3, emb_dtype=fc.BF16, B=1024, b=256, off=512, d=512, N=10_000, gamma=0.8, eps=1e-14,
              rho=6.5, tau_grad_scale=1.0)
    kw.update(over)
    return fc.make_config(**kw)


def fake_bufs(cfg, **over):
    """Non-null, 16-byte aligned fake addresses; nothing is dereferenced on the paths tested here."""
    vals = {n: 0x10000 * (i + 1) for i, n in enumerate(fc._BUF_FIELDS)}
    vals.update(over)
    return fc.fastclip_buffers(*[vals[n] for n in fc._BUF_FIELDS])


def test_library_exports_every_declared_function():
    lib = fc.load()
    header = open(os.path.join(ROOT, "include", "fastclip.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    names = set(re.findall(r"\b(fastclip_[a-z_]+)\s*\(", header))
    assert {"fastclip_step", "fastclip_workspace_bytes", "fastclip_check_indices", "fastclip_gamma_cosine",
            "fastclip_status_string", "fastclip_state_update", "fastclip_step_timed", "fastclip_validate"} <= names
    for n in names:
        assert hasattr(lib, n), n


def test_struct_sizes_match_header_layout():
    assert C.sizeof(fc.fastclip_config) == 16 + 8 * 8 + 4 * 4
    assert C.sizeof(fc.fastclip_buffers) == 24 * 8


def test_valid_config_and_workspace_size():
    cfg = good_cfg()
    assert fc.fastclip_validate(cfg, fake_bufs(cfg)) == fc.OK
    ws = fc.fastclip_workspace_bytes(cfg)
    # at least the two stored exp strips (bf16)
    assert ws >= 2 * 256 * 1024 * 2
    assert ws % 256 == 0
    small = fc.fastclip_workspace_bytes(good_cfg(emb_dtype=fc.F32, B=64, b=64, off=0, d=32))
    assert 0 < small < ws


@pytest.mark.parametrize("over,status", [
    (dict(B=1), fc.ERR_SHAPE), (dict(b=0), fc.ERR_SHAPE), (dict(off=-1), fc.ERR_SHAPE),
    (dict(off=900), fc.ERR_SHAPE), (dict(d=0), fc.ERR_SHAPE), (dict(ld_img=100), fc.ERR_SHAPE),
    (dict(ld_txt=511), fc.ERR_SHAPE), (dict(N=0), fc.ERR_SHAPE), (dict(N=100), fc.ERR_SHAPE),   # b > N
    (dict(state_stride=0), fc.ERR_SHAPE), (dict(state_stride=65), fc.ERR_SHAPE),
    (dict(gamma=0.0), fc.ERR_VALUE), (dict(gamma=1.5), fc.ERR_VALUE), (dict(gamma=float("nan")), fc.ERR_VALUE),
    (dict(eps=-1e-3), fc.ERR_VALUE), (dict(rho=float("inf")), fc.ERR_VALUE), (dict(version=7), fc.ERR_VALUE),
    (dict(emb_dtype=3), fc.ERR_VALUE), (dict(tau_grad_scale=float("nan")), fc.ERR_VALUE),
    (dict(d=100, ld_img=100, ld_txt=100), fc.ERR_UNSUPPORTED), (dict(ld_img=516), fc.ERR_UNSUPPORTED),
    (dict(B=(1 << 24) + 8, b=8), fc.ERR_UNSUPPORTED),
    (dict(B=(1 << 22), b=8), fc.ERR_UNSUPPORTED), (dict(ld_img=(1 << 22) + 8), fc.ERR_UNSUPPORTED),
])
def test_bad_configs_are_rejected(over, status):
    cfg = good_cfg(**over)
    assert fc.fastclip_validate(cfg, None) == status
    assert fc.fastclip_workspace_bytes(cfg) == 0
    # fastclip_step reports the same status before anything is launched
    assert fc.fastclip_step(cfg, fake_bufs(cfg), 0x1000, 1 << 40, stream=0, check=False) == status


def test_f32_path_accepts_any_width():
    assert fc.fastclip_validate(good_cfg(emb_dtype=fc.F32, d=19, ld_img=23, ld_txt=19), None) == fc.OK


def test_struct_size_and_flags_are_checked():
    cfg = good_cfg()
    cfg.struct_size = 8
    assert fc.fastclip_validate(cfg, None) == fc.ERR_SHAPE
    cfg = good_cfg()
    cfg.flags = 32
    assert fc.fastclip_validate(cfg, None) == fc.ERR_SHAPE
    cfg.flags = fc.GATHERED_STATE | fc.FINE_TILES | fc.SINGLE_PASS | fc.TILES_128
    assert fc.fastclip_validate(cfg, None) == fc.OK
    cfg.flags = fc.TILES_128 | fc.TILES_256            # one tile size or the other
    assert fc.fastclip_validate(cfg, None) == fc.ERR_VALUE
    assert fc.fastclip_validate(None, None) == fc.ERR_NULL


def test_single_pass_flag_adds_the_second_strip_only_when_the_whole_batch_is_local():
    """FASTCLIP_SINGLE_PASS keeps l2(j, p) in a strip of its own until the fold transposes it: one more strip of workspace
    when b == B on the bf16 path, nothing otherwise; a batch with more 256 x 256 tiles than compute units takes that form
    without the flag, ragged or not."""
    full = dict(B=520, b=520, off=0, d=64, ld_img=64, ld_txt=64)
    plain, single = good_cfg(flags=fc.TILES_256, **full), good_cfg(flags=fc.SINGLE_PASS | fc.TILES_256, **full)
    strip = 2 * 768 * 576                      # bf16, anchors padded to 256, columns to 64
    assert fc.fastclip_workspace_bytes(single) - fc.fastclip_workspace_bytes(plain) == strip
    share = dict(B=520, b=260, off=0, d=64, ld_img=64, ld_txt=64)
    assert fc.fastclip_workspace_bytes(good_cfg(flags=fc.SINGLE_PASS | fc.TILES_256, **share)) == fc.fastclip_workspace_bytes(good_cfg(flags=fc.TILES_256, **share))
    f32 = dict(emb_dtype=fc.F32, **full)
    assert fc.fastclip_workspace_bytes(good_cfg(flags=fc.SINGLE_PASS, **f32)) == fc.fastclip_workspace_bytes(good_cfg(**f32))
    big = dict(B=3000, b=3000, off=0, d=128, ld_img=128, ld_txt=128)
    assert fc.fastclip_workspace_bytes(good_cfg(flags=fc.SINGLE_PASS, **big)) == fc.fastclip_workspace_bytes(good_cfg(**big))


def test_describe_reports_the_plan():
    assert fc.fastclip_describe(good_cfg(B=1024, b=256, off=512, d=512))["tile"] == 128
    assert fc.fastclip_describe(good_cfg(B=1024, b=256, off=512, d=512, flags=fc.TILES_256))["tile"] == 256
    assert fc.fastclip_describe(good_cfg(B=1024, b=256, off=512, d=512, flags=fc.FINE_TILES))["tile"] == 64
    big = fc.fastclip_describe(good_cfg(B=32768, b=1024, off=0, d=1024))
    assert big["tile"] == 256 and big["nsplit"] == 8 and big["nparts"] == 128 and not big["fused_state"]
    sq = fc.fastclip_describe(good_cfg(B=4096, b=4096, off=0, d=768))
    assert sq["single_pass"] == 1 and sq["tile"] == 256
    assert fc.fastclip_describe(good_cfg(emb_dtype=fc.F32))["tile"] == 0
    g = fc.fastclip_describe(good_cfg(flags=fc.GATHERED_STATE))
    assert g["gathered"] == 1 and g["tile"] == 256
    with pytest.raises(RuntimeError):
        fc.fastclip_describe(good_cfg(B=1))


def test_plans_are_sane_over_a_sweep_of_shapes():
    """Every valid bf16 shape of a sweep: the plan's splits fit the column range, the partial sums count the contrast
    tiles of the chosen size, the workspace is large enough for the two stored strips, and the tile flags behave."""
    import itertools
    for B, frac, d, flags in itertools.product([2, 40, 257, 1000, 1024, 4000, 8192, 40003], [0.01, 0.3, 1.0],
                                                [8, 72, 512, 1024], [0, fc.TILES_128, fc.TILES_256, fc.SINGLE_PASS]):
        b = max(1, int(B * frac))
        cfg = good_cfg(B=B, b=b, off=B - b, d=d, N=max(b, 10), flags=flags)
        assert fc.fastclip_validate(cfg, None) == fc.OK, (B, b, d, flags)
        plan = fc.fastclip_describe(cfg)
        assert plan["tile"] in (128, 256)
        if flags == fc.TILES_256:
            assert plan["tile"] == 256
        if plan["single_pass"]:
            assert b == B and plan["tile"] == 256
        stage_cols = 32
        stages = -(-(-(-B // 64) * 64) // stage_cols)
        assert 1 <= plan["nsplit"] <= min(64, stages), (B, b, d, flags, plan)
        assert plan["nparts"] == -(-B // plan["tile"])
        rows = -(-b // 256) * 256
        assert fc.fastclip_workspace_bytes(cfg) >= 2 * 2 * rows * (-(-B // 64) * 64)


def test_tile_size_is_chosen_by_the_batch_size_unless_asked_for():
    """At most 128 large strip tiles: the library takes 128 x 128 tiles by itself (the layout FASTCLIP_TILES_128 asks for);
    FASTCLIP_TILES_128 reaches up to 191 large tiles; beyond that, with gathered state and in the single-pass form the tiles
    are large whatever is asked."""
    ws = fc.fastclip_workspace_bytes
    small = dict(B=1024, b=256, off=512, d=512)                      # 8 large tiles
    assert ws(good_cfg(**small)) == ws(good_cfg(flags=fc.TILES_128, **small)) != ws(good_cfg(flags=fc.TILES_256, **small))
    mid = dict(B=8192, b=640, off=0, d=512)                          # 192 large tiles... one too many for either
    assert ws(good_cfg(**mid)) == ws(good_cfg(flags=fc.TILES_128, **mid)) == ws(good_cfg(flags=fc.TILES_256, **mid))
    asked = dict(B=5120, b=1024, off=0, d=512)                       # 160 large tiles: only when asked for
    assert ws(good_cfg(**asked)) == ws(good_cfg(flags=fc.TILES_256, **asked)) != ws(good_cfg(flags=fc.TILES_128, **asked))
    assert ws(good_cfg(flags=fc.GATHERED_STATE, **small)) == ws(good_cfg(flags=fc.GATHERED_STATE | fc.TILES_128, **small))
    full = dict(B=512, b=512, off=0, d=128)
    assert ws(good_cfg(flags=fc.SINGLE_PASS, **full)) == ws(good_cfg(flags=fc.SINGLE_PASS | fc.TILES_128, **full))


def test_fine_tiles_flag_changes_the_workspace_only_for_small_batches():
    """FASTCLIP_FINE_TILES: a batch of 256 of 1024 finishes its output tiles in place (no split partial results, so a
    smaller workspace); a batch that fills the chip with 256 x 256 tiles, gathered state and the fp32 path ignore it."""
    small = dict(B=1024, b=256, off=512, d=512)
    assert fc.fastclip_workspace_bytes(good_cfg(flags=fc.FINE_TILES, **small)) < fc.fastclip_workspace_bytes(good_cfg(**small))
    for kw in (dict(B=32768, b=1024, off=0, d=1024), dict(flags_extra=fc.GATHERED_STATE, **small),
               dict(emb_dtype=fc.F32, **small)):
        extra = kw.pop("flags_extra", 0)
        assert fc.fastclip_workspace_bytes(good_cfg(flags=fc.FINE_TILES | extra, **kw)) == \
            fc.fastclip_workspace_bytes(good_cfg(flags=extra, **kw))


@pytest.mark.parametrize("version", [fc.V2, fc.V3])
def test_gathered_state_needs_its_arrays_and_more_workspace(version):
    plain = good_cfg(version=version, B=2048, b=512, off=512)
    cfg = good_cfg(version=version, B=2048, b=512, off=512, flags=fc.GATHERED_STATE)
    assert fc.fastclip_validate(cfg, None) == fc.OK
    assert fc.fastclip_workspace_bytes(cfg) > fc.fastclip_workspace_bytes(plain) > 0
    assert fc.fastclip_validate(cfg, fake_bufs(cfg)) == fc.OK
    assert fc.fastclip_validate(cfg, fake_bufs(cfg, u_glob_img=None)) == fc.ERR_NULL
    assert fc.fastclip_validate(cfg, fake_bufs(cfg, u_glob_txt=None)) == fc.ERR_NULL
    want = fc.ERR_NULL if version == fc.V2 else fc.OK
    assert fc.fastclip_validate(cfg, fake_bufs(cfg, tau_glob_img=None)) == want
    assert fc.fastclip_validate(cfg, fake_bufs(cfg, tau_glob_txt=None)) == want
    # without the flag the arrays are not required
    assert fc.fastclip_validate(plain, fake_bufs(plain, u_glob_img=None, u_glob_txt=None, tau_glob_img=None,
                                                 tau_glob_txt=None)) == fc.OK
    # a single worker holding the whole batch has no remote anchors: same workspace as without the flag
    whole = good_cfg(version=version, b=1024, off=0, flags=fc.GATHERED_STATE)
    assert fc.fastclip_workspace_bytes(whole) == fc.fastclip_workspace_bytes(good_cfg(version=version, b=1024, off=0))


@pytest.mark.parametrize("version,field,status", [
    (fc.V3, "img_glob", fc.ERR_NULL), (fc.V3, "idx", fc.ERR_NULL), (fc.V3, "u_txt", fc.ERR_NULL),
    (fc.V3, "tau", fc.ERR_NULL), (fc.V3, "d_tau", fc.ERR_NULL), (fc.V0, "d_tau", fc.ERR_NULL),
    (fc.V1, "d_tau", fc.OK), (fc.V3, "tau_img", fc.OK), (fc.V2, "tau_img", fc.ERR_NULL),
    (fc.V2, "d_tau_txt", fc.ERR_NULL), (fc.V2, "tau", fc.OK), (fc.V2, "d_tau", fc.OK),
    (fc.V3, "g_img", fc.OK), (fc.V3, "u_new_txt", fc.OK), (fc.V3, "loss", fc.ERR_NULL),
])
def test_required_pointers(version, field, status):
    cfg = good_cfg(version=version)
    assert fc.fastclip_validate(cfg, fake_bufs(cfg, **{field: None})) == status


def test_norms_come_in_pairs():
    cfg = good_cfg()
    assert fc.fastclip_validate(cfg, fake_bufs(cfg, norm_img=None, norm_txt=None)) == fc.OK
    assert fc.fastclip_validate(cfg, fake_bufs(cfg, norm_img=None)) == fc.ERR_NULL
    assert fc.fastclip_validate(cfg, fake_bufs(cfg, norm_txt=None)) == fc.ERR_NULL


def test_misaligned_matrices_and_workspace():
    cfg = good_cfg()
    assert fc.fastclip_validate(cfg, fake_bufs(cfg, img_glob=0x10002)) == fc.ERR_UNSUPPORTED
    assert fc.fastclip_validate(cfg, fake_bufs(cfg, d_txt=0x10004)) == fc.ERR_UNSUPPORTED
    need = fc.fastclip_workspace_bytes(cfg)
    bufs = fake_bufs(cfg)
    assert fc.fastclip_step(cfg, bufs, 0x1000, need - 1, stream=0, check=False) == fc.ERR_WORKSPACE
    assert fc.fastclip_step(cfg, bufs, 0x1010, need, stream=0, check=False) == fc.ERR_WORKSPACE
    assert fc.fastclip_step(cfg, bufs, None, need, stream=0, check=False) == fc.ERR_NULL
    with pytest.raises(fc.FastclipError):
        fc.fastclip_step(cfg, bufs, 0x1000, 16, stream=0)


def test_state_update_and_check_indices_argument_errors():
    lib = fc.load()
    assert lib.fastclip_state_update(None, 4, 10, 0.5, 3.0, 1, 1, 1, 1, 1, 1, None) == fc.ERR_NULL
    assert lib.fastclip_state_update(1, -1, 10, 0.5, 3.0, 1, 1, 1, 1, 1, 1, None) == fc.ERR_SHAPE
    assert lib.fastclip_state_update(1, 11, 10, 0.5, 3.0, 1, 1, 1, 1, 1, 1, None) == fc.ERR_SHAPE   # more indices than entries
    assert lib.fastclip_state_update(1, 4, 10, 0.0, 3.0, 1, 1, 1, 1, 1, 1, None) == fc.ERR_VALUE
    assert lib.fastclip_state_update(1, 4, 10, 0.5, 0.0, 1, 1, 1, 1, 1, 1, None) == fc.ERR_VALUE
    assert lib.fastclip_state_update(1, 0, 10, 0.5, 3.0, 1, 1, 1, 1, 1, 1, None) == fc.OK      # empty batch
    assert lib.fastclip_state_update_strided(1, 4, 10, 0, 0.5, 3.0, 1, 1, 1, 1, 1, 1, None) == fc.ERR_SHAPE
    assert lib.fastclip_state_update_strided(1, 4, 10, 65, 0.5, 3.0, 1, 1, 1, 1, 1, 1, None) == fc.ERR_SHAPE
    assert lib.fastclip_state_update_strided(1, 0, 10, 4, 0.5, 3.0, 1, 1, 1, 1, 1, 1, None) == fc.OK
    need = fc.fastclip_check_indices_workspace_bytes(100)
    assert need >= 256 + 200 * 8
    assert lib.fastclip_check_indices(None, 100, 10, 0x1000, need, None) == fc.ERR_NULL
    assert lib.fastclip_check_indices(0x2000, 100, 10, 0x1000, need - 1, None) == fc.ERR_WORKSPACE
    assert lib.fastclip_check_indices(0x2000, 0, 10, 0x1000, need, None) == fc.OK


def test_gamma_schedule_matches_oracle():
    for (ipe, E, gmin) in [(1, 100, 0.2), (10, 8, 0.2), (7, 3, 0.9), (1, 1, 0.5)]:
        for t in list(range(0, 130)) + [1000, 10 ** 6]:
            assert fc.fastclip_gamma_cosine(t, ipe, E, gmin) == pytest.approx(gamma_cosine(t, ipe, E, gmin), abs=1e-7)


def test_status_strings_and_phase_names():
    seen = {fc.fastclip_status_string(s) for s in range(8)}
    assert len(seen) == 8 and "ok" in seen
    assert fc.fastclip_status_string(99) == "unknown status"
    assert fc.fastclip_phase_name(1) == "strips" and fc.fastclip_phase_name(7) == "unused"


def test_temperature_update_argument_errors():
    good = dict(optimizer=fc.TAU_ADAMW, step=1, lr=1e-3, beta1=0.9, beta2=0.999)
    upd = fc.make_tau_update(**good)
    assert C.sizeof(fc.fastclip_tau_update) == 48 and C.sizeof(fc.fastclip_tau_state) == 9 * 8
    st3 = fc.make_tau_state(tau=0x1000, m=0x2000, v=0x3000)
    st2 = fc.make_tau_state(tau_img=0x1000, tau_txt=0x2000, m_img=0x3000, v_img=0x4000, m_txt=0x5000, v_txt=0x6000)
    call = lambda ver, u, s, idx=0x100, b=4, d=0x200, di=0x300, dt=0x400: fc.fastclip_temperature_update(
        ver, u, s, idx, b, 10, d, di, dt, stream=0, check=False)
    assert call(fc.V1, upd, st3) == fc.OK                                   # constant temperature: nothing to do
    assert call(fc.V3, None, st3) == fc.ERR_NULL and call(fc.V3, upd, None) == fc.ERR_NULL
    assert call(fc.V3, upd, fc.make_tau_state(tau=0x1000, m=0x2000)) == fc.ERR_NULL        # AdamW needs v
    assert call(fc.V3, upd, st3, d=None) == fc.ERR_NULL
    assert call(fc.V2, upd, st3) == fc.ERR_NULL                             # V2 needs the per-sample arrays
    assert call(fc.V2, upd, st2, idx=None) == fc.ERR_NULL
    assert call(fc.V2, upd, st2, b=-1) == fc.ERR_SHAPE
    assert call(fc.V2, upd, st2, b=11) == fc.ERR_SHAPE                      # more indices than the 10 entries
    assert call(fc.V2, fc.make_tau_update(state_stride=-1, **good), st2) == fc.ERR_SHAPE
    assert call(fc.V2, fc.make_tau_update(state_stride=65, **good), st2) == fc.ERR_SHAPE
    assert call(fc.V2, upd, st2, b=0) == fc.OK
    assert call(7, upd, st3) == fc.ERR_VALUE
    for bad in (dict(optimizer=0), dict(optimizer=5), dict(step=0), dict(lr=-1.0), dict(beta1=1.0), dict(beta2=-0.1),
                dict(lr=float("nan")), dict(eps=-1.0)):
        assert call(fc.V3, fc.make_tau_update(**{**good, **bad}), st3) == fc.ERR_VALUE, bad
    u = fc.make_tau_update(**good)
    u.struct_size = 8
    assert call(fc.V3, u, st3) == fc.ERR_SHAPE
    # SGD with momentum and Lion keep no second moment
    sg = fc.make_tau_update(**{**good, "optimizer": fc.TAU_SGDM})
    assert fc.fastclip_validate(good_cfg(), None) == fc.OK
    # the fused entry point checks the step's arguments first, then that the step reads the tensors it updates
    cfg = good_cfg(version=fc.V3)
    bufs = fake_bufs(cfg)
    assert fc.fastclip_step_update_tau(cfg, bufs, sg, fc.make_tau_state(tau=0x999, m=0x2000), 0x1000, 1 << 40,
                                       stream=0, check=False) == fc.ERR_VALUE
    # ... and that both describe the same layout of the per-sample arrays
    cfg2 = good_cfg(version=fc.V2, state_stride=4)
    bufs2 = fake_bufs(cfg2)
    st_same = fc.make_tau_state(tau_img=bufs2.tau_img, tau_txt=bufs2.tau_txt, m_img=0x3000, m_txt=0x5000)
    assert fc.fastclip_step_update_tau(cfg2, bufs2, sg, st_same, 0x1000, 1 << 40, stream=0, check=False) == fc.ERR_VALUE
    assert fc.fastclip_step_update_tau(cfg, bufs, None, None, 0x1000, 1 << 40, stream=0, check=False) == fc.ERR_NULL


def test_structs_keep_their_tensors_alive():
    """The structs carry plain addresses; a tensor handed to make_buffers / make_tau_state as a temporary must not be
    freed while the struct is in use (a freed moment array under a later kernel is a wild write)."""
    import gc
    import weakref

    class FakeTensor:            # what the binding asks of a tensor
        is_cuda = True

        def __init__(self, addr):
            self.addr = addr

        def data_ptr(self):
            return self.addr

    for make, field in ((fc.make_tau_state, "m_img"), (fc.make_buffers, "idx")):
        t = FakeTensor(0x4000)
        alive = weakref.ref(t)
        st = make(**{field: t})
        del t
        gc.collect()
        assert alive() is not None and getattr(st, field) == 0x4000
        del st
        gc.collect()
        assert alive() is None


def test_bench_refuses_more_than_one_gpu():
    """This build runs on one GPU only: bench.py --gpus N with N > 1 exits with a message, before touching a GPU."""
    import subprocess
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode != 0
    assert "ONE GPU" in r.stderr


def test_state_phase_and_static_step_argument_errors():
    """Every early return of fastclip_state_phase and fastclip_step_static (nothing is launched, nothing dereferenced)."""
    lib = fc.load()
    cfg = good_cfg(version=fc.V2, B=1000, b=1000, off=0)
    bufs = fake_bufs(cfg)
    need = fc.fastclip_state_phase_workspace_bytes(1000)
    assert need >= 2 * 8 * 8 and need % 256 == 0 and fc.fastclip_state_phase_workspace_bytes(0) == 0
    call = lambda c, b, sums=0x1000, coef=0x2000, ws=0x3000, nbytes=need, upd=None, st=None: \
        lib.fastclip_state_phase(C.byref(c), C.byref(b) if b is not None else None, upd, st, sums, coef, ws, nbytes, None)
    assert call(good_cfg(B=1), bufs) == fc.ERR_SHAPE
    assert call(cfg, None) == fc.ERR_NULL
    assert call(cfg, bufs, sums=None) == fc.ERR_NULL and call(cfg, bufs, coef=None) == fc.ERR_NULL
    assert call(cfg, fake_bufs(cfg, idx=None)) == fc.ERR_NULL
    assert call(cfg, fake_bufs(cfg, tau_img=None)) == fc.ERR_NULL
    assert call(good_cfg(version=fc.V3), fake_bufs(cfg, d_tau=None)) == fc.ERR_NULL
    assert call(cfg, bufs, nbytes=need - 1) == fc.ERR_WORKSPACE
    assert call(cfg, bufs, ws=0x3010) == fc.ERR_WORKSPACE
    upd = fc.make_tau_update(optimizer=fc.TAU_ADAMW, step=1, lr=1e-3, beta1=0.9, beta2=0.99, eps=1e-8)
    assert call(cfg, bufs, upd=C.byref(upd)) == fc.ERR_NULL          # update without its state
    # static step: too large for the array, bad shape
    big = good_cfg(B=32768, b=1024, off=0, d=1024)
    assert fc.fastclip_workspace_bytes(big) > fc.STATIC_SCRATCH_BYTES
    assert fc.fastclip_step_static(big, fake_bufs(big), stream=0, check=False) == fc.ERR_WORKSPACE
    assert fc.fastclip_step_static(good_cfg(b=0), bufs, stream=0, check=False) == fc.ERR_SHAPE
    assert fc.fastclip_step_static(cfg, fake_bufs(cfg, loss=None), stream=0, check=False) == fc.ERR_NULL


def test_normalize_rows_argument_errors():
    lib = fc.load()
    call = lambda raw=0x1000, rd=fc.F32, ldr=64, b=4, d=64, unit=0x2000, ud=fc.BF16, ldu=64, norm=0x3000: \
        lib.fastclip_normalize_rows(raw, rd, ldr, b, d, unit, ud, ldu, norm, None)
    assert call(raw=None) == fc.ERR_NULL and call(unit=None) == fc.ERR_NULL and call(norm=None) == fc.ERR_NULL
    assert call(b=-1) == fc.ERR_SHAPE and call(d=0) == fc.ERR_SHAPE and call(ldr=63) == fc.ERR_SHAPE and call(ldu=8) == fc.ERR_SHAPE
    assert call(rd=7) == fc.ERR_VALUE and call(ud=-1) == fc.ERR_VALUE
    assert call(unit=0x1000) == fc.ERR_VALUE                     # in place needs equal types
    assert call(b=0) == fc.OK                                    # nothing to do, nothing launched
    assert lib.fastclip_measure_record_rmw(None, 4, 10, 0x1000, 8, None) == fc.ERR_NULL
    assert lib.fastclip_measure_record_rmw(0x1000, 11, 10, 0x2000, 8, None) == fc.ERR_SHAPE
    assert lib.fastclip_measure_record_rmw(0x1000, 4, 10, 0x2000, 12, None) == fc.ERR_SHAPE
    assert lib.fastclip_measure_record_rmw(0x1000, 4, 10, 0x2010, 8, None) == fc.ERR_UNSUPPORTED
    assert lib.fastclip_measure_record_rmw(0x1000, 0, 10, 0x2000, 8, None) == fc.OK


def test_measure_strips_argument_errors():
    lib = fc.load()
    cfg = good_cfg(B=2048, b=512, off=512, d=128)
    bufs = fake_bufs(cfg)
    ms, stats = C.c_float(), (C.c_double * 6)()
    need = fc.fastclip_workspace_bytes(cfg) + fc.MEASURE_STRIPS_EXTRA_BYTES
    call = lambda c=cfg, ws=0x1000, nbytes=need, abl=0, reps=2: lib.fastclip_measure_strips(
        C.byref(c), C.byref(bufs), ws, nbytes, None, abl, reps, C.byref(ms), stats)
    assert call(nbytes=need - 1) == fc.ERR_WORKSPACE and call(ws=None) == fc.ERR_NULL and call(reps=0) == fc.ERR_SHAPE
    assert call(c=good_cfg(emb_dtype=fc.F32, B=64, b=64, off=0, d=32), nbytes=1 << 30) == fc.ERR_UNSUPPORTED
    assert call(c=good_cfg(B=2048, b=512, off=512, d=128, flags=fc.GATHERED_STATE), nbytes=1 << 30) == fc.ERR_UNSUPPORTED
    assert lib.fastclip_measure_mfma_ceiling(0, 16, 0x1000, 1 << 20, None, C.byref(ms), stats) == fc.ERR_SHAPE
    assert lib.fastclip_measure_mfma_ceiling(16, 16, 0x1000, 64, None, C.byref(ms), stats) == fc.ERR_WORKSPACE
