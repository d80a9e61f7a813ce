"""The kernels' own sources, compiled for the host against a stand-in for the HIP runtime and the gfx950 builtins
(tests/emu), run one small step per code path under AddressSanitizer and are compared with the oracle.

What this can show: an access outside a buffer (every buffer is an exact-size allocation, the matrices end with the
last row's d elements), a barrier that not every thread reaches (the run would hang: bounded by a time-out), wrong
indexing (the outputs would disagree with the oracle).  What it cannot: timing, the asynchrony of direct-to-LDS loads
(they copy at once here), anything the GPU compiler does.  It is also the only place where the opt-in fine-tile path
runs as long as it is kept off the GPU."""
from __future__ import annotations

import os
import subprocess
import sys

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, os.path.join(ROOT, "tests", "emu"))
import build_emu  # noqa: E402

from oracle import ADAMW, LION, V0, V1, V2, V3, ema_update, fcco_step, normalize_rows, temperature_update  # noqa: E402
from paper_2407_01445_amd import binding as fc  # noqa: E402
from paper_2407_01445_amd.workloads import draw_indices, make_embeddings  # noqa: E402

pytestmark = pytest.mark.skipif(build_emu.host_compiler() is None, reason="no host clang++ to build the emulation with")


# FASTCLIP_EMU_SANITIZER=thread (missing barriers show as data races on the LDS arrays) or =memory (with the workspace
# and the outputs left uninitialised: a value nobody wrote that reaches a branch, an address or an output) instead of
# the default AddressSanitizer; all three are clean on every case below.
SANITIZER = os.environ.get("FASTCLIP_EMU_SANITIZER", "address")


@pytest.fixture(scope="module")
def emu_step():
    return build_emu.build("-fsanitize=" + SANITIZER)


def bf16_bits(x32):
    return (np.ascontiguousarray(x32, np.float32).view(np.uint32) >> 16).astype(np.uint16)


def run_case(exe, tmp_path, *, B, b, off, d, version, dtype="bf16", flags=0, ld_img=None, ld_txt=None, N=900, tau=0.07,
             eps=1e-6, rho=6.5, gamma=0.6, seed=1, gathered=False):
    ld_img, ld_txt = ld_img or d, ld_txt or d
    rng = np.random.default_rng(seed)
    img, txt = make_embeddings(seed + 41, B, d, 0.5, dtype)
    idx = draw_indices(seed + 42, b, N)
    u0i = np.where(rng.random(N) < 0.5, 0.0, rng.uniform(0.05, 2.0, N)).astype(np.float32)
    u0t = np.where(rng.random(N) < 0.5, 0.0, rng.uniform(0.05, 2.0, N)).astype(np.float32)
    t_img = rng.uniform(0.05, 0.1, N).astype(np.float32)
    t_txt = rng.uniform(0.05, 0.1, N).astype(np.float32)
    glob = None
    if gathered:       # u^{t+1} and temperatures of every global row as other workers would have sent them
        glob = dict(u_img=rng.uniform(0.05, 2.0, B).astype(np.float32), u_txt=rng.uniform(0.05, 2.0, B).astype(np.float32),
                    tau_img=rng.uniform(0.05, 0.1, B).astype(np.float32), tau_txt=rng.uniform(0.05, 0.1, B).astype(np.float32))
        flags |= fc.GATHERED_STATE

    def matrix(x, ld):            # row stride ld, NaN in the padding, no padding behind the last row
        full = np.full((B, ld), np.nan, np.float32)
        full[:, :d] = x
        flat = full.reshape(-1)[: (B - 1) * ld + d]
        return bf16_bits(flat) if dtype == "bf16" else flat

    fin, fout = str(tmp_path / "case.in"), str(tmp_path / "case.out")
    with open(fin, "wb") as f:
        np.array([version, fc.BF16 if dtype == "bf16" else fc.F32, flags, B, b, off, d, ld_img, ld_txt, N, 1,
                  1 if gathered else 0], np.int64).tofile(f)
        np.array([gamma, eps, rho, tau, 1.0 / N], np.float32).tofile(f)
        matrix(img, ld_img).tofile(f)
        matrix(txt, ld_txt).tofile(f)
        idx.astype(np.int64).tofile(f)
        u0i.tofile(f)
        u0t.tofile(f)
        if version == V2:
            t_img.tofile(f)
            t_txt.tofile(f)
        if gathered:
            glob["u_img"].tofile(f)
            glob["u_txt"].tofile(f)
            if version == V2:
                glob["tau_img"].tofile(f)
                glob["tau_txt"].tofile(f)
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0", TSAN_OPTIONS="report_thread_leaks=0")
    if SANITIZER == "memory":
        env["EMU_UNINIT"] = "1"
    r = subprocess.run([exe, fin, fout], capture_output=True, text=True, timeout=600, env=env)
    assert r.returncode == 0 and "Sanitizer" not in r.stderr, \
        "the CPU build of the kernels failed (sanitizer report below)\n" + r.stderr[:6000]
    out = np.fromfile(fout, np.float32)
    fields = [("d_img", b * d), ("d_txt", b * d), ("loss", 1)]
    if version in (V0, V3):
        fields.append(("d_tau", 1))
    if version == V2:
        fields += [("d_tau_img", b), ("d_tau_txt", b)]
    fields += [("g_img", b), ("g_txt", b), ("u_new_img", b), ("u_new_txt", b), ("u_img", N), ("u_txt", N)]
    got, p = {}, 0
    for k, n in fields:
        got[k] = out[p:p + n].astype(np.float64)
        p += n
    assert p == out.size
    ui, ut = u0i.astype(np.float64), u0t.astype(np.float64)
    kw = {}
    if gathered:
        kw = dict(u_glob_img=glob["u_img"].astype(np.float64), u_glob_txt=glob["u_txt"].astype(np.float64))
        if version == V2:
            kw.update(tau_glob_img=glob["tau_img"].astype(np.float64), tau_glob_txt=glob["tau_txt"].astype(np.float64))
    want = fcco_step(img.astype(np.float64), txt.astype(np.float64), off, b, idx, ui, ut, version=version, gamma=gamma,
                     eps=eps, rho=rho, tau=float(np.float32(tau)), tau_img=t_img.astype(np.float64),
                     tau_txt=t_txt.astype(np.float64), tau_grad_scale=1.0 / N, **kw)
    tol = 2e-2 if dtype == "bf16" else 1e-5
    errs = {}
    for k in ("d_img", "d_txt"):
        errs[k] = np.max(np.abs(got[k].reshape(b, d) - want[k])) / np.max(np.abs(want[k]))
    for k in ("g_img", "g_txt", "u_new_img", "u_new_txt"):
        errs[k] = np.max(np.abs(got[k] - want[k]) / np.abs(want[k]))
    errs["loss"] = abs(got["loss"][0] - want["loss"]) / want["loss_abs"]
    if version in (V0, V3):
        errs["d_tau"] = abs(got["d_tau"][0] - want["d_tau"]) / want["d_tau_abs"]
    if version == V2:
        for k in ("d_tau_img", "d_tau_txt"):
            errs[k] = np.max(np.abs(got[k] - want[k])) / np.max(np.abs(want[k]))
    # the state: the oracle's arrays after the step, everywhere (untouched entries bit for bit)
    mask = np.ones(N, bool)
    mask[idx] = False
    assert np.array_equal(got["u_img"][mask], u0i[mask].astype(np.float64))
    assert np.array_equal(got["u_txt"][mask], u0t[mask].astype(np.float64))
    errs["u_img"] = np.max(np.abs(got["u_img"][idx] - ui[idx]) / ui[idx])
    errs["u_txt"] = np.max(np.abs(got["u_txt"][idx] - ut[idx]) / ut[idx])
    bad = {k: v for k, v in errs.items() if not v <= tol}
    assert not bad, bad


CASES = [
    # fp32 accuracy path
    dict(B=37, b=11, off=13, d=19, version=V2, dtype="f32", ld_img=23),
    # MFMA path, every tile ragged: guarded strip tiles on the ring (rows replaced by the last one), ragged last stage,
    # contraction with a guarded tail, fused state phase in the fold; padding between the rows of one side
    dict(B=300, b=140, off=100, d=72, version=V3, ld_img=80, flags=fc.TILES_256),
    dict(B=40, b=40, off=0, d=16, version=V0, flags=fc.TILES_256),
    # whole tiles: the persistent eight-wave strip kernel and the contraction's ring, next to a ragged anchor tile
    dict(B=512, b=300, off=212, d=128, version=V2, flags=fc.TILES_256),
    # the whole batch local, similarity matrix formed once on ragged tiles (column pass of the guarded kernel)
    dict(B=300, b=300, off=0, d=72, version=V2, flags=fc.SINGLE_PASS),
    # ... and on whole tiles (column pass of the persistent kernel)
    dict(B=512, b=512, off=0, d=128, version=V3, flags=fc.SINGLE_PASS),
    # contrast side over every global anchor (second strip, remote fold)
    dict(B=300, b=100, off=50, d=72, version=V2, gathered=True),
    # the library's own choice for a small batch: 128 x 128 tiles
    # 128 x 128 tiles (opt-in): ragged everywhere with a guarded last stage; whole stages on the ring with rows replaced;
    # the whole batch local with a width below one stage; several splits with the finalize kernel
    dict(B=300, b=140, off=100, d=72, version=V3, ld_txt=80),
    dict(B=512, b=300, off=212, d=128, version=V2, flags=fc.TILES_128),
    dict(B=257, b=257, off=0, d=8, version=V0, flags=fc.TILES_128),
    dict(B=5120, b=64, off=640, d=64, version=V1, flags=fc.TILES_128),
    # fine tiles (opt-in): one split with the output tiles finished in place, and several splits with the finalize kernel
    dict(B=300, b=140, off=100, d=72, version=V3, flags=fc.FINE_TILES, ld_txt=80),
    dict(B=5120, b=64, off=640, d=64, version=V1, flags=fc.FINE_TILES),
]


@pytest.mark.parametrize("case", CASES, ids=lambda c: "-".join("%s%s" % (k, v) for k, v in c.items()))
def test_step_of_the_host_built_kernels_matches_the_oracle_under_asan(emu_step, tmp_path, case):
    run_case(emu_step, tmp_path, **case)


@pytest.mark.parametrize("seed", range(8))
def test_random_small_shapes_on_the_host_built_kernels(emu_step, tmp_path, seed):
    """Shapes, strides, version and path drawn at random (seeded): B up to 300, any b and off, widths of 8 .. 320 that are
    no whole stages, padded rows; tile size asked for or left to the library, fine tiles, single pass, gathered state."""
    import random
    rng = random.Random(1000 + seed)
    B = rng.choice([rng.randint(2, 40), rng.randint(41, 300), 256])
    full = rng.random() < 0.3
    b = B if full else rng.randint(1, B)
    off = 0 if full else rng.randint(0, B - b)
    d = 8 * rng.choice([1, 2, 3, 4, 8, 9, 16, 17, 24, 32, 33, 40])
    path = ["256", "128", "auto", "fine", "single", "gathered", "128", "256"][seed]
    flags = {"256": fc.TILES_256, "128": fc.TILES_128, "auto": 0, "fine": fc.FINE_TILES, "single": fc.SINGLE_PASS,
             "gathered": 0}[path]
    if path == "single":
        b, off = B, 0
    run_case(emu_step, tmp_path, B=B, b=b, off=off, d=d, version=rng.randint(0, 3), flags=flags,
             N=max(b, 50) + rng.randint(0, 500), ld_img=d + 8 * rng.randint(0, 2), ld_txt=d + 8 * rng.randint(0, 2),
             seed=77 + seed, gathered=(path == "gathered"))


# ------------------------------------------------------------------ the step with the temperature update fused in
UPD = dict(lr=2e-3, step=3, beta1=0.9, beta2=0.98, eps=1e-8, tau_min=0.02, lr_drop_below=0.06, lr_drop_factor=1.0 / 3.0)


@pytest.mark.parametrize("case", [
    # V2 on records {u_1, tau_1, m_1, v_1, u_2, tau_2, m_2, v_2} that the state kernel moves as 16-byte words per side
    dict(B=300, b=140, off=100, d=72, version=V2, optimizer=ADAMW, stride=8, flags=fc.TILES_256),
    # ... records with four floats of padding that must stay untouched; the state phase inside the fold (small tiles)
    dict(B=300, b=140, off=100, d=72, version=V2, optimizer=ADAMW, stride=12),
    # dense arrays, field by field
    dict(B=40, b=40, off=0, d=16, version=V2, optimizer=LION, stride=1),
    # the global temperature stepped by a kernel of its own once its gradient is complete
    dict(B=300, b=140, off=100, d=72, version=V3, optimizer=ADAMW, stride=1),
], ids=lambda c: "-".join("%s%s" % (k, v) for k, v in c.items()))
def test_step_with_temperature_update_of_the_host_built_kernels(emu_step, tmp_path, case):
    """fastclip_step_update_tau: every output of the step, the state, and the temperatures with their moments after
    Proc. temperature_update, against the oracle's step followed by its temperature update."""
    B, b, off, d, version, S = case["B"], case["b"], case["off"], case["d"], case["version"], case["stride"]
    N, gamma, eps, rho, tau = max(700, b + 100), 0.6, 1e-6, 6.5, 0.07
    rng = np.random.default_rng(5)
    img, txt = make_embeddings(51, B, d, 0.5, "bf16")
    idx = draw_indices(52, b, N)
    f32 = lambda a: np.asarray(a, np.float32)
    st = dict(u_img=f32(np.where(rng.random(N) < 0.5, 0.0, rng.uniform(0.05, 2.0, N))),
              u_txt=f32(np.where(rng.random(N) < 0.5, 0.0, rng.uniform(0.05, 2.0, N))),
              tau_img=f32(rng.uniform(0.04, 0.1, N)), tau_txt=f32(rng.uniform(0.04, 0.1, N)),
              m_img=f32(rng.normal(0, 0.1, N)), v_img=f32(rng.uniform(0.0, 0.05, N)),
              m_txt=f32(rng.normal(0, 0.1, N)), v_txt=f32(rng.uniform(0.0, 0.05, N)))
    m0, v0 = np.float32(0.03), np.float32(0.002)
    fin, fout = str(tmp_path / "case.in"), str(tmp_path / "case.out")
    with open(fin, "wb") as f:
        np.array([version, fc.BF16, case.get("flags", 0), B, b, off, d, d, d, N, S, 0], np.int64).tofile(f)
        np.array([gamma, eps, rho, tau, 1.0 / N], np.float32).tofile(f)
        bf16_bits(img).tofile(f)
        bf16_bits(txt).tofile(f)
        idx.astype(np.int64).tofile(f)
        st["u_img"].tofile(f)
        st["u_txt"].tofile(f)
        if version == V2:
            st["tau_img"].tofile(f)
            st["tau_txt"].tofile(f)
        np.array([case["optimizer"], UPD["step"]], np.int64).tofile(f)
        np.array([UPD["lr"], UPD["beta1"], UPD["beta2"], UPD["eps"], UPD["tau_min"], UPD["lr_drop_below"],
                  UPD["lr_drop_factor"]], np.float32).tofile(f)
        if version == V2:
            for k in ("m_img", "v_img", "m_txt", "v_txt"):
                st[k].tofile(f)
        else:
            np.array([m0], np.float32).tofile(f)
            np.array([v0], np.float32).tofile(f)
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0", TSAN_OPTIONS="report_thread_leaks=0")
    r = subprocess.run([emu_step, fin, fout, "tau"], capture_output=True, text=True, timeout=600, env=env)
    assert r.returncode == 0 and "Sanitizer" not in r.stderr, r.stderr[:6000]
    out = np.fromfile(fout, np.float32).astype(np.float64)
    fields = [("d_img", b * d), ("d_txt", b * d), ("loss", 1)]
    fields += [("d_tau", 1)] if version != V2 else [("d_tau_img", b), ("d_tau_txt", b)]
    fields += [("g_img", b), ("g_txt", b), ("u_new_img", b), ("u_new_txt", b), ("u_img", N), ("u_txt", N)]
    fields += [(k, N) for k in ("tau_img", "tau_txt", "m_img", "v_img", "m_txt", "v_txt")] if version == V2 else \
              [("tau", 1), ("m", 1), ("v", 1)]
    got, p = {}, 0
    for k, n in fields:
        got[k] = out[p:p + n]
        p += n
    assert p == out.size
    # the oracle: the step with the temperatures of before the call, then the temperature update from its gradients
    w = {k: v.astype(np.float64) for k, v in st.items()}
    want = fcco_step(img.astype(np.float64), txt.astype(np.float64), off, b, idx, w["u_img"], w["u_txt"], version=version,
                     gamma=gamma, eps=eps, rho=rho, tau=float(np.float32(tau)), tau_img=w["tau_img"].copy(),
                     tau_txt=w["tau_txt"].copy(), tau_grad_scale=1.0 / N)
    kw = {k: (float(np.float32(v)) if isinstance(v, float) else v) for k, v in UPD.items()}
    if version == V2:
        temperature_update(V2, want, optimizer=case["optimizer"], tau_img=w["tau_img"], tau_txt=w["tau_txt"], idx=idx,
                           m_img=w["m_img"], v_img=w["v_img"], m_txt=w["m_txt"], v_txt=w["v_txt"], **kw)
        for k in ("tau_img", "tau_txt", "m_img", "v_img", "m_txt", "v_txt"):
            if case["optimizer"] == LION and k.startswith("v_"):
                assert np.array_equal(got[k], st[k].astype(np.float64))          # Lion keeps no second moment
                continue
            scale = np.max(np.abs(w[k]))
            assert np.max(np.abs(got[k] - w[k])) <= 2e-2 * scale, k
            mask = np.ones(N, bool)
            mask[idx] = False
            assert np.array_equal(got[k][mask], st[k][mask].astype(np.float64)), k    # other samples untouched
    else:
        t_new, m_new, v_new = temperature_update(version, want, optimizer=case["optimizer"], tau=float(np.float32(tau)),
                                                 m=float(m0), v=float(v0), **kw)
        assert got["tau"][0] == pytest.approx(t_new, rel=1e-4)
        assert got["m"][0] == pytest.approx(m_new, rel=2e-2) and got["v"][0] == pytest.approx(v_new, rel=4e-2)
    for k in ("d_img", "d_txt"):
        assert np.max(np.abs(got[k].reshape(b, d) - want[k])) <= 2e-2 * np.max(np.abs(want[k])), k
    for k in ("g_img", "g_txt", "u_new_img", "u_new_txt"):
        assert np.max(np.abs(got[k] - want[k]) / np.abs(want[k])) <= 2e-2, k
    assert np.max(np.abs(got["u_img"] - w["u_img"])) <= 2e-2 * np.max(w["u_img"])
    assert np.max(np.abs(got["u_txt"] - w["u_txt"])) <= 2e-2 * np.max(w["u_txt"])


# ------------------------------------------------------------------ the small entry points
@pytest.mark.parametrize("b,d,n", [(37, 19, 300), (5, 4104, 2), (130, 72, 1), (1, 1, 1000)])
def test_small_entry_points_of_the_host_built_kernels(emu_step, tmp_path, b, d, n):
    """fastclip_normalize_rows (a wavefront per row, padded rows on both sides), fastclip_check_indices (hash table on
    the device; distinct indices pass, a repeated one is reported), fastclip_state_update (Eq. 1 alone)."""
    rng = np.random.default_rng(b + d)
    ld_raw, ld_unit, N = d + 3, d + 5, 4 * n + 7
    raw = np.full((b, ld_raw), np.nan, np.float32)
    raw[:, :d] = rng.normal(0, 1, (b, d)) * rng.uniform(0.1, 30.0, (b, 1))
    idx = draw_indices(9, n, N)
    sums = [rng.uniform(1.0, 50.0, n).astype(np.float32) for _ in range(2)]
    u0 = [np.where(rng.random(N) < 0.5, 0.0, rng.uniform(0.05, 2.0, N)).astype(np.float32) for _ in range(2)]
    gamma, M = np.float32(0.3), np.float32(77.0)
    fin, fout = str(tmp_path / "misc.in"), str(tmp_path / "misc.out")
    with open(fin, "wb") as f:
        np.array([b, d, ld_raw, ld_unit, N, n], np.int64).tofile(f)
        np.array([gamma, M], np.float32).tofile(f)
        raw.reshape(-1)[: (b - 1) * ld_raw + d].tofile(f)
        idx.astype(np.int64).tofile(f)
        for a in sums + u0:
            a.tofile(f)
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0", TSAN_OPTIONS="report_thread_leaks=0")
    r = subprocess.run([emu_step, "misc", fin, fout], capture_output=True, text=True, timeout=600, env=env)
    assert r.returncode == 0 and "Sanitizer" not in r.stderr, r.stderr[:6000]
    blob = open(fout, "rb").read()
    n_unit = (b - 1) * ld_unit + d
    norm = np.frombuffer(blob, np.float32, b, 0).astype(np.float64)
    bits = np.frombuffer(blob, np.uint16, n_unit, 4 * b)
    st = np.frombuffer(blob, np.int32, 2, 4 * b + 2 * n_unit)
    rest = np.frombuffer(blob, np.float32, 2 * N + 2 * n, 4 * b + 2 * n_unit + 8).astype(np.float64)
    want_unit, want_norm = normalize_rows(raw[:, :d])
    assert np.max(np.abs(norm - want_norm) / want_norm) <= 1e-6
    full = np.zeros(b * ld_unit, np.uint16)
    full[:n_unit] = bits
    unit = (full.reshape(b, ld_unit)[:, :d].astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    assert np.max(np.abs(unit - want_unit)) <= 2.0 ** -8                       # one rounding to bf16 of values <= 1
    assert st[0] == fc.OK and st[1] == (fc.ERR_INDEX if n > 1 else fc.OK)
    u_img, u_txt, new_img, new_txt = rest[:N], rest[N:2 * N], rest[2 * N:2 * N + n], rest[2 * N + n:]
    for got, got_new, u_before, s_ in ((u_img, new_img, u0[0], sums[0]), (u_txt, new_txt, u0[1], sums[1])):
        want = u_before.astype(np.float64)
        new = ema_update(want, idx, s_.astype(np.float64) / float(M), float(gamma))
        assert np.max(np.abs(got - want) / np.maximum(want, 1e-30)) <= 1e-6
        assert np.max(np.abs(got_new - new) / new) <= 1e-6
