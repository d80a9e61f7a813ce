"""Random small shapes through the host build of the kernels (tests/emu) under AddressSanitizer, every path by random
flags, each compared with the oracle:  python tests/emu/fuzz_shapes.py <seed> <count>.  Not collected by pytest (the
seeded subset in tests/test_kernels_on_cpu.py is); about 7 s per case."""
import sys, pathlib, tempfile, time, random, traceback
import os
HERE = os.path.dirname(os.path.abspath(__file__))
for p in (os.path.dirname(os.path.dirname(HERE)), os.path.dirname(HERE), HERE):
    sys.path.insert(0, p)
import build_emu, test_kernels_on_cpu as t
from paper_2407_01445_amd import binding as fc
seed0 = int(sys.argv[1]); count = int(sys.argv[2])
exe = build_emu.build()
rng = random.Random(seed0)
fails = 0
for it in range(count):
    B = rng.choice([rng.randint(2, 40), rng.randint(41, 300), rng.randint(257, 700), rng.choice([256, 512, 768])])
    full = rng.random() < 0.3
    b = B if full else rng.randint(1, B)
    off = 0 if full else rng.randint(0, B - b)
    d = 8 * rng.choice([1, 2, 3, 4, 8, 9, 16, 17, 24, 32, 33, 40])
    version = rng.randint(0, 3)
    path = rng.choice(["256", "128", "auto", "fine", "single", "gathered"])
    flags = {"256": fc.TILES_256, "128": fc.TILES_128, "auto": 0, "fine": fc.FINE_TILES,
             "single": fc.SINGLE_PASS | (fc.TILES_256 if rng.random() < 0.5 else 0), "gathered": 0}[path]
    kw = dict(B=B, b=b, off=off, d=d, version=version, flags=flags, N=max(b, 50) + rng.randint(0, 500),
              ld_img=d + 8 * rng.randint(0, 2), ld_txt=d + 8 * rng.randint(0, 2), seed=seed0 * 1000 + it,
              gathered=(path == "gathered"))
    t0 = time.time()
    try:
        t.run_case(exe, pathlib.Path(tempfile.mkdtemp()), **kw)
        print("ok   %5.1fs %s %s" % (time.time() - t0, path, kw), flush=True)
    except Exception as e:
        fails += 1
        print("FAIL %5.1fs %s %s\n%s" % (time.time() - t0, path, kw, str(e)[:3000]), flush=True)
print("done", count, "fails", fails)
