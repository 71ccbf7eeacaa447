"""The oracle's C under AddressSanitizer and UndefinedBehaviorSanitizer (CPU only): the whole path
of configuration 1, the partial-macroblock case and a turned-box case run in a child process that
loads a sanitized build; any out-of-bounds access, misaligned access or signed overflow aborts it."""
import os
import subprocess
import sys
import tempfile

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

CHILD = r'''
import ctypes, sys
import numpy as np
sys.path.insert(0, sys.argv[2])
import oracle, workloads as wl
oracle._lib = ctypes.CDLL(sys.argv[1]); oracle._lib.orc_budget.restype = ctypes.c_long
cfg = wl.config(1)
frames, imp = wl.make_frames(cfg), wl.make_importance(cfg)
blob = wl.make_weights(cfg.net, 0, "fp32")
r = oracle.run_path(frames, imp, wl.make_segments(cfg), cfg.net, blob, cfg.halo, cfg.bin_size)
assert r.plan.n_bins == 9 and len(r.list) == 60
r = oracle.run_path(frames, imp, wl.make_segments(cfg), cfg.net, blob, cfg.halo, cfg.bin_size, exact_border=True)
c2 = wl.replace(cfg, width=168, height=100, n_frames=2, net=wl.Net("edsr", 4, 1, 3, 0.05))
f2, i2 = wl.make_frames(c2), wl.make_importance(c2)
i2[:, -1, :] += 5.0; i2[:, :, -1] += 5.0
r = oracle.run_path(f2, i2, np.array([[0, 2, 60]], dtype=np.uint32), c2.net, wl.make_weights(c2.net, 0, "fp32"), 5, 96)
assert r.mask[:, -1, :].all()
c3 = wl.replace(cfg, n_frames=3, width=160, height=112, importance="uniform", frac=0.5)
f3, i3 = wl.make_frames(c3), wl.make_importance(c3)
r = oracle.run_path(f3, i3, wl.make_segments(c3), c3.net, blob, 4, 64, rotate=True, sort_policy="area", conn=4, T=2)
assert r.plan.boxes[:, 5].sum() > 0
hr, sel = oracle.unpack(f3, 2, r.net_out, np.array([[0, 0, 0, 60, 60], [1, 0, 0xFFFF, 0, 0]], dtype=np.int32))
from oracle import temporal as OT
phi, nb = OT.phi(wl.make_residuals(96, 64, 2, 4, seed=1), 12, 2)
print("SANITIZED_OK", r.plan.n_bins)
'''


def test_oracle_runs_clean_under_asan_and_ubsan():
    with tempfile.TemporaryDirectory() as tmp:
        lib = os.path.join(tmp, "librh_oracle_san.so")
        subprocess.check_call(["gcc", "-O1", "-g", "-std=c11", "-Wall", "-fopenmp", "-ffp-contract=off",
                               "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer",
                               "-shared", "-fPIC", "-o", lib, os.path.join(ROOT, "oracle", "rh_oracle.c"), "-lm"])
        asan = subprocess.check_output(["gcc", "-print-file-name=libasan.so"], text=True).strip()
        env = dict(os.environ, LD_PRELOAD=asan + (" " + os.environ["LD_PRELOAD"] if os.environ.get("LD_PRELOAD") else ""),
                   ASAN_OPTIONS="detect_leaks=0:abort_on_error=1", UBSAN_OPTIONS="halt_on_error=1:print_stacktrace=1",
                   OMP_NUM_THREADS="4")
        r = subprocess.run([sys.executable, "-c", CHILD, lib, ROOT], capture_output=True, text=True, env=env, timeout=600)
        assert r.returncode == 0 and "SANITIZED_OK" in r.stdout, r.stdout[-2000:] + r.stderr[-4000:]
