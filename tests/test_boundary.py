"""The C boundary: the library loads, exports every symbol sr.h declares, and rejects bad
arguments on the host (no GPU needed for any of this)."""
import ctypes
import os
import re

import numpy as np

import paper_2605_05802_amd as sr

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "sr.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(sr_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    L = sr.lib()
    names = declared_symbols()
    assert set(names) == set(sr.EXPORTS)
    for n in names:
        assert hasattr(L, n), n


def test_strerror_texts():
    assert sr.strerror(sr.SR_OK) == "ok"
    for code in (sr.SR_E_ARG, sr.SR_E_NOMEM, sr.SR_E_STATE, sr.SR_E_HIP):
        assert len(sr.strerror(code)) > 3


def test_host_side_argument_checks():
    L = sr.lib()
    lens = (ctypes.c_int * 1)(5)
    fake = ctypes.c_void_p(4096)       # never dereferenced: all of these fail validation first
    assert L.sr_gate_batch(None, 4, 8, 30, lens, 1, 0.3, None, None, None) == sr.SR_E_ARG
    assert L.sr_gate_batch(fake, 4, 1, 30, lens, 1, 0.3, None, None, None) == sr.SR_E_ARG       # G < 2
    assert L.sr_gate_batch(fake, 4, 17, 30, lens, 1, 0.3, None, None, None) == sr.SR_E_ARG      # G > 16
    assert L.sr_gate_batch(fake, 4, 8, 4, lens, 1, 0.3, None, None, None) == sr.SR_E_ARG        # prefix > stride
    assert L.sr_gate_batch(fake, 4, 8, 30, lens, 0, 0.3, None, None, None) == sr.SR_E_ARG
    assert L.sr_gate_batch(fake, 4, 8, 30, lens, 1, -0.1, None, None, None) == sr.SR_E_ARG
    big = (ctypes.c_int * 1)(33)
    assert L.sr_gate_batch(fake, 4, 8, 64, big, 1, 0.3, None, None, None) == sr.SR_E_ARG        # prefix > 32
    assert L.sr_gate_batch(fake, 0, 8, 30, lens, 1, 0.3, None, None, None) == sr.SR_OK          # empty: no launch

    h = ctypes.c_void_p()
    shape = sr.ModelShape(2, 256, 4, 2, 64, 688, 1024, 1e-6, 1e6, 1)
    opt = sr.Options(32, 256, 8, 16, 0, 1 << 24)
    assert L.sr_init(None, ctypes.byref(shape), 4, 8, 0.3, ctypes.byref(opt)) == sr.SR_E_ARG
    assert L.sr_init(ctypes.byref(h), ctypes.byref(shape), 4, 1, 0.3, ctypes.byref(opt)) == sr.SR_E_ARG
    bad = sr.ModelShape(2, 256, 4, 3, 64, 688, 1024, 1e-6, 1e6, 1)                              # 4 % 3 != 0
    assert L.sr_init(ctypes.byref(h), ctypes.byref(bad), 4, 8, 0.3, ctypes.byref(opt)) == sr.SR_E_ARG
    bad_opt = sr.Options(48, 256, 8, 16, 0, 1 << 24)
    assert L.sr_init(ctypes.byref(h), ctypes.byref(shape), 4, 8, 0.3, ctypes.byref(bad_opt)) == sr.SR_E_ARG
    assert L.sr_decode_step(None, None, None, None) == sr.SR_E_ARG
    assert L.sr_gate(None, 1, None, None, None) == sr.SR_E_ARG
    assert L.sr_retire_and_compact(None, None, None) == sr.SR_E_ARG
    L.sr_destroy(None)


def test_product_never_touches_the_checker():
    pkg = os.path.join(ROOT, "paper_2605_05802_amd")
    for dirpath, _, files in os.walk(pkg):
        if "_build" in dirpath:
            continue
        for f in files:
            if f.endswith((".py", ".hip", ".h")):
                text = open(os.path.join(dirpath, f)).read()
                assert "oracle" not in text.lower(), f
                assert "sro_" not in text, f


def test_bench_refuses_more_than_one_gpu_and_fails_loudly_without_one():
    """`bench.py --gpus 2` exits with a message before touching any device (the library runs on one GPU);
    without a GPU the default run exits non-zero instead of falling back to the CPU."""
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode != 0 and "one GPU" in (r.stderr + r.stdout)
    assert not r.stdout.strip().startswith("{")
    import torch
    if not torch.cuda.is_available():
        r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--steps", "1"], capture_output=True,
                           text=True, timeout=300)
        assert r.returncode != 0 and "no GPU" in r.stderr and not r.stdout.strip().startswith("{")
