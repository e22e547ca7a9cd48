"""The oracle under AddressSanitizer and UndefinedBehaviorSanitizer (host code only, no GPU).

oracle/sparseloco_oracle.c is compiled together with tests/oracle_sanitize_main.c with
-fsanitize=address,undefined (every report is fatal) and run in a subprocess over the worked example of
tests/golden/, ragged flat tensors, tiled tensors with edge tiles on both sides, kappa >= n_c, every source mode
and both quantiser modes.  Its outputs must equal those of the ordinary build byte for byte, so the run also
shows that the sanitised build computes the same thing."""
import json
import os
import struct
import subprocess

import numpy as np
import pytest

import oracle

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def build_driver(tmp_path):
    exe = str(tmp_path / "oracle_sanitize")
    cmd = ["gcc", "-O1", "-g", "-std=c99", "-ffp-contract=off", "-fno-fast-math", "-fopenmp",
           "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer",
           "-static-libasan", "-static-libubsan", "-Wall", "-Wextra",
           os.path.join(ROOT, "tests", "oracle_sanitize_main.c"), os.path.join(ROOT, "oracle", "sparseloco_oracle.c"),
           "-o", exe, "-lm"]
    subprocess.check_call(cmd)
    return exe


def make_cases():
    rng = np.random.default_rng(2024)
    cases = []

    def add(shape, geom, tiled, kappa, quant, R, mode, beta=0.95, lr=1.0, theta=None, src=None, ef=None):
        rows, cols = shape
        n = rows * cols
        theta = (rng.standard_normal(n) * 0.02).astype(np.float32) if theta is None else theta
        if src is None:
            d = [(rng.standard_t(3, n) * 1e-3).astype(np.float32) for _ in range(R)]
            if mode == 0:
                src = [(theta - x).astype(np.float32) for x in d]
            elif mode == 1:
                src = d
            else:
                src = [((x.view(np.uint32) >> 16).astype(np.uint16)) * (rng.random(n) < 0.5).astype(np.uint16) for x in d]
        ef = [(rng.standard_normal(n) * 1e-4).astype(np.float32) for _ in range(R)] if ef is None else ef
        cases.append(dict(shape=shape, geom=geom, tiled=tiled, kappa=kappa, quant=quant, R=R, mode=mode, beta=beta,
                          lr=lr, theta=theta, src=src, ef=ef))

    g = json.load(open(os.path.join(ROOT, "tests", "golden", "worked_example.json")))
    th = np.array(g["theta_outer"], np.float32)
    add((1, 8), g["chunk"], 0, g["kappa"], 1, 2, 0, theta=th,
        src=[(th - np.array(r["delta_decimal"], np.float32)).astype(np.float32) for r in g["replicas"]],
        ef=[np.array(r["ef"], np.float32) for r in g["replicas"]])
    for n in (1, 7, 4095, 4096, 4097, 3 * 4096 + 17):                      # ragged flat tensors
        add((1, n), 4096, 0, 32, 1, 3, 0)
    add((1, 2 * 4096 + 4), 4096, 0, 64, 0, 2, 1, lr=0.8)                    # identity quantiser, partial chunk of 4
    add((1, 5000), 4096, 0, 4096, 1, 2, 2)                                  # kappa >= n_c everywhere, bf16 source
    add((1, 100), 8, 0, 8, 1, 2, 1)                                         # kappa = chunk
    add((1, 100), 16, 0, 1, 1, 1, 1)                                        # kappa = 1
    for shape in ((130, 70), (64, 64), (63, 65), (200, 3), (3, 200), (1, 5000), (65, 129)):   # tiles, both edges
        add(shape, 64, 1, 32, 1, 2, 0)
    add((70, 66), 64, 1, 200, 0, 2, 2)                                      # tiles smaller than kappa, bf16
    add((9, 9), 4, 1, 3, 1, 3, 1)                                           # small tiles, many of them
    zeros = np.zeros(4096 + 10, np.float32)
    add((1, 4096 + 10), 4096, 0, 32, 1, 2, 1, theta=zeros, src=[zeros, zeros], ef=[zeros.copy(), zeros.copy()])
    return cases


def expected(case):
    """The same case through the ordinary build, single tensor."""
    shape = case["shape"]
    tiled = bool(case["tiled"])
    geo = dict(shapes=[shape], tile=case["geom"]) if tiled else dict(chunk=case["geom"])
    quant = bool(case["quant"])
    th = [case["theta"].copy()]
    out = []
    pairs, aux = [], []
    for r in range(case["R"]):
        ef = [case["ef"][r].copy()]
        if case["mode"] == 0:
            p, a = oracle.compress(ef, case["kappa"], case["beta"], theta_outer=th, theta_local=[case["src"][r]],
                                   quant=quant, **geo)
        else:
            p, a = oracle.compress(ef, case["kappa"], case["beta"], delta=[case["src"][r]], quant=quant, **geo)
        pairs.append(p), aux.append(a)
        out += [p.tobytes(), a.tobytes(), ef[0].tobytes()]
    dbar = oracle.aggregate([shape] if tiled else [shape[0] * shape[1]], pairs, aux, case["kappa"], quant=quant,
                            **({"tile": case["geom"]} if tiled else {"chunk": case["geom"]}))
    oracle.outer_update(th, dbar, case["lr"])
    out += [dbar[0].tobytes(), th[0].tobytes()]
    return b"".join(out)


def test_oracle_is_clean_under_asan_and_ubsan(tmp_path):
    exe = build_driver(tmp_path)
    cases = make_cases()
    blob = [struct.pack("<i", len(cases))]
    for c in cases:
        blob.append(struct.pack("<qqiiiiiiff", c["shape"][0], c["shape"][1], c["geom"], c["tiled"], c["kappa"],
                                c["quant"], c["R"], c["mode"], c["beta"], c["lr"]))
        blob.append(c["theta"].tobytes())
        for r in range(c["R"]):
            blob.append(np.ascontiguousarray(c["src"][r]).tobytes())
            blob.append(c["ef"][r].tobytes())
    (tmp_path / "cases.bin").write_bytes(b"".join(blob))
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0:verify_asan_link_order=0",
               UBSAN_OPTIONS="print_stacktrace=1:halt_on_error=1", OMP_NUM_THREADS="4")
    run = subprocess.run([exe, str(tmp_path / "cases.bin"), str(tmp_path / "out.bin")], capture_output=True, text=True,
                         env=env, timeout=300)
    assert run.returncode == 0, run.stdout + run.stderr
    assert "runtime error" not in run.stderr and "AddressSanitizer" not in run.stderr, run.stderr
    got = (tmp_path / "out.bin").read_bytes()
    want = b"".join(expected(c) for c in cases)
    assert len(got) == len(want)
    assert got == want, "the sanitised build computes something else"
    # the worked example is the first case: its first replica's pairs are the paper-reading's 0x1000 0x3004 0x0006
    assert got[:6] == bytes.fromhex("0010" "0430" "0600")
