"""CPU sanitizer runs (no GPU): the oracle's C code and the host half of the library - descriptor checks, launch
planner, workspace sizes, mask builder - are built with AddressSanitizer and UndefinedBehaviorSanitizer and driven
through pinned cases.  A memory error or undefined behaviour aborts the run and fails the test; results are also
compared with the regular builds and with values fixed by hand."""
from __future__ import annotations

import json
import os
import shutil
import subprocess
import tempfile

import numpy as np
import pytest

import oracle
import synth_inputs as si

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HERE = os.path.join(ROOT, "tests", "sanitize")
SAN = ["-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-O1", "-g"]
# the sanitizer runtime is linked into the executables; leak checking needs ptrace, which containers often refuse
RUN_ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:verify_asan_link_order=0:abort_on_error=0",
               UBSAN_OPTIONS="print_stacktrace=1:halt_on_error=1")


def _num(x):
    return " ".join(repr(float(v)) for v in np.asarray(x, dtype=np.float64).ravel())


def _int(x):
    return " ".join(str(int(v)) for v in np.asarray(x).ravel())


@pytest.fixture(scope="module")
def workdir():
    d = tempfile.mkdtemp(prefix="tv_sanitize_")
    yield d
    shutil.rmtree(d, ignore_errors=True)


def test_oracle_under_address_and_undefined_behaviour_sanitizers(workdir):
    exe = os.path.join(workdir, "oracle_san")
    subprocess.run(["gcc", "-std=c11", *SAN, "-static-libasan", os.path.join(ROOT, "oracle", "confu_oracle.c"),
                    os.path.join(HERE, "oracle_driver.c"), "-lm", "-o", exe], check=True)
    rng = np.random.default_rng(2024)
    lines, expect = [], []

    # tree attention: small trees with contemplate rows and soft-prompt slots, two head layouts
    for (T, C, P, s, Hq, Hkv, D) in [(7, 2, 5, 2, 4, 2, 8), (1, 0, 0, 0, 2, 2, 4), (12, 12, 9, 4, 6, 3, 16)]:
        nodes = si.random_tree(rng, T, 4, 3)
        if C == T:
            parent, kind, _, _ = si.interleave_contemplates_per_node(nodes)
        else:
            parent, kind, _ = si.append_contemplates_chained(nodes, C)
        M = len(parent)
        q, k, v = rng.standard_normal((M, Hq, D)), rng.standard_normal((P + M, Hkv, D)), rng.standard_normal((P + M, Hkv, D))
        lines.append(f"A {M} {Hq} {Hkv} {D} {P} {s} {0.3!r} {_int(parent)} {_int(kind)} {_num(q)} {_num(k)} {_num(v)}")
        out, lse = oracle.tree_attention(q, k, v, parent, kind, soft_len=s, scale=0.3, return_lse=True)
        expect.append(("A", np.concatenate([out.ravel(), lse.ravel()])))

    # acceptance: every rule on random small cases, and the example worked by hand in exact fractions
    def accept_case(tl, dl, token, parent, un, temp, rule, anchor):
        T, V = tl.shape
        C = 0 if anchor is None else len(anchor)
        parts = [f"C {T} {V} {C} {temp!r} {rule} {0 if dl is None else 1}", _num(tl)]
        if dl is not None:
            parts.append(_num(dl))
        parts += [_int(token), _int(parent), _num(un), _int([] if anchor is None else anchor)]
        lines.append(" ".join(parts))
        r = oracle.tree_accept(tl, dl, token, parent, un, temperature=temp, rule=rule, con_anchor=anchor)
        expect.append(("C", r))

    for rule in (oracle.RULE_GREEDY, oracle.RULE_DETERMINISTIC, oracle.RULE_DRAFT_WOR, oracle.RULE_DRAFT_WR,
                 oracle.RULE_SAMPLE_MATCH):
        for trial in range(3):
            T, V = 9, 40
            parent = si.random_tree(rng, T, 4, 3)
            tl = (rng.standard_normal((T, V)) * 2).astype(np.float32)
            dl = (0.8 * tl + 0.6 * rng.standard_normal((T, V))).astype(np.float32) \
                if rule in (oracle.RULE_DRAFT_WOR, oracle.RULE_DRAFT_WR) else None
            token = np.array([int(np.argsort(-tl[max(p, 0)])[rng.integers(0, 3)]) for p in parent], dtype=np.int32)
            un = rng.random(2 * T, dtype=np.float32)
            accept_case(tl, dl, token, parent, un, 0.0 if rule == oracle.RULE_GREEDY else 0.7, rule,
                        np.array([0, int(rng.integers(0, T))], dtype=np.int32))
    with open(os.path.join(ROOT, "tests", "golden", "accept_rational_example.json")) as f:
        g = json.load(f)
    p, q = np.array(g["p"]), np.array(g["q"])
    tl = np.tile(np.log(p).astype(np.float32), (2, 1))
    dl = np.tile(np.log(q).astype(np.float32), (2, 1))
    par = np.array([-1, 0], dtype=np.int32)
    worked = []          # (uniform of the child, expected n_accepted): the child proposes token 2, accepted iff u < 1/3
    for u1, acc in [(0.30, 1), (0.3333, 1), (0.3334, 0), (0.9, 0)]:
        accept_case(tl, dl, np.array([0, 2], np.int32), par, np.array([0.0, u1, 0.5, 0.5], np.float32), 1.0,
                    oracle.RULE_DRAFT_WOR, None)
        worked.append((len(expect) - 1, acc))
    # a malformed tree is refused, not walked
    lines.append(f"C 3 4 0 1.0 {oracle.RULE_DETERMINISTIC} 0 {_num(np.zeros(12))} 0 1 2 -1 2 1 {_num(np.zeros(6))}")
    expect.append(("C", None))

    r = subprocess.run([exe], input="\n".join(lines) + "\n", capture_output=True, text=True, env=RUN_ENV, timeout=300)
    assert r.returncode == 0, r.stderr[-4000:]
    got = r.stdout.strip().split("\n")
    assert len(got) == len(expect)
    for line, (tag, ref) in zip(got, expect):
        f = line.split()
        assert f[0] == tag
        if tag == "A":
            assert f[1] == "0"
            np.testing.assert_allclose(np.array(f[2:], dtype=np.float64), ref, rtol=1e-12, atol=1e-13)
        elif ref is None:
            assert f[1] != "0"
        else:
            assert f[1] == "0"
            vals = [int(x) for x in f[2:]]
            assert vals[:5] == [ref["n_accepted"], ref["final_token"], ref["final_kind"], ref["last_node"], ref["selected_con"]]
            assert vals[5:] == list(ref["path"])
    for idx, acc in worked:
        assert int(got[idx].split()[2]) == acc
        if not acc:      # the residual of the worked example is the point mass on token 0
            assert int(got[idx].split()[3]) == 0


def test_host_side_of_the_library_under_address_and_undefined_behaviour_sanitizers(workdir):
    import re
    from paper_2603_08899_amd import build as lib_build
    clangxx = os.path.join(os.path.dirname(lib_build.HIPCC), "..", "llvm", "bin", "clang++")
    inc = ["-I", os.path.join(ROOT, "include"), "-I", lib_build.CSRC]
    objs = []
    for src in lib_build.SOURCES:          # host code only: kernels are declared, never launched
        obj = os.path.join(workdir, src.replace(".hip", ".o"))
        subprocess.run([lib_build.HIPCC, "--cuda-host-only", "-std=c++17", *SAN, *inc, "-c",
                        os.path.join(lib_build.CSRC, src), "-o", obj], check=True, capture_output=True)
        objs.append(obj)
    # a host-only object still names the device image that a full build would embed: empty stand-ins
    undefined = subprocess.run(["nm", "-u", *objs], check=True, capture_output=True, text=True).stdout
    stubs = os.path.join(workdir, "device_image_stubs.cpp")
    with open(stubs, "w") as f:
        for sym in sorted(set(re.findall(r"__hip_fatbin_[0-9a-f]+", undefined))):
            f.write(f"extern \"C\" {{ extern const unsigned long long {sym}[16]; const unsigned long long {sym}[16] = {{0}}; }}\n")
    drv = os.path.join(workdir, "host_driver.o")
    subprocess.run([clangxx, "-std=c++17", *SAN, *inc, "-c", os.path.join(HERE, "host_driver.cpp"), "-o", drv],
                   check=True, capture_output=True)
    exe = os.path.join(workdir, "host_san")
    rocm_lib = os.path.join(os.path.dirname(lib_build.HIPCC), "..", "lib")
    subprocess.run([clangxx, "-fsanitize=address,undefined", "-static-libsan", drv, *objs, stubs, "-L", rocm_lib,
                    "-lamdhip64", f"-Wl,-rpath,{rocm_lib}", "-o", exe], check=True, capture_output=True)
    r = subprocess.run([exe], capture_output=True, text=True, env=RUN_ENV, timeout=300)
    assert r.returncode == 0, (r.stdout[-2000:], r.stderr[-4000:])
    assert "host driver: ok" in r.stdout
