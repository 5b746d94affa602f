"""The CPU oracles and the library's host-side parser and planner under AddressSanitizer and
UndefinedBehaviorSanitizer: both parse untrusted spec text (hex bytes, lists of bounds, operator
ids) and record offsets with hand-written C and C++.  Stand-alone executables built with
gcc / g++ (-fsanitize=address,undefined, run-time linked statically), fed the bad specs, random
operator DAGs, the benchmark specs and hand-built records; any report fails the test."""
import os
import random
import shutil
import subprocess

import numpy as np
import pytest

from paper_2210_07768_amd import workloads as W
from helpers import BAD_SPECS, FRAMING_RECORDS, FRAMING_SPEC, random_dag
from test_clean_oracle_pins import SPEC as CLEAN_SPEC

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
FLAGS = ["-g", "-O1", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-static-libasan", "-fno-omit-frame-pointer"]
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0:exitcode=77:verify_asan_link_order=0", UBSAN_OPTIONS="print_stacktrace=1")


def _build(tmp_path, name, compiler, sources, extra=()):
    if shutil.which(compiler) is None:
        pytest.skip(f"no {compiler} here")
    exe = str(tmp_path / name)
    r = subprocess.run([compiler, *FLAGS, *extra, "-o", exe, *sources], capture_output=True, text=True)
    if r.returncode != 0 and "asan" in r.stderr.lower() and "cannot find" in r.stderr.lower():
        pytest.skip("the sanitizer run-time is not installed here")
    assert r.returncode == 0, r.stderr[-2000:]
    return exe


def _run(cmd):
    r = subprocess.run(cmd, capture_output=True, text=True, env=ENV, timeout=300)
    assert r.returncode == 0 and "runtime error" not in r.stderr and "AddressSanitizer" not in r.stderr, (cmd, r.stdout[-500:], r.stderr[-3000:])
    return r.stdout


def _write(tmp_path, stem, spec, records):
    (tmp_path / f"{stem}.spec").write_text(spec)
    (tmp_path / f"{stem}.raw").write_bytes(b"".join(records))
    np.cumsum([0] + [len(r) for r in records]).astype(np.uint64).tofile(str(tmp_path / f"{stem}.off"))
    return [str(tmp_path / f"{stem}.{ext}") for ext in ("spec", "raw", "off")]


def _cases(tmp_path):
    rng = random.Random(2)
    cases = [("framing", FRAMING_SPEC, FRAMING_RECORDS * 3)]
    for name, spec in sorted(BAD_SPECS.items()):
        cases.append((f"bad_{len(cases)}", spec, FRAMING_RECORDS))
    for k in range(12):
        spec, _, _ = random_dag(rng, rng.randrange(2, 9), rng.randrange(1, 9))
        recs = [("\t".join(",".join("abcab"[:rng.randint(0, 4)] for _ in range(rng.randint(1, 3))) for _ in range(rng.randint(0, 5)))
                 + ("\n" if i % 3 else "")).encode() for i in range(40)]
        cases.append((f"dag_{k}", spec, recs))
    for cfg, n in ((1, 64), (2, 20), (3, 50), (4, 20), (5, 30)):
        w = W.get(cfg, n)
        raw, off = w.generate()
        b = raw.tobytes()
        cases.append((w.name, w.spec, [b[int(off[i]):int(off[i + 1])] for i in range(n)]))
    cases.append(("junk", "fbx 1\nfields 3\nop \x00\xff hash slot=99999999999999999999 seed=-1 emit=2 field=1e9 multi=x\n", [b"a\tb\n"]))
    cases.append(("long_prefix", "fbx 1\nfields 1\nop a filter slot=0 seed=0 emit=1 field=0 multi=1 prefix=" + "61" * 300 + "\n", [b"a,b\n"]))
    return cases


def test_oracles_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    exe = _build(tmp_path, "oracle_driver", "gcc",
                 [os.path.join(ROOT, "oracle", "fbx_oracle.c"), os.path.join(ROOT, "oracle", "fbx_clean_oracle.c"),
                  os.path.join(ROOT, "tests", "sanitize", "oracle_driver.c")], extra=["-std=c11", "-D_GNU_SOURCE"])
    ok = 0
    for stem, spec, recs in _cases(tmp_path):
        out = _run([exe, "extract", *_write(tmp_path, stem, spec, recs)])
        ok += out.startswith("ok")
    assert ok >= 18                                   # (the framing spec, the random DAGs and the five workloads at least)
    rng = random.Random(4)
    clean_specs = [CLEAN_SPEC, "fbxclean 1\nfields 2\nfill field=0 value=\n", "fbxclean 1\nfields 70000\n", "fbxclean 1\nfields 2\nkey field=1 name=" + "6b" * 255 + "\n",
                   "fbxclean 1\nfields 2\nkeep field=9 prefix=61\n", "junk\x00\n"]
    recs = [("\t".join("".join(rng.choice("ab:;k") for _ in range(rng.randint(0, 9))) for _ in range(rng.randint(0, 5))) + "\n").encode() for _ in range(100)]
    for k, spec in enumerate(clean_specs):
        _run([exe, "clean", *_write(tmp_path, f"clean_{k}", spec, recs)])


def test_host_planner_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    csrc = os.path.join(ROOT, "paper_2210_07768_amd", "csrc")
    exe = _build(tmp_path, "plan_driver", "g++",
                 [os.path.join(csrc, "fbx_plan.cpp"), os.path.join(ROOT, "tests", "sanitize", "plan_driver.cpp")],
                 extra=["-std=c++17", "-I", csrc, "-I", os.path.join(ROOT, "include")])
    files = []
    for stem, spec, recs in _cases(tmp_path):
        files.append(_write(tmp_path, stem, spec, recs)[0])
    # arities that double until the sign limit is reached, and a very wide plan
    lines = ["fbx 1", "fields 1", "op c0 hash slot=0 seed=1 emit=0 field=0 multi=0"]
    lines += [f"op c{k} concat slot={k} emit=0 a=c{k - 1} b=c{k - 1}" for k in range(1, 40)]
    files.append(_write(tmp_path, "doubling", "\n".join(lines) + "\n", [b"a\n"])[0])
    wide = ["fbx 1", "fields 3000"] + [f"op h{k} hash slot={k} seed={k} emit=1 field={k} multi={k % 2}" for k in range(3000)]
    files.append(_write(tmp_path, "wide", "\n".join(wide) + "\n", [b"a\n"])[0])
    out = _run([exe, *files])
    assert out.count("status 0") >= 18 and "status -2" in out    # (framing, twelve random DAGs, five workloads; bad specs refused)
