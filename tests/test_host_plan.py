"""Host-side logic of libfbx without a GPU: the library loads, exports what the
header declares, parses and layers specs like the oracle does, and reports
errors through the C ABI."""
import ctypes
import os
import random
import re

import pytest

from oracle import fbx_oracle as O
from paper_2210_07768_amd import binding as B
from paper_2210_07768_amd import workloads as W
from helpers import BAD_SPECS, FRAMING_SPEC, random_dag

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    hdr = open(os.path.join(ROOT, "include", "fbx.h")).read()
    declared = set(re.findall(r"\b(fbx_[a-z_]+)\s*\(", hdr))
    assert declared == set(B.EXPORTS)
    L = ctypes.CDLL(B.LIB_PATH)
    for name in declared:
        assert hasattr(L, name), name


@pytest.mark.parametrize("name", sorted(BAD_SPECS))
def test_plan_create_rejects_bad_specs(name):
    with pytest.raises(B.FbxError) as e:
        B.Plan(BAD_SPECS[name])
    assert e.value.status == B.E_SPEC
    assert "line" in str(e.value) or "spec" in str(e.value)


def test_plan_create_null_arguments():
    L = B.lib()
    assert L.fbx_plan_create(None, 0, None) == B.E_ARG
    L.fbx_plan_destroy(None)  # NULL is fine
    assert L.fbx_status_str(B.E_NOMEM).decode() == "workspace too small"


@pytest.mark.parametrize("cfg", [1, 2, 3, 4, 5])
def test_layers_and_arity_match_oracle_on_configs(cfg):
    w = W.get(cfg, 8)
    p = B.Plan(w.spec)
    n_ops, n_layers, layers, arity = p.info()
    o_layers, o_arity = O.spec_layers(w.spec)
    assert n_ops == w.n_ops == len(o_layers)
    assert n_layers == w.n_layers == max(o_layers)
    assert layers == o_layers
    assert arity == o_arity
    p.close()


def test_layer_rule_properties_on_random_dags():
    # Section 4, "Scheduling": roots in layer 1, every other operator one below its
    # deepest input, hence every edge goes from a lower to a strictly higher layer.
    rng = random.Random(11)
    for _ in range(50):
        spec, ids, deps = random_dag(rng, rng.randrange(1, 8), rng.randrange(0, 25))
        p = B.Plan(spec)
        _, n_layers, layers, arity = p.info()
        layer = dict(zip(ids, layers))
        for op, ins in deps.items():
            if not ins:
                assert layer[op] == 1
            else:
                assert layer[op] == 1 + max(layer[i] for i in ins)
                assert all(layer[i] < layer[op] for i in ins)
        assert n_layers == max(layers)
        o_layers, o_arity = O.spec_layers(spec)
        assert layers == o_layers and arity == o_arity
        p.close()


def test_options_and_calls_without_workspace():
    p = B.Plan(FRAMING_SPEC)
    p.set_option("fused", 1)
    p.set_option("profile", 0)
    for key, val in (("profile", 7), ("fused", 2), ("nonsense", 1)):
        with pytest.raises(B.FbxError) as e:
            p.set_option(key, val)
        assert e.value.status == B.E_ARG
    assert p.workspace_hint(1000, 10) > 0
    # no workspace yet: rejected on the host before anything touches a GPU
    with pytest.raises(B.FbxError) as e:
        p.extract_raw(0, 0, 1, 0)
    assert e.value.status == B.E_ARG
    res = B.Result()
    assert B.lib().fbx_extract(p._h, None, 0, None, 0, None, ctypes.byref(res)) == B.E_ARG
    p.close()


def test_compile_option_and_counters_on_the_host():
    p = B.Plan(FRAMING_SPEC)
    assert p.compiled() == (0, 0.0)
    p.set_option("compile", 1)
    p.set_option("compile", 0)
    with pytest.raises(B.FbxError) as e:
        p.set_option("compile", 2)
    assert e.value.status == B.E_ARG
    assert p.compiled() == (0, 0.0)       # nothing is compiled before a call needs it
    p.close()


def test_tile_kernel_source_compiles_for_a_plan_with_the_run_time_compiler():
    """What plan option compile=1 does on the GPU machine, as far as it goes without a GPU: the tile
    kernel's source, with a plan's numbers defined as literals the way fbx_jit.cpp writes them, goes
    through the HIP run-time compilation library for gfx950 (host-only code must stay behind its
    guards, the three modes must build, the kernels must carry the expected names)."""
    try:
        rtc = ctypes.CDLL("libhiprtc.so")
    except OSError:
        try:
            rtc = ctypes.CDLL("/opt/rocm/lib/libhiprtc.so")
        except OSError:
            pytest.skip("no run-time compilation library here")
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    csrc = os.path.join(root, "paper_2210_07768_amd", "csrc")
    # the texts the library itself writes for the largest benchmark workload: the three launch modes
    # on its usual tiles, and the writing kernel on tiles of 64 records with its single-sign operators
    # as straight-line code generated for the plan (one case per operator)
    w = W.get(5)
    texts = []
    plan = B.Plan(w.spec)
    plan.set_option("compile", 1)
    for mode in (0, 1, 2):
        texts.append((mode, plan.kernel_source(787 * w.n_records, w.n_records, mode)))
    assert "P.log2T = 5u;" in texts[0][1] and "#define FBX_LANE_OPS 0" in texts[0][1]
    for k, v in {"tile_log2": 6, "lds_budget": 160 * 1024, "tile_threads": 1024, "lane_ops": 2}.items():
        plan.set_option(k, v)
    texts.append((1, plan.kernel_source(787 * w.n_records, w.n_records, 1)))
    assert "P.log2T = 6u;" in texts[-1][1] and "#define FBX_TILE_THREADS 1024" in texts[-1][1]
    assert texts[-1][1].count("lane_hash1(") == 88 and texts[-1][1].count("lane_bucket1(") == 8 and texts[-1][1].count("lane_x11(") == 60
    plan.close()
    clang_inc = None
    base = os.path.join(os.environ.get("ROCM_PATH", "/opt/rocm"), "lib", "llvm", "lib", "clang")
    for v in sorted(os.listdir(base)) if os.path.isdir(base) else []:
        if os.path.exists(os.path.join(base, v, "include", "stddef.h")):
            clang_inc = os.path.join(base, v, "include")
    if clang_inc is None:
        pytest.skip("the compiler's headers are not installed here")
    for mode, text in texts:
        text = text.encode()
        prog = ctypes.c_void_p()
        assert rtc.hiprtcCreateProgram(ctypes.byref(prog), text, b"fbx_tile_fixed.hip", 0, None, None) == 0
        opts = [o.encode() for o in ("--offload-arch=gfx950", "-O3", "-std=c++17", "-I" + csrc, "-I" + os.path.join(root, "include"),
                                      "-I" + os.path.join(os.environ.get("ROCM_PATH", "/opt/rocm"), "include"), "-I" + clang_inc,
                                      "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
                                      "-mllvm", "-amdgpu-atomic-optimizer-strategy=None")]
        rc = rtc.hiprtcCompileProgram(prog, len(opts), (ctypes.c_char_p * len(opts))(*opts))
        n = ctypes.c_size_t()
        rtc.hiprtcGetProgramLogSize(prog, ctypes.byref(n))
        log = ctypes.create_string_buffer(max(n.value, 1))
        rtc.hiprtcGetProgramLog(prog, log)
        assert rc == 0, log.value.decode()[:2000]
        rtc.hiprtcGetCodeSize(prog, ctypes.byref(n))
        code = ctypes.create_string_buffer(n.value)
        assert rtc.hiprtcGetCode(prog, code) == 0
        assert f"fbx_tile_fixed_{mode}".encode() in code.raw and n.value > 10000
        rtc.hiprtcDestroyProgram(ctypes.byref(prog))


def test_fixed_arity_beyond_the_sign_limit_is_a_spec_error():
    """Concatenating an operator with itself doubles its fixed arity: 25 doublings (2^25 signs per
    record) are accepted, the 26th reaches the per-record sign limit and the spec is refused."""
    def spec(doublings):
        lines = ["fbx 1", "fields 1", "op c0 hash slot=0 seed=1 emit=0 field=0 multi=0"]
        for k in range(1, doublings + 1):
            lines.append(f"op c{k} concat slot={k} emit={1 if k == doublings else 0} a=c{k - 1} b=c{k - 1}")
        return "\n".join(lines) + "\n"
    plan = B.Plan(spec(25))
    assert plan.info()[3][-1] == 1 << 25
    plan.close()
    with pytest.raises(B.FbxError) as e:
        B.Plan(spec(26))
    assert e.value.status == B.E_SPEC and "2^26" in str(e.value)


def test_rows_that_follow_other_rows_are_found():
    """The planner marks ragged operators whose count per record is scale * (an earlier ragged operator's) + add:
    the kernel text compiled for the plan carries their number."""
    import re
    from helpers import FOLLOW_SPEC
    plan = B.Plan(FOLLOW_SPEC)
    text = plan.kernel_source(100_000, 1000, 2)
    assert re.search(r"P\.n_ragged = 12u;", text) and re.search(r"P\.n_alias = 8u;", text)
    plan.close()
    w = W.get(5, 1000)
    plan = B.Plan(w.spec)
    assert re.search(r"P\.n_alias = 4u;", plan.kernel_source(787_000, 1000, 2))  # the four crosses of a single sign with a list
    plan.close()
