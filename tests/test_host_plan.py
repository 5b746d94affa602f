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
from helpers import BAD_SPECS, FRAMING_SPEC

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


def _random_dag(rng, n_roots, n_rest):
    lines = ["fbx 1", "fields 4"]
    ids, deps = [], {}
    for i in range(n_roots):
        kind = rng.choice(["hash", "ngram", "bucket", "filter"])
        common = f"slot={i} seed={rng.getrandbits(64)} emit={rng.randrange(2)} field={rng.randrange(4)}"
        if kind == "hash":
            lines.append(f"op r{i} hash {common} multi={rng.randrange(2)}")
        elif kind == "ngram":
            lines.append(f"op r{i} ngram {common} n={rng.randrange(1, 9)}")
        elif kind == "bucket":
            b = sorted(rng.randrange(-100, 100) for _ in range(rng.randrange(0, 6)))
            lines.append(f"op r{i} bucket {common} multi={rng.randrange(2)} bounds={','.join(map(str, b))}")
        else:
            lines.append(f"op r{i} filter {common} multi={rng.randrange(2)} prefix={bytes([rng.randrange(97, 100)]).hex()}")
        ids.append(f"r{i}")
        deps[f"r{i}"] = ()
    for i in range(n_rest):
        a, b = rng.choice(ids), rng.choice(ids)
        if rng.random() < 0.5:
            lines.append(f"op n{i} cross slot={1000 + i} seed={rng.getrandbits(64)} emit=1 a={a} b={b}")
        else:
            lines.append(f"op n{i} concat slot={1000 + i} emit=1 a={a} b={b}")
        ids.append(f"n{i}")
        deps[f"n{i}"] = (a, b)
    return "\n".join(lines) + "\n", ids, deps


def test_layer_rule_properties_on_random_dags():
    # Section 4, "Scheduling": roots in layer 1, every other operator one below its
    # deepest input, hence every edge goes from a lower to a strictly higher layer.
    rng = random.Random(11)
    for _ in range(50):
        spec, ids, deps = _random_dag(rng, rng.randrange(1, 8), rng.randrange(0, 25))
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
