"""Spec texts and hand-built records shared by the CPU and GPU tests."""

FRAMING_SPEC = ("fbx 1\nfields 4\n"
                "# comment line\n"
                "op a hash slot=0 seed=3 emit=1 field=0 multi=0\n"
                "op b hash slot=1 seed=4 emit=1 field=1 multi=1\n"
                "op c bucket slot=2 seed=5 emit=1 field=2 multi=1 bounds=0,1000000,2500000\n"
                "op d ngram slot=3 seed=6 emit=1 field=3 n=3\n"
                "op e filter slot=4 seed=7 emit=1 field=1 multi=1 prefix=78\n"
                "op f filter slot=5 seed=8 emit=1 field=0 multi=0 prefix=\n"
                "op g cross slot=6 seed=9 emit=1 a=b b=c\n"
                "op h concat slot=7 emit=1 a=g b=a\n"
                "op i cross slot=8 seed=10 emit=1 a=a b=a\n"
                "op j hash slot=9 seed=0 emit=0 field=3 multi=0\n"
                "op k concat slot=10 emit=1 a=j b=j\n")



FRAMING_RECORDS = [
    b"ab\tx,y,,z\t1.5,-2,abc\thello world\n",   # plain
    b"ab\tx,y,,z\t1.5\thello world",             # no trailing newline
    b"only\n",                                   # missing fields -> empty strings
    b"\n",                                       # empty record (all fields empty)
    b"",                                         # zero-length record
    b"\t\t\t\n",                                 # all fields present and empty
    b"a,b\txa,xb,x,,ax\t3\tab\textra\tfields\n", # extra fields ignored, n-gram shorter than n
    b"q\t,\t,\tabc\n",                           # lone commas -> two empty items
    b"w\tx\t2.5\tabcd\n\n",                      # only ONE trailing newline is dropped
]

BAD_SPECS = {
    "no header": "fields 2\n",
    "bad version": "fbx 2\nfields 2\n",
    "no fields": "fbx 1\n",
    "zero fields": "fbx 1\nfields 0\n",
    "unknown kind": "fbx 1\nfields 2\nop a frob slot=0 seed=0 emit=1 field=0\n",
    "unknown key": "fbx 1\nfields 2\nop a hash slot=0 seed=0 emit=1 field=0 multi=0 zz=1\n",
    "missing key": "fbx 1\nfields 2\nop a hash slot=0 seed=0 emit=1 field=0\n",
    "repeated key": "fbx 1\nfields 2\nop a hash slot=0 slot=1 seed=0 emit=1 field=0 multi=0\n",
    "field out of range": "fbx 1\nfields 2\nop a hash slot=0 seed=0 emit=1 field=2 multi=0\n",
    "duplicate id": "fbx 1\nfields 2\nop a hash slot=0 seed=0 emit=1 field=0 multi=0\n"
                    "op a hash slot=1 seed=0 emit=1 field=0 multi=0\n",
    "forward reference": "fbx 1\nfields 2\nop x cross slot=0 seed=0 emit=1 a=a b=a\n"
                         "op a hash slot=1 seed=0 emit=1 field=0 multi=0\n",
    "self reference": "fbx 1\nfields 2\nop x cross slot=0 seed=0 emit=1 a=x b=x\n",
    "unsorted bounds": "fbx 1\nfields 2\nop a bucket slot=0 seed=0 emit=1 field=0 multi=0 bounds=3,2\n",
    "bad bound": "fbx 1\nfields 2\nop a bucket slot=0 seed=0 emit=1 field=0 multi=0 bounds=3,,4\n",
    "duplicate emitted slot": "fbx 1\nfields 2\nop a hash slot=0 seed=0 emit=1 field=0 multi=0\n"
                              "op b hash slot=0 seed=1 emit=1 field=1 multi=0\n",
    "odd hex prefix": "fbx 1\nfields 2\nop a filter slot=0 seed=0 emit=1 field=0 multi=0 prefix=abc\n",
    "ngram width": "fbx 1\nfields 2\nop a ngram slot=0 seed=0 emit=1 field=0 n=9\n",
    "seed on concat": "fbx 1\nfields 2\nop a hash slot=0 seed=0 emit=1 field=0 multi=0\n"
                      "op c concat slot=1 seed=3 emit=1 a=a b=a\n",
    "seed too large": "fbx 1\nfields 2\nop a hash slot=0 seed=18446744073709551616 emit=1 field=0 multi=0\n",
}


def random_dag(rng, n_roots, n_rest):
    """A random operator DAG over four fields: (spec text, operator ids in spec order, inputs of each)."""
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


# Ragged operators of later layers whose count per record follows from one earlier ragged operator's
# (eight of them) and two that do not (a product of two lists, a concat over two different lists).
FOLLOW_SPEC = ("fbx 1\nfields 4\n"
        "op s0 hash slot=0 seed=1 emit=1 field=0 multi=0\n"
        "op s1 hash slot=1 seed=2 emit=1 field=1 multi=0\n"
        "op m hash slot=2 seed=3 emit=1 field=2 multi=1\n"
        "op k hash slot=3 seed=4 emit=1 field=3 multi=1\n"
        "op two concat slot=4 emit=1 a=s0 b=s1\n"            # fixed arity 2
        "op x1 cross slot=5 seed=5 emit=1 a=s0 b=m\n"        # 1 * count(m)
        "op c1 concat slot=6 emit=1 a=m b=s1\n"              # count(m) + 1
        "op mk cross slot=7 seed=6 emit=1 a=m b=k\n"         # a product: placed by its own look-back
        "op x2 cross slot=8 seed=7 emit=1 a=two b=m\n"       # 2 * count(m)
        "op c2 concat slot=9 emit=1 a=two b=k\n"             # count(k) + 2
        "op c3 concat slot=10 emit=1 a=x2 b=c1\n"            # 3 * count(m) + 1
        "op x3 cross slot=11 seed=8 emit=1 a=c1 b=two\n"     # 2 * count(m) + 2
        "op c4 concat slot=12 emit=1 a=c3 b=c2\n"            # over two different operators: its own look-back
        "op x4 cross slot=13 seed=9 emit=0 a=s1 b=c3\n"      # 3 * count(m) + 1, not emitted, read by c5
        "op c5 concat slot=14 emit=1 a=x4 b=x3\n")           # 5 * count(m) + 3
