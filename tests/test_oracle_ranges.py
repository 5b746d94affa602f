"""The oracle run range by range on several threads is the oracle: same signs, same offsets."""
import numpy as np

from oracle import fbx_oracle as O
from paper_2210_07768_amd import workloads as W
from oracle_ranges import extract_parallel


def test_ranges_laid_end_to_end_equal_one_call():
    for cfg, n in ((2, 150), (3, 400), (4, 230), (5, 333)):
        w = W.get(cfg, n)
        raw, off = w.generate()
        want = O.extract(w.spec, raw, off)
        for workers in (1, 3, 8):
            slots, slot_ids, total, malformed = extract_parallel(w.spec, raw, off, workers=workers)
            assert list(slot_ids) == list(want.slot_ids)
            assert total == want.n_values_total and malformed == want.n_malformed_numeric
            for s in want.slot_ids:
                ov, oo, arity = want.slots[s]
                assert slots[s][2] == arity
                assert np.array_equal(slots[s][0], ov) and np.array_equal(slots[s][1], oo), (w.name, s, workers)
