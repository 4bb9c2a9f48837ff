"""Pins for the implicit-casting result type (section 3.2.1 of the paper)."""
import itertools

import exactmath as X
from oracle import binding as O


def test_examples_printed_in_the_paper():
    """The worked examples of section 3.2.1, kept as a text fixture with their citation."""
    import os
    path = os.path.join(os.path.dirname(__file__), "golden", "promotion_examples.txt")
    rows = [ln.split() for ln in open(path) if ln.strip() and not ln.startswith("#")]
    assert len(rows) == 7
    for a, b, want in rows:
        assert O.promote(a, b) == want and O.promote(b, a) == want, (a, b)


def test_matches_brute_force_containment_over_all_pairs():
    for a, b in itertools.product(X.ALL, X.ALL):
        assert O.promote(a, b) == X.promote(a, b), (a, b)


def test_properties():
    for a, b in itertools.product(X.ALL, X.ALL):
        r = O.promote(a, b)
        assert r == O.promote(b, a)                       # symmetric
        assert O.promote(a, a) == a                       # idempotent
        assert O.promote(r, a) == r and O.promote(r, b) == r  # result absorbs its inputs
        if a in X.COMPLEX or b in X.COMPLEX:
            assert r in X.COMPLEX
        if a == "bool":
            assert r == b


def test_numpy_agrees_where_numpy_has_the_type():
    # The paper says it follows numpy for implicit casting.  numpy has no complex-half type.
    # numpy differs in one place by design: uint64 with a signed integer gives float64 there
    # too, so no exclusion is needed.
    import numpy as np
    nd = {"bool": np.bool_, "int8": np.int8, "int16": np.int16, "int32": np.int32, "int64": np.int64,
          "uint8": np.uint8, "uint16": np.uint16, "uint32": np.uint32, "uint64": np.uint64,
          "half": np.float16, "float": np.float32, "double": np.float64,
          "cfloat": np.complex64, "cdouble": np.complex128}
    back = {np.dtype(v): k for k, v in nd.items()}
    for a, b in itertools.product(nd, nd):
        want = back[np.promote_types(nd[a], nd[b])]
        assert O.promote(a, b) == want, (a, b, want)
