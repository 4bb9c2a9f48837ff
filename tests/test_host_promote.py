"""Host-side implicit casting of the library (section 3.2.1) against the paper's examples, the
oracle's independent implementation and the brute-force containment rule."""
import itertools

import exactmath as X
import paper_1810_08723_amd as ocn
from oracle import binding as O
from paper_1810_08723_amd import binding as B


def test_paper_examples():
    assert ocn.promote("int8", "uint8") == "int16"
    for f in ("half", "float", "double"):
        assert ocn.promote("int64", f) == "double" and ocn.promote(f, "uint64") == "double"


def test_all_pairs_agree_with_oracle_and_brute_force():
    for a, b in itertools.product(X.ALL, X.ALL):
        r = ocn.promote(a, b)
        assert r == O.promote(a, b) == X.promote(a, b), (a, b, r)


def test_bad_dtype_is_an_error():
    assert B.lib().ocn_promote(15, 0) == B.ERR["DTYPE"]
    assert B.lib().ocn_promote(0, -1) == B.ERR["DTYPE"]
