"""Pins of the serialisation oracle (oracle/serialize_oracle.py) against what the paper and arithmetic fix:
hand-worked cases, the token count against the range the paper reports, decoding, exact rounding."""
import os
from fractions import Fraction

import numpy as np

from oracle import serialize_oracle as S
from paper_2604_24273_amd import synth

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "serialize_hand_cases.txt")


def read_cases(path=GOLDEN):
    cases, cur = [], None
    for line in open(path):
        line = line.rstrip("\n")
        if not line or line.startswith("#"):
            continue
        key, _, rest = line.partition(" ")
        if key == "case":
            cur = {"name": rest}
            cases.append(cur)
        elif key == "state":
            cur["state"] = np.asarray([float(t) for t in rest.split()], dtype=np.float32)
        elif key == "text":
            cur["text"] = rest
        elif key == "ids":
            cur["ids"] = [int(t) for t in rest.split()]
    return cases


def test_hand_cases():
    cases = read_cases()
    assert len(cases) >= 4
    for c in cases:
        assert S.serialize_text(c["state"]) == c["text"], c["name"]
        assert S.serialize_ids(c["state"]) == c["ids"], c["name"]


def test_token_count_is_in_the_range_the_paper_reports():
    # Sec. 5.2: MuJoCo states of 17 - 27 dimensions give 15 - 40 tokens
    for n in range(17, 28):
        s = synth.normal(5, 700 + n, (n,), 2.0)
        ids = S.serialize_ids(s)
        assert len(ids) == n + 2
        assert 15 <= len(ids) <= 40
        assert ids[0] == S.BOS_ID and ids[1] == S.STATE_ID
        assert all(S.NUM_BASE <= i < S.BYTE_BASE for i in ids[2:])
        assert max(ids) < S.VOCAB_SIZE


def test_ids_decode_back_to_the_text():
    for seed in range(20):
        s = synth.normal(6, 720 + seed, (1 + seed,), 4.0)
        assert S.detokenize(S.serialize_ids(s)).decode("ascii") == S.serialize_text(s)


def test_one_decimal_rendering_is_the_correctly_rounded_one():
    # nearest tenth of the exact value: |10 x - m| <= 1/2 in exact arithmetic, ties even; and monotone in x
    xs = np.sort(np.concatenate([synth.normal(7, 740, (2000,), 3.0), np.asarray([0.25, 0.75, -0.25, 2.5, 0.15], np.float32)]))
    prev = -10 ** 9
    for x in xs:
        m = S.tenths(x)
        if abs(float(x)) < 9.85:
            d = abs(Fraction(float(x)) * 10 - m)
            assert d <= Fraction(1, 2)
            if d == Fraction(1, 2):
                assert m % 2 == 0
        assert m >= prev
        prev = m
    assert S.tenths(np.float32("nan")) == 0 and S.tenths(np.float32("inf")) == 99 and S.tenths(np.float32("-inf")) == -99
    assert S.number_text(0) == "0.0" and S.number_text(-5) == "-0.5" and S.number_text(99) == "9.9"


def test_tokenizer_is_total_and_greedy():
    # arbitrary bytes fall back to byte tokens; a number string inside free text is still one token
    ids = S.tokenize("go north 1.5".encode("utf-8"))
    assert ids[0] == S.BOS_ID
    assert S.detokenize(ids) == b"go north 1.5"
    assert ids[-1] == S.NUM_BASE + 99 + 15                      # " 1.5"
    assert all(i >= S.BYTE_BASE for i in ids[1:-1])
    assert S.tokenize(b"") == [S.BOS_ID]
    weird = bytes(range(256))
    assert S.detokenize(S.tokenize(weird)) == weird
    # every vocabulary entry tokenises to itself
    for i, s in enumerate(S.vocabulary()):
        if i >= 1:
            assert S.tokenize(s) == [S.BOS_ID, i], (i, s)
