"""CPU oracle for the state-to-token front end, serialize(s_t) of Sec. 3.1, Eq. 3.

TEST INFRASTRUCTURE ONLY: the plain definition the library's host-side
serialiser is checked against.  Nothing in the product path imports it, and it
imports nothing from the package.

What the paper fixes: serialize(.) turns an environment state into natural
language text that the frozen backbone reads (Sec. 3.1, Eq. 3); for MuJoCo
states of 17 to 27 dimensions the text is 15 to 40 tokens (Sec. 5.2), i.e.
about one token per state dimension.  The paper gives neither the text format
nor the tokenizer (the backbone's own tokenizer is not available here).  The
reading used, also stated in the design document:

  text   "state:" followed, for each dimension in order, by a space and the
         value clamped to [-9.9, 9.9] and written with one decimal, correctly
         rounded from the exact fp32 value (exact ties to the even digit);
         a value that rounds to zero is written "0.0" (no "-0.0"); NaN is
         written "0.0".
  tokens a stand-in vocabulary of 457 entries: id 0 begin-of-state, id 1 the
         string "state:", ids 2 .. 200 the strings " -9.9" .. " 9.9" in
         increasing order (id = 2 + 99 + round(10 v)), ids 201 .. 456 the 256
         single bytes (id = 201 + byte).  Text is tokenised greedily, longest
         entry first, after the begin-of-state token; the byte entries make the
         tokenizer total on any byte string.

With this vocabulary a state of n dimensions is n + 2 tokens: 19 to 29 for
n = 17 .. 27, inside the range the paper reports.

Parity pins (tests/test_serialize_oracle_pins.py): hand-worked cases in
tests/golden/serialize_hand_cases.txt, the token count n + 2 and its place in
the paper's 15 - 40 range, decoding the ids back to the text, rounding ties
and clamping cases worked by hand, agreement of the one-decimal rendering with
exact rational arithmetic on random fp32 values.
"""
from __future__ import annotations

from fractions import Fraction
from typing import List, Sequence

import numpy as np

BOS_ID = 0
STATE_ID = 1
NUM_BASE = 2          # id of " -9.9"
BYTE_BASE = 201       # id of byte 0
VOCAB_SIZE = 457
CLAMP_TENTHS = 99     # |value| is clamped to 9.9


def tenths(x) -> int:
    """The integer m with m / 10 the one-decimal rendering of the fp32 value x after clamping: the
    exact value times ten, rounded to the nearest integer, exact ties to even; NaN gives 0."""
    x = np.float32(x)
    if np.isnan(x):
        return 0
    if x >= np.float32(9.9):      # fp32(9.9) = 9.8999996...: everything at or above it renders as 9.9
        return CLAMP_TENTHS
    if x <= np.float32(-9.9):
        return -CLAMP_TENTHS
    t = Fraction(float(x)) * 10   # exact: a float is a dyadic rational
    fl = t.numerator // t.denominator
    rem = t - fl
    if rem > Fraction(1, 2) or (rem == Fraction(1, 2) and fl % 2 != 0):
        fl += 1
    return max(-CLAMP_TENTHS, min(CLAMP_TENTHS, int(fl)))


def number_text(m: int) -> str:
    """One-decimal text of m / 10, m in -99 .. 99; zero has no sign."""
    sign = "-" if m < 0 else ""
    a = abs(m)
    return "%s%d.%d" % (sign, a // 10, a % 10)


def serialize_text(state: Sequence[float]) -> str:
    """serialize(s) as text (Sec. 3.1, Eq. 3; format as stated in the module docstring)."""
    return "state:" + "".join(" " + number_text(tenths(v)) for v in np.asarray(state, dtype=np.float32).ravel())


def vocabulary() -> List[bytes]:
    """The stand-in vocabulary, entry i is the byte string of token id i (entry 0, begin-of-state, is empty)."""
    v = [b"", b"state:"]
    v += [(" " + number_text(m)).encode("ascii") for m in range(-CLAMP_TENTHS, CLAMP_TENTHS + 1)]
    v += [bytes([b]) for b in range(256)]
    assert len(v) == VOCAB_SIZE
    return v


def tokenize(text: bytes) -> List[int]:
    """Begin-of-state, then greedy longest-match over the vocabulary (the byte entries always match)."""
    if isinstance(text, str):
        text = text.encode("utf-8")
    vocab = vocabulary()
    by_len = sorted(((s, i) for i, s in enumerate(vocab) if len(s) > 1), key=lambda p: -len(p[0]))
    ids = [BOS_ID]
    pos = 0
    while pos < len(text):
        for s, i in by_len:
            if text.startswith(s, pos):
                ids.append(i)
                pos += len(s)
                break
        else:
            ids.append(BYTE_BASE + text[pos])
            pos += 1
    return ids


def detokenize(ids: Sequence[int]) -> bytes:
    vocab = vocabulary()
    return b"".join(vocab[i] for i in ids)


def serialize_ids(state: Sequence[float]) -> List[int]:
    """Token ids of serialize(s): what the frozen encoder reads for this state."""
    return tokenize(serialize_text(state))
