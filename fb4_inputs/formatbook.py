"""Default FB4 formatbook, as data.

The paper draws its 32-dialect formatbook in a figure (Fig. 2a) and states in
the text (Sec. 3.1, "Formatbook Design") only the rules it was built by.  The
table below is this repository's own table built to those rules; it is input
data for both the CPU oracle and the GPU library (each takes the formatbook as
an argument) and carries none of the method's arithmetic.

Rules met (Sec. 3.1; Sec. 3.4 for the range buckets; App. B for the ordering):
  * 32 dialects, 8 ascending integer magnitudes each, drawn from 0..15;
  * index 0 is magnitude 0 in every dialect (App. E.1);
  * every dialect's largest magnitude lies in 8..15 (one "dynamic range" per
    possible integer block maximum), dialect IDs ordered by that range;
  * narrower ranges get fewer dialects: 2,2,3,3,4,5,6,7 for ranges 8..15;
  * within a range the dialects run from small-magnitude-dense to
    large-magnitude-preserving.
Dialect 11 is the FP4-E2M1 value set times two and dialect 23 the uniform
step-2 grid; tests use them as textbook special cases.
"""

import numpy as np

DEFAULT_FORMATBOOK = np.array(
    [
        [0, 1, 2, 3, 4, 5, 6, 8],      # D0   range 8
        [0, 1, 2, 3, 4, 6, 7, 8],      # D1
        [0, 1, 2, 3, 4, 5, 7, 9],      # D2   range 9
        [0, 1, 2, 3, 5, 7, 8, 9],      # D3
        [0, 1, 2, 3, 4, 5, 7, 10],     # D4   range 10
        [0, 1, 2, 3, 4, 6, 8, 10],     # D5
        [0, 1, 2, 4, 6, 8, 9, 10],     # D6
        [0, 1, 2, 3, 4, 5, 8, 11],     # D7   range 11
        [0, 1, 2, 3, 5, 7, 9, 11],     # D8
        [0, 1, 2, 4, 6, 8, 10, 11],    # D9
        [0, 1, 2, 3, 4, 5, 8, 12],     # D10  range 12
        [0, 1, 2, 3, 4, 6, 8, 12],     # D11  (E2M1 x 2)
        [0, 1, 2, 4, 6, 8, 10, 12],    # D12
        [0, 1, 3, 5, 7, 9, 11, 12],    # D13
        [0, 1, 2, 3, 4, 6, 9, 13],     # D14  range 13
        [0, 1, 2, 3, 5, 7, 10, 13],    # D15
        [0, 1, 2, 4, 6, 8, 11, 13],    # D16
        [0, 1, 3, 5, 7, 9, 11, 13],    # D17
        [0, 2, 4, 6, 8, 10, 12, 13],   # D18
        [0, 1, 2, 3, 4, 6, 9, 14],     # D19  range 14
        [0, 1, 2, 3, 5, 7, 10, 14],    # D20
        [0, 1, 2, 4, 6, 8, 11, 14],    # D21
        [0, 1, 3, 5, 7, 9, 12, 14],    # D22
        [0, 2, 4, 6, 8, 10, 12, 14],   # D23  (uniform step 2)
        [0, 2, 5, 8, 10, 12, 13, 14],  # D24
        [0, 1, 2, 3, 4, 6, 10, 15],    # D25  range 15
        [0, 1, 2, 3, 5, 8, 11, 15],    # D26
        [0, 1, 2, 4, 6, 8, 11, 15],    # D27
        [0, 1, 3, 5, 7, 9, 12, 15],    # D28
        [0, 2, 4, 6, 8, 10, 12, 15],   # D29
        [0, 2, 4, 7, 9, 11, 13, 15],   # D30
        [0, 3, 6, 9, 11, 13, 14, 15],  # D31
    ],
    dtype=np.uint8,
)

# Two one-dialect formatbooks used as textbook special cases by the tests.
E2M1_X2_FORMATBOOK = np.array([[0, 1, 2, 3, 4, 6, 8, 12]], dtype=np.uint8)
UNIFORM_STEP2_FORMATBOOK = np.array([[0, 2, 4, 6, 8, 10, 12, 14]], dtype=np.uint8)


def default_formatbook() -> np.ndarray:
    """A fresh copy of the default [32][8] uint8 formatbook."""
    return DEFAULT_FORMATBOOK.copy()


def range_buckets(formatbook: np.ndarray) -> list:
    """DIDs grouped by dynamic range: bucket r (0..7) holds the dialects whose
    largest magnitude is 8 + r (Sec. 3.4: one dialect per range, block maxima
    8..15).  Pure bookkeeping on the table."""
    tops = np.asarray(formatbook)[:, 7].astype(int)
    return [[int(d) for d in np.nonzero(tops == 8 + r)[0]] for r in range(8)]
