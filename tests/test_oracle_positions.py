"""Pins for the oracle's positional index with a restart per cell (Section 3.2), CPU only:
a hand-written example and an independent formulation with the library's run grouping."""
import numpy as np

from oracle import mate_oracle as orc
from paper_2109_04312_amd import synth

L, G, P = synth.TOK_LOCAL, synth.TOK_GLOBAL, synth.TOK_PAD


def test_cell_positions_hand_example_and_groupby():
    import itertools
    flags = np.array([[G, G, L, L, L, L, L, G, L, P, L, L]], np.uint8)
    row = np.array([[0, 0, 1, 1, 1, 2, 2, 0, 2, 0, 2, 2]], np.int32)
    col = np.array([[0, 0, 1, 1, 2, 2, 2, 0, 2, 0, 2, 3]], np.int32)
    #                q  q  |cell  | c | cell | q  c  pad c  c      (a question token and a pad end a cell)
    want = np.array([[0, 1, 0, 1, 0, 0, 1, 7, 0, 0, 0, 0]], np.int32)
    assert np.array_equal(orc.cell_positions(row, col, flags), want)
    # independent formulation: runs of equal (flag, row, column) keys via the library's groupby
    rng = np.random.default_rng(5)
    for seed in range(4):
        st = synth.random_structure(rng, 3, 120, max_rows=5, max_cols=4, max_global=9, max_cell=6,
                                    scatter=seed >= 2)
        got = orc.cell_positions(st.row_ids, st.col_ids, st.flags)
        for b in range(st.B):
            keys = [(int(f), int(r), int(c)) if f == L else (int(f), -1, p)   # non-table tokens: runs of one
                    for p, (f, r, c) in enumerate(zip(st.flags[b], st.row_ids[b], st.col_ids[b]))]
            p = 0
            for key, run in itertools.groupby(keys):
                n = len(list(run))
                if key[0] == L:
                    assert np.array_equal(got[b, p:p + n], np.arange(n))
                elif key[0] == G:
                    assert got[b, p] == p
                else:
                    assert got[b, p] == 0
                p += n
