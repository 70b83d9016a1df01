"""GPU parity on inputs whose scores span a wide range, so that the parts of the kernels that
merge partial softmaxes are exercised where it matters: the running-maximum rescale of the
streaming forward long after the first key tile, the merge of the chunks of a question-token
owner whose maxima differ by hundreds of score units, and exp(s - lse) in both backward kernels
at large |s|.  One softmax over (question keys U own row / column keys), as the head equation
of Section 3 asks, is exactly what these branches implement.

Inputs (synth.draw_wide_range_tensors): raw scores q.k with a standard deviation of 60 (7.5 after
the scale of 1/8), key norms growing along the sequence, and five table tokens per sequence whose
keys score 150 .. 350 more than the rest against every query, placed late in the sequence.
Segment path, dense-mask path and bucketed tables, forward and backward, element by element
against the float64 oracle with the same tolerances as everywhere else."""
import numpy as np
import pytest

from paper_2109_04312_amd import synth
from tests import helpers as hp
from tests.test_wide_range_inputs import wide_workload

pytestmark = pytest.mark.gpu
ROW, COL = synth.HEAD_ROW, synth.HEAD_COL


def check(w, dense=False, bucketed=None, backward=True, pairs=None, label=""):
    print(f"wide-range case {label or w.name} dtype={w.dtype} shape={w.shape} dense={dense} "
          f"bucketed={bucketed}", flush=True)
    got, seg = hp.run_hip(w, backward, dense=dense, bucketed=bucketed)
    if seg is not None:
        hp.compare_segments(seg, w.structure, bucketed=bucketed)
    ref = hp.run_oracle(w, backward, pairs, bucketed=bucketed)
    slack = None
    if backward and w.dtype == "bf16":
        # forward results are held to the usual bounds; gradients get twice what the bf16 format
        # itself costs on inputs of this magnitude (helpers.format_cost) on top of them
        cost = hp.format_cost(w, sorted(ref), bucketed=bucketed)
        slack = {bh: {n: 2.0 * c[n] for n in ("dq", "dk", "dv")} for bh, c in cost.items()}
        print("   bf16 format cost (max |model - oracle|):",
              {n: f"{max(c[n] for c in cost.values()):.2e}" for n in ("o", "dq", "dk", "dv")}, flush=True)
    print(hp.report(hp.compare(got, ref, w, label or w.name, slack=slack)), flush=True)


def test_segment_path_wide_scores():
    # 150 question tokens: two owner tiles; ~1900 table tokens: the question owners' key stream is
    # cut into chunks; rows of ~24 tokens, columns of ~320
    w = wide_workload(3, "bf16", N=2600, n_global=150, rows=80, cols=6, mean_cell=4.0)
    check(w)


def test_f32_path_wide_scores_forward():
    """The fp32 path (one wavefront per query, a running maximum over 64-key batches) on the same
    inputs, forward.  Scaled scores reach +-50 here, and an fp32 score of that size carries a
    rounding error of ~50 * 2^-24 * sqrt(64) in the exponent, so the 1e-4 of the N(0,1) inputs
    (|score| < 8) is scaled by max|LSE| / 8."""
    w = wide_workload(3, "f32", N=2600, n_global=150, rows=80, cols=6, mean_cell=4.0)
    print(f"wide-range case f32 forward shape={w.shape}", flush=True)
    got, _ = hp.run_hip(w, backward=False)
    ref = hp.run_oracle(w, False, None)
    for (b, h), d in ref.items():
        nonpad = w.structure.flags[b] != synth.TOK_PAD
        kappa = max(1.0, float(np.abs(d["lse"][nonpad]).max()) / 8.0)
        for name in ("o", "lse"):
            err = np.abs(got[name][b, h] - d[name])[nonpad]
            print(f"   {name}[{b},{h}] max-abs {err.max():.2e} (bound {1e-4 * kappa:.2e})", flush=True)
            assert err.max() <= 1e-4 * kappa, (name, b, h, err.max())


def test_segment_path_wide_scores_long_segments_and_batch():
    # long cells: row segments of ~150 tokens and column segments of ~600 (several key tiles per
    # query in both head kinds), two sequences of different shape in one batch
    w = wide_workload(4, "bf16", N=4096, n_global=64, rows=24, cols=6, mean_cell=25.0, B=2, H=2)
    check(w)


def test_dense_path_wide_scores():
    w = wide_workload(5, "bf16", N=1024, n_global=70, rows=30, cols=5, mean_cell=5.0, B=2)
    check(w, dense=True)


@pytest.mark.parametrize("mode", [(116, 42), (40, 64)])
def test_bucketed_tables_wide_scores(mode):
    # the global part is cut at G (question tokens past it stream as table tokens) and windows at
    # three buckets of R: the same kernels on other tables
    w = wide_workload(6, "bf16", N=2600, n_global=150, rows=80, cols=6, mean_cell=4.0)
    check(w, bucketed=mode, label=f"wide bucketed {mode}")
