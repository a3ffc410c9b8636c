"""Shared helpers of the GPU parity tests: run a workload through the C ABI (via the thin
binding) and through the oracle, and compare to the stated bar:

  * relative Frobenius error <= 1e-3 per output tensor: the run's logits and probs
    matrices, and each tenant's logits and probs matrices when the tenant has at least
    MIN_ROWS_PER_TENSOR rows in the comparison;
  * a tenant's matrices of MIN_ROWS_PER_TENSOR .. ONE_FLIP_ROWS - 1 rows may set aside their one
    worst row (which must be <= ROW_TOL like every row) and must then be <= 1e-3: one row at
    the row bar moves a tensor of n rows by 1e-2 / sqrt(n), which is below 1e-3 only from
    ONE_FLIP_ROWS = 100 rows on; seen on the full c3 mix, where a tenant with exactly 16 rows
    has one row with a flip and reads 1.1e-3 while its 15 other rows agree to 1e-7;
  * every tenant's matrices and every single row <= ROW_TOL.  With bf16 hidden activations
    a row's error is bimodal: ~1e-7 when every hidden value rounds the same way as in the
    fp64 oracle, ~1e-3 once one value sitting on a rounding boundary goes the other way,
    because that one-ulp difference is amplified by the re-quantisation of every later
    layer.  An exactly rounded fp32 accumulation shows the same (up to 2.5e-3 per row in
    simulation on the five mixes; 7.2e-3 for one request of a 33-unit-wide linear net with
    three small logits, reproduced on the CPU by taking the other bfloat16 neighbour of the
    one value that lies 3e-8 from a rounding boundary: tests/test_tolerance_model.py), so a
    tensor of one or two rows cannot be held to 1e-3; it is held to ROW_TOL instead;
  * so that the looser bar cannot hide a systematic error in the tiles that serve small
    tenants: all rows of tenants below MIN_ROWS_PER_TENSOR, taken together as one matrix,
    must be <= 1e-3 once there are MIN_ROWS_PER_TENSOR of them, the median error of those
    rows must be <= CLEAN_ROW (most rows see no flip at all), and, where the caller states
    the share of rows that must be flip-free (`min_clean_frac`, for the mixes whose nets are
    shallow enough that flips are rare), that share of all rows must be <= CLEAN_ROW;
  * deep bf16 nets (`deep=True`; the resnet18-shaped tenants: twenty convolutions, up to millions of
    hidden values per request) are compared at DEEP_REL_TOL per tensor and DEEP_ROW_TOL per row: with
    that many rounded values most rows hold several flips, and their effects add up to a few 1e-3
    (on the reduced net the GPU's one flipped row of 40, 6.59e-3, is exactly the row and the value
    that the exactly-rounded-fp32 evaluation of tests/test_tolerance_model.py gets, and already puts
    the 40-row tensor at 1.26e-3).  The kernels themselves are held to ~1e-6 on the same nets in fp32;
  * labels bit-exact wherever the oracle's top-2 logit margin exceeds 1e-2; elsewhere the
    label must be one of the oracle's two best classes.
"""
import numpy as np
import torch

import oracle
import paper_1901_06887_amd as mt
from paper_1901_06887_amd import torch_io

REL_FRO_TOL = 1e-3
ROW_TOL = 1e-2
MIN_ROWS_PER_TENSOR = 16
ONE_FLIP_ROWS = 100     # (ROW_TOL / REL_FRO_TOL) ** 2: from here on one row at the row bar cannot move a tensor past 1e-3
MARGIN = 1e-2
DEEP_REL_TOL = 1e-2     # deep bf16 nets: flips in most rows, see above
DEEP_ROW_TOL = 3e-2
CLEAN_ROW = 1e-5        # a row without a rounding flip agrees to ~1e-7 (bf16 mixes) or ~1e-6 (fp32)


def make_context(w, max_requests=None, max_tenants=None):
    ctx = mt.context_for(w.tenants, w.dtype, max_requests or max(1, w.n_requests), max_tenants=max_tenants)
    mt.register_tenants(ctx, w.tenants)
    return ctx


def gpu_run(ctx, w, ids=None, inputs=None, poison=False):
    ids = w.tenant_ids if ids is None else ids
    inputs = w.inputs if inputs is None else inputs
    d_ids = torch.from_numpy(np.ascontiguousarray(ids, dtype=np.int32)).cuda()
    d_x = torch_io.to_device(inputs, w.dtype)
    if poison:
        ctx.debug_poison()
    out = mt.serve(ctx, d_ids, d_x)
    torch.cuda.synchronize()
    return (out.logits.cpu().numpy().astype(np.float64), out.probs.cpu().numpy().astype(np.float64),
            out.labels.cpu().numpy(), out.n_classes.cpu().numpy())


def rel_fro(g, o):
    d = np.linalg.norm(g - o)
    n = np.linalg.norm(o)
    return d / n if n > 0 else d


def compare(w, gpu, orc, rows=None, what="", min_clean_frac=None, deep=False):
    """gpu/orc = (logits, probs, labels, n_classes) over the same rows (all, or `rows`)."""
    rel_tol, row_tol = (DEEP_REL_TOL, DEEP_ROW_TOL) if deep else (REL_FRO_TOL, ROW_TOL)
    g_lg, g_pr, g_lb, g_nc = gpu
    o_lg, o_pr, o_lb, o_nc = orc
    ids = w.tenant_ids if rows is None else w.tenant_ids[rows]
    assert np.array_equal(g_nc, o_nc), what
    C = o_lg.shape[1]
    assert np.all(g_lg[:, C:] == 0) and np.all(g_pr[:, C:] == 0)
    g_lg, g_pr = g_lg[:, :C], g_pr[:, :C]
    assert np.all(np.isfinite(g_lg)) and np.all(np.isfinite(g_pr)), what
    worst = 0.0
    for t in np.unique(ids):
        sel = ids == t
        n_t = int(sel.sum())
        tol = rel_tol if n_t >= MIN_ROWS_PER_TENSOR else row_tol
        for g, o in ((g_lg[sel], o_lg[sel]), (g_pr[sel], o_pr[sel])):
            e = rel_fro(g, o)
            if e > tol and MIN_ROWS_PER_TENSOR <= n_t < ONE_FLIP_ROWS:
                # one row with a rounding flip: set the worst row aside (it is still held to ROW_TOL below)
                keep = np.ones(n_t, dtype=bool)
                keep[int(np.argmax(np.linalg.norm(g - o, axis=1)))] = False
                e = rel_fro(g[keep], o[keep])
            worst = max(worst, e)
            assert e <= tol, "%s tenant %d (%d rows) rel fro %.3e" % (what, t, n_t, e)
    row_err = np.linalg.norm(g_lg - o_lg, axis=1) / np.maximum(np.linalg.norm(o_lg, axis=1), 1e-30)
    assert row_err.max() <= row_tol, "%s: a row is off by %.3e" % (what, row_err.max())
    # the rows of small tenants, pooled: the looser per-tensor bar above must not hide a systematic error
    ids_u, cnt_u = np.unique(ids, return_counts=True)
    small = np.isin(ids, ids_u[cnt_u < MIN_ROWS_PER_TENSOR])
    if int(small.sum()) >= MIN_ROWS_PER_TENSOR:
        for g, o in ((g_lg[small], o_lg[small]), (g_pr[small], o_pr[small])):
            assert rel_fro(g, o) <= rel_tol, "%s: the %d rows of small tenants together are off by %.3e" % (what, int(small.sum()), rel_fro(g, o))
        if not deep:
            assert np.median(row_err[small]) <= CLEAN_ROW, "%s: median row error of small tenants %.3e" % (what, np.median(row_err[small]))
    clean = float(np.mean(row_err <= CLEAN_ROW))
    if min_clean_frac is not None:
        assert clean >= min_clean_frac, "%s: only %.3f of the rows are free of rounding flips" % (what, clean)
    compare.last_clean_frac = clean
    assert rel_fro(g_lg, o_lg) <= rel_tol and rel_fro(g_pr, o_pr) <= rel_tol, what
    # labels
    srt = np.sort(o_lg + np.where(np.arange(C)[None, :] < o_nc[:, None], 0.0, -np.inf), axis=1)
    margin = srt[:, -1] - srt[:, -2] if C > 1 else np.full(len(ids), np.inf)
    clear = margin > MARGIN
    assert np.array_equal(g_lb[clear], o_lb[clear]), "%s: %d label mismatches on clear-margin rows" % (
        what, int(np.sum(g_lb[clear] != o_lb[clear])))
    for i in np.nonzero(~clear)[0]:
        top2 = np.argsort(-o_lg[i, :o_nc[i]], kind="stable")[:2]
        assert g_lb[i] in top2, what
    assert np.allclose(g_pr.sum(axis=1), 1.0, atol=1e-5), what
    return worst


def oracle_rows(w, rows=None, threads=16):
    models = oracle.models_from_workload(w)
    ids = w.tenant_ids if rows is None else w.tenant_ids[rows]
    x = w.inputs if rows is None else w.inputs[rows]
    lg, pr, lb, nc, _ = oracle.run_batch(models, ids, x.astype(np.float64), threads=threads)
    return lg, pr, lb, nc


def sample_rows(w, ctx_counts, n_random, bm=32, seed=0):
    """Rows to check one by one at full size: for every tenant the first and last rows of its
    segment and the rows around every 32-row boundary (every tile shape of the kernels is a
    multiple of 32 rows: 32, 64, 128 and 256), plus a random sample."""
    rng = np.random.default_rng(seed)
    pick = set(rng.choice(w.n_requests, size=min(n_random, w.n_requests), replace=False).tolist())
    for t in np.unique(w.tenant_ids):
        idx = np.nonzero(w.tenant_ids == t)[0]          # arrival order == order inside the segment
        edges = {0, len(idx) - 1}
        for b in range(bm, len(idx), bm):
            edges |= {b - 1, b}
        pick |= {int(idx[e]) for e in edges if 0 <= e < len(idx)}
    return np.array(sorted(pick), dtype=np.int64)
