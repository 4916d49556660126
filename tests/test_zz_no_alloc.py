"""mpq_gemm_static (the product with the library's own device scratch as workspace, for callers that
cannot allocate) against mpq_gemm with a caller-owned workspace: same kernels, so the same bits, and
within the tolerance of the oracle.  Two calls in a row through the C ABI, the second on a smaller
input; the file's name sorts it after the other GPU tests."""
import numpy as np
import pytest

import mpq_synth as synth
import oracle
import paper_2311_16442_amd as mpq
from gpu_util import Guarded, Workspace, rel_err, to_dev

pytestmark = pytest.mark.gpu
TOL = 2e-3


def one_call(torch, N, K, M, seed):
    lg = synth.make_matrix(synth.MatrixSpec("na", N, K, 64, 16, 0.10, 0.005, seed))
    om, pk = oracle.Matrix.from_logical(lg), mpq.pack_logical(lg)
    blob = to_dev(torch, pk.blob)
    X = synth.make_x(seed + 1, M, K)
    Xd = to_dev(torch, X.view(np.int16))
    ws = Workspace(torch, mpq, pk.header, M)
    assert 0 < ws.bytes <= mpq.STATIC_SCRATCH_BYTES        # the path that needs scratch memory is the one that runs
    Y_ref = Guarded(torch, M * N)
    rep = mpq.gemm_planned(pk.header, blob, Xd, Y_ref.view, M, workspace=ws.view)
    assert rep.kernel == mpq.KERNEL_BATCH_RANGES
    want = Y_ref.check_and_get().reshape(M, N)
    ws.check()
    Y = Guarded(torch, M * N)
    mpq.gemm_static(pk.header, blob, Xd, Y.view, M)
    got = Y.check_and_get().reshape(M, N)
    assert np.array_equal(got, want)
    e_floor, e_max = rel_err(got, om.gemm(X, threads=8))
    assert e_floor <= TOL, (e_floor, e_max)


def test_static_scratch_entry_point_matches_the_workspace_one():
    import torch
    assert torch.cuda.is_available(), "this test needs the MI355X"
    one_call(torch, 272, 11008, 32, 5151)     # 17 tiles, long rows: several K ranges of partial sums
    one_call(torch, 96, 11008, 9, 5252)       # smaller matrix, smaller batch, right after it: the array keeps the first call's contents


def test_static_scratch_entry_point_refuses_what_does_not_fit():
    import torch
    assert torch.cuda.is_available(), "this test needs the MI355X"
    # 18750 row tiles: the partial sums of a batch of 32 (two batch halves, fp32) need 38 MB, more than the
    # library holds; a batch of 8 needs 19 MB and runs
    N, K = 300000, 64
    lg = synth.make_matrix(synth.MatrixSpec("tall", N, K, 64, 1, 0.0, 0.001, 5353))
    om, pk = oracle.Matrix.from_logical(lg), mpq.pack_logical(lg)
    blob = to_dev(torch, pk.blob)
    assert mpq.gemm_workspace_size(pk.header, 32) > mpq.STATIC_SCRATCH_BYTES >= mpq.gemm_workspace_size(pk.header, 8) > 0
    X = synth.make_x(5354, 32, K)
    Xd = to_dev(torch, X.view(np.int16))
    Y = Guarded(torch, 32 * N)
    with pytest.raises(mpq.MpqError) as e:
        mpq.gemm_static(pk.header, blob, Xd, Y.view, 32)
    assert e.value.status == mpq.MPQ_ERR_SIZE
    Y.check_and_get()                                     # nothing was written
    Y8 = Guarded(torch, 8 * N)
    mpq.gemm_static(pk.header, blob, Xd, Y8.view, 8)      # the first 8 rows of X
    e_floor, e_max = rel_err(Y8.check_and_get().reshape(8, N), om.gemm(X[:8], threads=8))
    assert e_floor <= TOL, (e_floor, e_max)
    with pytest.raises(mpq.MpqError) as e:
        mpq.gemm_static(pk.header, blob, Xd, Y.view, 33)  # batch beyond the limit: refused before anything else
    assert e.value.status == mpq.MPQ_ERR_SHAPE
