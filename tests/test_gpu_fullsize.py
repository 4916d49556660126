"""GPU parity at the benchmark's full sizes, in the launch configuration bench.py times: the
Llama2-7B, Llama3-8B and Llama2-70B layer shapes of the benchmark configurations.  Products are
checked on every row against the oracle where that takes seconds, else on sampled rows (the
oracle computes any row on its own); dequantized weights are checked bit for bit on sampled rows."""
import numpy as np
import pytest

import mpq_synth as synth
import oracle
import paper_2311_16442_amd as mpq
from gpu_util import Guarded, Workspace, rel_err, to_dev

pytestmark = pytest.mark.gpu
TOL = 2e-3


@pytest.fixture(scope="module")
def torch():
    import torch as t
    assert t.cuda.is_available(), "these tests need the MI355X"
    return t


def sample_rows(N, count, seed):
    rng = np.random.default_rng(seed)
    rows = set(range(16)) | set(range(N - 16, N)) | set(int(r) for r in rng.integers(0, N, size=count))
    return np.array(sorted(rows), dtype=np.int64)


def sub_matrix(lg, rows):
    """Oracle matrix holding only `rows` of the logical matrix (rows decode independently)."""
    s = lg.spec
    counts = (lg.row_ptr[rows + 1] - lg.row_ptr[rows]).astype(np.int64)
    rp = np.zeros(rows.size + 1, dtype=np.int32)
    rp[1:] = np.cumsum(counts)
    idx = np.concatenate([np.arange(lg.row_ptr[r], lg.row_ptr[r + 1]) for r in rows]) if rows.size else np.zeros(0, int)
    idx = idx.astype(np.int64)
    if getattr(s, "g2_axis", 0) == 1:
        # pairs shared by g2 rows: give every sampled row its own copy (blocks of one row)
        return oracle.Matrix(rows.size, s.K, s.g1, 1, lg.is4, lg.codes[rows], lg.s_int[rows], lg.z1[rows],
                             lg.s2[rows // s.g2], lg.z2[rows // s.g2], rp, lg.col[idx], lg.val[idx], g2_axis=1)
    return oracle.Matrix(rows.size, s.K, s.g1, s.g2, lg.is4, lg.codes[rows], lg.s_int[rows], lg.z1[rows],
                         lg.s2[rows], lg.z2[rows], rp, lg.col[idx], lg.val[idx])


def check_products(torch, lg, pk, blob, Ms, all_rows):
    s = lg.spec
    rows = np.arange(s.N) if all_rows else sample_rows(s.N, 96, s.seed)
    om = oracle.Matrix.from_logical(lg) if all_rows else sub_matrix(lg, rows)
    for M in Ms:
        X = synth.make_x(s.seed + M, M, s.K)
        Y = Guarded(torch, M * s.N)
        if M == 1:
            mpq.gemv(pk.header, blob, to_dev(torch, X[0].view(np.int16)), Y.view)
        else:
            ws = Workspace(torch, mpq, pk.header, M)
            mpq.gemm(pk.header, blob, to_dev(torch, X.view(np.int16)), Y.view, M, workspace=ws.view)
            ws.check()
        got = Y.check_and_get().reshape(M, s.N)
        ref = om.gemm(X, threads=8)
        # the floor of the error measure uses the rms over the rows that were checked
        e_floor, e_max = rel_err(got[:, rows], ref)
        print(f"{s.name} {s.N}x{s.K} M={M}: rows checked {rows.size}, err {e_floor:.2e}", flush=True)
        assert e_floor <= TOL, (s.name, M, e_floor, e_max)


def check_dequant_rows(torch, lg, pk, blob):
    s = lg.spec
    if s.N * s.K > 550e6:      # keep the fp16 output near 1 GB at most (the largest matrix of the benchmark is 470e6 weights)
        return
    # every row where the oracle needs a few seconds (the Llama2-7B shapes), 48 sampled rows of larger matrices
    rows = np.arange(s.N) if s.N * s.K <= 100e6 else sample_rows(s.N, 48, s.seed + 7)
    sub = sub_matrix(lg, rows)
    for add in ((True, False) if rows.size == s.N else (True,)):   # the dense part alone takes other stores
        out = Guarded(torch, s.N * s.K)
        mpq.dequant(pk.header, blob, out.view, add_outliers=add)
        torch.cuda.synchronize()
        got = out.buf[128:128 + s.N * s.K].view(s.N, s.K)[torch.from_numpy(rows).cuda()].cpu().numpy().view(np.uint16)
        host_head = out.buf[:128].cpu().numpy().view(np.uint16)
        host_tail = out.buf[128 + s.N * s.K:].cpu().numpy().view(np.uint16)
        assert np.all(host_head == 0x7B7B) and np.all(host_tail == 0x7B7B)
        assert np.array_equal(got, sub.dequant(add)), (s.name, add)
        del out, got


@pytest.mark.parametrize("idx", [0, 1, 2, 3])
def test_llama2_7b_layer_every_row(torch, idx):
    spec = synth.config_specs(1)[idx]
    lg = synth.make_matrix(spec)
    pk = mpq.pack_logical(lg)
    blob = to_dev(torch, pk.blob)
    check_products(torch, lg, pk, blob, [1], all_rows=True)
    check_products(torch, lg, pk, blob, [4, 16, 32], all_rows=False)
    check_dequant_rows(torch, lg, pk, blob)


@pytest.mark.parametrize("f4,p_o", [(0.0, 0.0), (0.25, 0.015), (0.0, 0.015), (0.25, 0.0)])
def test_llama2_7b_format_sweep_corners(torch, f4, p_o):
    # corners of the sweep over the 4-bit fraction and the outlier fraction (configuration 2)
    spec = synth.config_specs(2, f4=f4, p_o=p_o)[1]
    lg = synth.make_matrix(spec)
    pk = mpq.pack_logical(lg)
    blob = to_dev(torch, pk.blob)
    check_products(torch, lg, pk, blob, [1, 16], all_rows=True)


@pytest.mark.parametrize("idx", [0, 1, 2, 3, 4])
def test_llama3_8b_shapes_group_128(torch, idx):
    spec = synth.config_specs(3)[idx]
    lg = synth.make_matrix(spec)
    pk = mpq.pack_logical(lg)
    blob = to_dev(torch, pk.blob)
    check_products(torch, lg, pk, blob, [1], all_rows=spec.N * spec.K < 150e6)
    check_dequant_rows(torch, lg, pk, blob)


@pytest.mark.parametrize("idx", [0, 1, 2, 3])
def test_llama2_70b_shapes_sampled(torch, idx):
    # all four shapes of the Llama2-70B slice, the 57344 x 8192 gate+up matrix included (the largest of
    # the benchmark: 155 MB packed, the plane-sum kernel at M = 1, the K-range kernel at M = 8)
    spec = synth.config_specs(4)[idx]
    lg = synth.make_matrix(spec)
    pk = mpq.pack_logical(lg)
    blob = to_dev(torch, pk.blob)
    check_products(torch, lg, pk, blob, [1, 8], all_rows=False)
    check_dequant_rows(torch, lg, pk, blob)


@pytest.mark.parametrize("layer", [1, 2, 3, 4])
def test_llama2_70b_distinct_layers_sampled(torch, layer):
    # the decode sweep runs over layers that differ; layers 1..4 (seeded by their index), each with a
    # different one of the four shapes, sampled rows, M in {1, 8}
    spec = synth.config_specs(4, layer_index=layer)[layer % 4]
    assert spec.seed != synth.config_specs(4)[layer % 4].seed
    lg = synth.make_matrix(spec)
    pk = mpq.pack_logical(lg)
    blob = to_dev(torch, pk.blob)
    check_products(torch, lg, pk, blob, [1, 8], all_rows=False)


@pytest.mark.parametrize("M", [4, 32])
def test_llama2_7b_gate_up_at_the_heavy_sweep_corner(torch, M):
    # 25 % 4-bit groups and 1.5 % outliers on the largest Llama2-7B matrix (configuration 2), M = 4 and 32
    spec = synth.config_specs(2, f4=0.25, p_o=0.015)[2]
    lg = synth.make_matrix(spec)
    pk = mpq.pack_logical(lg)
    blob = to_dev(torch, pk.blob)
    check_products(torch, lg, pk, blob, [M], all_rows=False)


@pytest.mark.parametrize("meta", [0, 1])
@pytest.mark.parametrize("idx", [1, 3])
def test_llama2_7b_shapes_at_the_papers_operating_point(torch, idx, meta):
    # g1 = g2 = 16, second-order pairs shared by 16 rows (Sec. 2.2), 25 % 4-bit groups (Sec. 3.3); with byte-wide
    # scales and zero points, and with the paper's aligned metadata (Sec. 3.3 "Memory Alignment")
    base = synth.config_specs(1)[idx]
    spec = synth.MatrixSpec(base.name, base.N, base.K, 16, 16, 0.25, 0.005, base.seed, 1, meta)
    lg = synth.make_matrix(spec)
    pk = mpq.pack_logical(lg)
    blob = to_dev(torch, pk.blob)
    check_products(torch, lg, pk, blob, [1], all_rows=True)
    check_products(torch, lg, pk, blob, [4, 8, 32], all_rows=False)   # four pieces per unit in the batch kernels
    check_dequant_rows(torch, lg, pk, blob)


@pytest.mark.parametrize("fmt", [(16, 16, 0.25, 1, 0), (16, 16, 0.25, 1, 1), (32, 16, 0.10, 0, 0)], ids=["g16", "g16_aligned", "g32"])
def test_dequant_of_gate_up_with_narrow_groups(torch, fmt):
    # 22016 x 4096, every row: 43 ranges of 16 rows x 2048 columns per workgroup, the launch that bench.py times
    g1, g2, f4, axis, meta = fmt
    base = synth.config_specs(1)[2]
    lg = synth.make_matrix(synth.MatrixSpec(base.name, base.N, base.K, g1, g2, f4, 0.005, base.seed, axis, meta))
    pk = mpq.pack_logical(lg)
    check_dequant_rows(torch, lg, pk, to_dev(torch, pk.blob))



@pytest.mark.parametrize("M", [9, 12, 14])
def test_llama2_7b_qkv_at_batches_that_fit_one_chunk(torch, M):
    # 12288 x 4096 (17.7 MB) with 9 to 14 activation rows: the resident-activation kernel with 16 or 8 waves
    lg = synth.make_matrix(synth.config_specs(1)[0])
    pk = mpq.pack_logical(lg)
    check_products(torch, lg, pk, to_dev(torch, pk.blob), [M], all_rows=False)
