"""GPU parity: the HIP library, called through its C ABI, against the CPU oracle
on the same seeded bytes.  Codes and integer accumulators must be bit-exact,
fp32 outputs within 1e-6 relative (they are expected to be identical: the scale
is a power of two, so alpha f + beta is one correctly rounded operation)."""
import numpy as np
import pytest

import oracle
import workloads as wl
from helpers import assert_out_close, compare_luts, oracle_pipeline, random_trees

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def mad():
    import torch
    import paper_2106_10860_amd as m
    assert torch.cuda.is_available()
    m.lib()   # raises if the HIP library is not built: there is no fallback
    return m


@pytest.fixture
def options(mad):
    """Sets kernel-selection switches of the library for one test; all back to 0 afterwards."""
    def set_option(option, value):
        mad.maddness_set_option(option, value)
    yield set_option
    for opt in range(4):
        mad.maddness_set_option(opt, 0)


def dev(x):
    import torch
    return torch.from_numpy(np.ascontiguousarray(x)).cuda()


def acc_buf(N, M):
    """Accumulator buffer; int16 storage stands in for uint16 (same bytes)."""
    import torch
    return torch.zeros((N, M), dtype=torch.int16, device="cuda")


def acc_np(t):
    return t.cpu().numpy().view(np.uint16)


def run_all(mad, A, sd, th, P, B, lda_pad=0, ldo_pad=0, label=""):
    """Runs encode, build_luts, scan and encode_scan on the GPU and checks each
    against the oracle.  Returns the number of table bytes that differ by one."""
    import torch
    N, D = A.shape
    M = B.shape[1]
    C = sd.shape[0]
    ref = oracle_pipeline(A, sd, th, P, B)

    A_d = torch.zeros((N, D + lda_pad), dtype=torch.float32, device="cuda")
    A_d[:, :D] = dev(A)
    A_v = A_d[:, :D]
    params = mad.Params(dev(sd), dev(th), dev(P))

    # g(A)
    codes_d = mad.maddness_encode(params, A_v)
    torch.cuda.synchronize()
    assert (codes_d.cpu().numpy() == ref["packed"]).all(), f"{label}: codes differ"

    # h(B)
    luts_d, scale_d, offset_d = mad.maddness_build_luts(params, dev(B))
    torch.cuda.synchronize()
    n_flip = compare_luts(luts_d.cpu().numpy(), scale_d.cpu().numpy(), offset_d.cpu().numpy(), ref, P, B)

    def fresh_out():
        o = torch.full((N, M + ldo_pad), -7.0, dtype=torch.float32, device="cuda")
        return o, o[:, :M]

    for which, (luts, scale, offset) in {
        "oracle tables": (dev(ref["luts"]), dev(ref["scale"]), dev(ref["offset"])),
        "gpu tables": (luts_d, scale_d, offset_d),
    }.items():
        if which == "oracle tables":
            want_out, want_acc = ref["out"], ref["acc"]
        else:
            want_out, want_acc, ov = oracle.scan(ref["packed"], C, luts.cpu().numpy(),
                                                 scale.cpu().numpy(), offset.cpu().numpy())
        # f from codes
        full, view = fresh_out()
        acc = acc_buf(N, M)
        mad.maddness_scan(C, codes_d, luts, scale, offset, out=view, acc=acc)
        torch.cuda.synchronize()
        assert (acc_np(acc) == want_acc).all(), f"{label}: scan accumulators differ ({which})"
        assert_out_close(view.cpu().numpy(), want_out, f"{label}: scan out ({which})")
        if ldo_pad:
            assert (full[:, M:] == -7.0).all(), "scan wrote outside its columns"
        # fused g, f
        full, view = fresh_out()
        acc2 = acc_buf(N, M)
        codes2 = torch.zeros_like(codes_d)
        mad.maddness_encode_scan(params, A_v, luts, scale, offset, out=view, acc=acc2, codes=codes2)
        torch.cuda.synchronize()
        assert (codes2.cpu().numpy() == ref["packed"]).all(), f"{label}: fused codes differ"
        assert (acc_np(acc2) == want_acc).all(), f"{label}: fused accumulators differ ({which})"
        assert_out_close(view.cpu().numpy(), want_out, f"{label}: fused out ({which})")
        assert (view.cpu().numpy() == want_out).all(), f"{label}: fused out not bit-identical ({which})"
        if ldo_pad:
            assert (full[:, M:] == -7.0).all(), "fused kernel wrote outside its columns"
        # optional outputs left out
        out3 = mad.maddness_encode_scan(params, A_v, luts, scale, offset)
        torch.cuda.synchronize()
        assert (out3.cpu().numpy() == want_out).all(), f"{label}: fused out without acc/codes differs"
    return n_flip


# (N, D, M, C, lda_pad, ldo_pad): ragged row counts, widths that are not multiples
# of 4 / 16 / 64, odd C, unaligned rows (D = 27), several column tiles, maximum C.
SHAPES = [
    (1, 8, 1, 1, 0, 0),
    (63, 27, 2, 4, 0, 0),
    (1000, 27, 2, 3, 1, 3),
    (257, 64, 10, 16, 0, 0),
    (777, 128, 100, 32, 4, 4),
    (513, 512, 256, 32, 0, 0),
    (300, 96, 300, 8, 0, 1),
    (4099, 512, 257, 31, 0, 0),
    (70, 33, 7, 5, 3, 0),
    (200, 64, 512, 64, 0, 0),      # tables larger than LDS: several column tiles
    (300, 48, 1030, 33, 0, 2),     # several tiles, ragged last tile
    (130, 40, 64, 256, 0, 0),      # maximum C
    (2050, 1024, 512, 64, 0, 0),   # the stress workload's D, M, C
    (66000, 16, 4, 2, 0, 0),       # many rows, tiny everything else
    (3000, 256, 512, 32, 0, 0),    # C = 32 with two 256-column tiles
    (1500, 1024, 400, 64, 0, 0),   # C = 64, ragged last 128-column tile
    # many rows with tables larger than LDS: fused kernel with the scan on the matrix cores
    (16400, 64, 512, 64, 0, 0),
    (20001, 128, 300, 32, 0, 4),   # C = 32, one pass of 8 x 64 columns, ragged
    (16390, 96, 130, 64, 4, 2),    # M = 130: last wavefront's columns partly outside
    (17000, 256, 1024, 64, 0, 0),  # four passes of 256 columns
    # the same kernel for shapes the table-in-LDS kernels do not take
    (16500, 1024, 256, 32, 0, 0),  # C = 32, rows of 4 KiB
    (16400, 2048, 64, 64, 4, 0),   # rows of 8 KiB, one wavefront's worth of columns
    (16390, 2048, 132, 32, 0, 0),  # C = 32, rows of 8 KiB: two rows staged per wavefront
    (20000, 512, 16, 32, 0, 0),    # a quarter of one wavefront's columns
    (16384, 1000, 40, 64, 0, 0),   # D not a multiple of C
    # many rows: the same kernel although the tables would fit in LDS, and its first phase
    # alone for maddness_encode
    (262144 + 37, 64, 256, 32, 0, 0),
    (262144 + 5, 128, 36, 64, 4, 0),
    (262144 + 9, 64, 128, 16, 0, 0),
    (20000, 128, 300, 16, 0, 4),   # C = 16 with more columns than the table-in-LDS kernel takes
    # output rows that do not start on 128-byte lines: results gathered in LDS, whole rows written
    (16400, 64, 1032, 32, 0, 0),   # three passes: 512 + 512 + 8 columns
    (16399, 64, 522, 64, 4, 0),    # C = 64: 256 + 256 + 10 columns, an odd number of 16-row groups somewhere
    (16500, 64, 512, 32, 0, 0),    # the same S phase for exactly one pass of 8 x 64 columns, aligned rows
    (16500, 128, 452, 16, 0, 60),  # ... with the last block partly filled
    # a multiple of 8 codebooks other than 16, 32, 64: the next larger kernel with padding codebooks
    (16400, 96, 132, 24, 0, 0),
    (20000, 64, 64, 8, 4, 0),
    (16390, 80, 36, 40, 0, 2),
    (17000, 112, 260, 56, 0, 0),
    (16500, 1024, 100, 24, 0, 0),
    (262144 + 3, 64, 36, 24, 0, 0),   # many rows: maddness_encode through the padded first phase
    (262144 + 3, 64, 36, 40, 4, 0),
    (16500, 1024, 260, 16, 4, 0),  # C = 16, rows of 4 KiB
    # many rows of any other shape: the phased kernel's form for rows of A that start and end anywhere, any
    # number of codebooks up to 64, any M, any pitch of the outputs
    (16400, 27, 2, 4, 0, 0),       # the image workload's D, M, C: rows too short for it, the general kernels
    (20000, 510, 250, 30, 1, 3),   # rows of 2044 bytes, 15 code bytes per row, output rows of 1012 bytes
    (16390, 131, 7, 5, 2, 0),      # 3 code bytes per row (the last high nibble unused), rows 532 bytes apart
    (16390, 253, 7, 5, 0, 0),      # rows of 1012 bytes: with the 12 bytes before an aligned start exactly 1 KiB
    (17000, 512, 10, 16, 0, 0),    # M = 10: aligned rows of A, output rows of 40 bytes; one block of columns,
                                   # shared by the eight wavefronts
    (16500, 256, 70, 20, 1, 5),    # two blocks of columns, four wavefronts each
    (16390, 600, 33, 40, 0, 0),    # C = 40 in the kernel for 64: two blocks of 32 columns
    (16500, 100, 257, 31, 0, 0),   # M = 4 * 64 + 1
    (16400, 1000, 130, 33, 0, 1),  # 33 codebooks in the kernel for 64
    (16385, 2045, 66, 64, 0, 1),   # rows of 8180 bytes, the longest it takes
    (16400, 511, 1030, 17, 0, 0),  # three passes of 512 columns, the last one of 6
    (262144 + 5, 130, 36, 12, 1, 0),   # ... and maddness_encode through the same first phase
    # output rows without padding between them: written as ranges of floats in 16-byte pieces
    (16390, 510, 250, 30, 0, 0),   # four blocks of columns (four wavefronts compute, four write), a last unit of 6 rows
    (16397, 300, 200, 50, 1, 0),   # seven blocks of 32 columns, two groups of rows per step
    (16400, 512, 250, 32, 0, 6),   # a pitch of 256: rows on 16-byte boundaries, each a range of its own
    (16400, 512, 249, 32, 0, 0),   # odd M: every row starts at another offset within 16 bytes
    # the ends of the ranges the library takes, with many rows
    (16500, 512, 40, 256, 0, 0),   # the most codebooks a 16-bit sum holds (255 x 256 < 65536)
    (16400, 64, 4100, 16, 0, 0),   # nine passes of 512 columns, the last of four
    (16400, 8192, 36, 64, 0, 0),   # rows of 32 KiB: longer than the staged forms take
]


@pytest.mark.parametrize("shape", SHAPES, ids=lambda s: "N%d_D%d_M%d_C%d_p%d_%d" % s)
def test_parity_random_parameters(mad, shape):
    N, D, M, C, lda_pad, ldo_pad = shape
    print("case", shape, flush=True)
    rng = np.random.default_rng(hash(shape) % (1 << 31))
    _, A, B = wl.random_problem(N * 7 + D, N, D, M, latent=min(8, D), N_train=4)
    sd, th = random_trees(rng, A, C)
    P = rng.standard_normal((C, 16, D)).astype(np.float32)
    run_all(mad, A, sd, th, P, B, lda_pad, ldo_pad, label=str(shape))


@pytest.mark.parametrize("shape", [(20001, 128, 300, 32, 0, 4), (16390, 96, 130, 64, 4, 2), (16400, 2048, 64, 64, 4, 0),
                                   (262144 + 37, 64, 256, 32, 0, 0), (20000, 128, 300, 16, 0, 4), (16400, 96, 132, 24, 0, 0),
                                   (20000, 510, 250, 30, 1, 3), (16390, 131, 7, 5, 2, 0), (16400, 1000, 130, 33, 0, 1),
                                   (16390, 510, 250, 30, 0, 0), (16397, 300, 200, 50, 1, 0)],
                         ids=lambda s: "N%d_D%d_M%d_C%d_p%d_%d" % s)
def test_parity_phased_kernel_many_regions(mad, shape, options):
    """The phased kernel with a few rows per wavefront and region: many regions, a ragged last one."""
    N, D, M, C, lda_pad, ldo_pad = shape
    print("case regions", shape, flush=True)
    options(mad.MADDNESS_OPT_PHASED_ROWS, 6)
    if C % 8:
        options(mad.MADDNESS_OPT_MAX_WORKGROUPS, 5)      # every workgroup takes many regions in turn
    rng = np.random.default_rng(hash(shape) % (1 << 31))
    _, A, B = wl.random_problem(N * 3 + D, N, D, M, latent=min(8, D), N_train=4)
    sd, th = random_trees(rng, A, C)
    P = rng.standard_normal((C, 16, D)).astype(np.float32)
    run_all(mad, A, sd, th, P, B, lda_pad, ldo_pad, label="regions " + str(shape))


def test_special_values(mad):
    """NaN, infinities and signed zeros in A; thresholds equal to data values."""
    rng = np.random.default_rng(77)
    N, D, M, C = 512, 32, 12, 8
    _, A, B = wl.random_problem(77, N, D, M)
    specials = np.array([np.nan, np.inf, -np.inf, -0.0, 0.0, 1e-45, -1e-45, 3.4e38], dtype=np.float32)
    A[rng.integers(0, N, 600), rng.integers(0, D, 600)] = specials[rng.integers(0, len(specials), 600)]
    sd, th = random_trees(rng, A, C)
    th[0, :15] = 0.0          # -0.0 >= +0.0 must go right
    th[1, :15] = -0.0
    th[2, 3] = np.nan         # a NaN threshold sends everything left
    th[3, 0] = np.inf
    P = rng.standard_normal((C, 16, D)).astype(np.float32)
    run_all(mad, A, sd, th, P, B, label="special values")


def test_degenerate_tables(mad):
    """A zero column of B (range 0), identical prototypes, a constant table."""
    rng = np.random.default_rng(78)
    N, D, M, C = 100, 16, 9, 4
    _, A, B = wl.random_problem(78, N, D, M)
    B[:, 2] = 0.0
    P = rng.standard_normal((C, 16, D)).astype(np.float32)
    P[1] = P[1, 0]            # codebook 1: all prototypes equal
    sd, th = random_trees(rng, A, C)
    run_all(mad, A, sd, th, P, B, label="degenerate tables")


@pytest.mark.parametrize("shape", [(1500, 64, 40, 8), (5000, 512, 256, 32), (20000, 128, 300, 32), (17000, 64, 100, 64)],
                         ids=["general", "row_streaming", "matrix_cores_C32", "matrix_cores_C64"])
def test_accumulators_without_fp32_output(mad, shape):
    """out = NULL: only the uint16 accumulators (and codes) are produced."""
    import torch
    N, D, M, C = shape
    rng = np.random.default_rng(91)
    _, A, B = wl.random_problem(91, N, D, M)
    sd, th = random_trees(rng, A, C)
    P = rng.standard_normal((C, 16, D)).astype(np.float32)
    ref = oracle_pipeline(A, sd, th, P, B)
    params = mad.Params(dev(sd), dev(th), dev(P))
    luts, scale, offset = dev(ref["luts"]), dev(ref["scale"]), dev(ref["offset"])
    acc = acc_buf(N, M)
    codes = torch.zeros((N, (C + 1) // 2), dtype=torch.uint8, device="cuda")
    r = mad.maddness_encode_scan(params, dev(A), luts, scale, offset, acc=acc, codes=codes, want_out=False)
    torch.cuda.synchronize()
    assert r is None
    assert (acc_np(acc) == ref["acc"]).all() and (codes.cpu().numpy() == ref["packed"]).all()
    acc2 = acc_buf(N, M)
    o, _ = mad.maddness_scan(C, codes, luts, scale, offset, acc=acc2, want_out=False)
    torch.cuda.synchronize()
    assert o is None and (acc_np(acc2) == ref["acc"]).all()


def test_calls_on_a_side_stream(mad):
    """Work is enqueued on the stream that is passed in, not on the null stream."""
    import torch
    N, D, M, C = 4096, 128, 64, 16
    rng = np.random.default_rng(92)
    _, A, B = wl.random_problem(92, N, D, M)
    sd, th = random_trees(rng, A, C)
    P = rng.standard_normal((C, 16, D)).astype(np.float32)
    ref = oracle_pipeline(A, sd, th, P, B)
    params = mad.Params(dev(sd), dev(th), dev(P))
    A_d, B_d = dev(A), dev(B)
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        luts, scale, offset = mad.maddness_build_luts(params, B_d, stream=side)
        out = mad.maddness_encode_scan(params, A_d, luts, scale, offset, stream=side)
    side.synchronize()
    want, _, _ = oracle.scan(ref["packed"], C, luts.cpu().numpy(), scale.cpu().numpy(), offset.cpu().numpy())
    assert (out.cpu().numpy() == want).all()


@pytest.mark.parametrize("shape", [(512, 10, 16), (64, 100, 32), (27, 2, 4), (512, 256, 32), (96, 37, 5)],
                         ids=lambda s: "D%d_M%d_C%d" % s)
def test_pooled_table_build(mad, shape):
    """Appendix A as printed: one scale and one offset per codebook, pooled over columns."""
    import torch
    D, M, C = shape
    rng = np.random.default_rng(D * 1000 + M)
    P = (rng.standard_normal((C, 16, D)) * rng.uniform(0.2, 3.0, size=(C, 1, 1))).astype(np.float32)
    B = (rng.standard_normal((D, M)) / np.sqrt(D)).astype(np.float32)
    T = oracle.build_luts_f64(P, B)
    luts_o, scale_o, offset_o, l, delta = oracle.quantize_luts_pooled(T)
    ref = dict(T=T, luts=luts_o, scale=scale_o, offset=offset_o, l=np.full(M, l, dtype=np.int32),
               delta=np.repeat(delta[:, None], M, axis=1))
    params = mad.Params(torch.zeros((C, 4), dtype=torch.int32, device="cuda"),
                        torch.zeros((C, 16), dtype=torch.float32, device="cuda"), dev(P))
    luts, scale, offset = mad.maddness_build_luts_pooled(params, dev(B))
    torch.cuda.synchronize()
    compare_luts(luts.cpu().numpy(), scale.cpu().numpy(), offset.cpu().numpy(), ref, P, B)
    # the scan consumes them like the per-column variant
    N = 300
    codes = rng.integers(0, 16, size=(N, C)).astype(np.uint8)
    packed = oracle.pack(codes)
    want, want_acc, _ = oracle.scan(packed, C, luts.cpu().numpy(), scale.cpu().numpy(), offset.cpu().numpy())
    got, _ = mad.maddness_scan(C, dev(packed), luts, scale, offset)
    torch.cuda.synchronize()
    assert (got.cpu().numpy() == want).all()


def test_row_strides_beyond_32_bits(mad):
    """lda and ldo so large that element offsets exceed 2^32: the kernels must do
    their row arithmetic in 64 bits.  (17 GiB + 17 GiB of address space, touched
    sparsely.)"""
    import torch
    N, D, M, C = 66000, 64, 128, 32
    big = 65536                                   # row stride in elements: 66000 * 65536 > 2^32
    rng = np.random.default_rng(93)
    _, A, B = wl.random_problem(93, N, D, M)
    sd, th = random_trees(rng, A, C)
    P = rng.standard_normal((C, 16, D)).astype(np.float32)
    ref = oracle_pipeline(A, sd, th, P, B)
    params = mad.Params(dev(sd), dev(th), dev(P))
    luts, scale, offset = dev(ref["luts"]), dev(ref["scale"]), dev(ref["offset"])
    A_big = torch.empty((N, big), dtype=torch.float32, device="cuda")
    A_big[:, :D] = dev(A)
    out_big = torch.empty((N, big), dtype=torch.float32, device="cuda")
    for a_view, o_view in ((A_big[:, :D], out_big[:, :M]),            # aligned: row-streaming kernels
                           (A_big[:, 1:D + 1], out_big[:, 1:M + 1])): # unaligned: general kernels
        if a_view.data_ptr() % 16:
            a_view.copy_(dev(A))
        o_view.fill_(-1.0)
        codes = mad.maddness_encode(params, a_view)
        mad.maddness_encode_scan(params, a_view, luts, scale, offset, out=o_view)
        torch.cuda.synchronize()
        assert (codes.cpu().numpy() == ref["packed"]).all()
        assert (o_view.cpu().numpy() == ref["out"]).all()
        o_view.fill_(-1.0)
        mad.maddness_scan(C, codes, luts, scale, offset, out=o_view)
        torch.cuda.synchronize()
        assert (o_view.cpu().numpy() == ref["out"]).all()
    del A_big, out_big
    torch.cuda.empty_cache()


def test_empty_input_is_a_no_op(mad):
    import torch
    A = torch.zeros((0, 16), dtype=torch.float32, device="cuda")
    params = mad.Params(torch.zeros((2, 4), dtype=torch.int32, device="cuda"),
                        torch.zeros((2, 16), dtype=torch.float32, device="cuda"))
    luts = torch.zeros((2, 16, 4), dtype=torch.uint8, device="cuda")
    s = torch.ones(4, device="cuda"); o = torch.zeros(4, device="cuda")
    assert mad.maddness_encode(params, A).shape == (0, 1)
    assert mad.maddness_encode_scan(params, A, luts, s, o).shape == (0, 4)
    torch.cuda.synchronize()


@pytest.mark.parametrize("cfg", [1, 2, 3, 6])
def test_parity_paper_shaped_workloads(mad, cfg):
    """Workloads 1-3 and 6 in full, with learned trees and ridge prototypes."""
    from paper_2106_10860_amd.learn import learn
    w = wl.get_workload(cfg)
    print("workload", w.name, flush=True)
    model = learn(wl.make_A_train(w), w.subspaces)
    A, B = wl.make_A(w), wl.make_B(w)
    run_all(mad, A, model.split_dims, model.thresholds, model.prototypes, B, label=w.name)


# (N, D, M, C, ldo, option MADDNESS_OPT_KERNELS) -> the kernel maddness_encode_scan must select
ROUTES = [
    ((1 << 18, 512, 256, 32, 256, 0), "fused_mfma_kernel, A by rows"),      # many rows: phased, scan on the matrix cores
    ((1 << 18, 512, 256, 32, 256, 1), "rows_kernel"),                       # ... switched off: lookups on the vector ALUs
    ((1 << 17, 512, 256, 32, 256, 0), "rows_kernel"),                       # fewer rows: tables in LDS
    ((20000, 1024, 512, 64, 512, 0), "fused_mfma_kernel, A by rows"),       # tables larger than LDS
    ((20000, 1024, 512, 64, 512, 1), "tiled_rows_kernel"),
    ((1 << 18, 510, 250, 30, 250, 0), "fused_mfma_kernel, A by rows [C = 32, DV = 2, NT = 4, DT = 0, SCAN = true, GATHER = true, PAD = true, ODD = true]"),
    ((20000, 131, 7, 5, 7, 0), "fused_mfma_kernel, A by rows [C = 16, DV = 1"),
    ((20000, 27, 2, 4, 2, 0), "scan_kernel<true>"),                         # the image workload's shape: rows too short
    ((5000, 64, 40, 8, 40, 0), "scan_kernel<true>"),                        # few rows of such a shape: the general kernel
    ((20000, 512, 256, 32, 256, 2), "scan_kernel<true>"),
]


@pytest.mark.parametrize("shape,kernel", ROUTES, ids=lambda v: v if isinstance(v, str) else "N%d_D%d_M%d_C%d_ldo%d_opt%d" % v)
def test_kernel_selection(mad, shape, kernel, options):
    """maddness_last_kernel() names the kernel a call launched; the routes the parity lists rely on."""
    import torch
    N, D, M, C, ldo, opt = shape
    options(mad.MADDNESS_OPT_KERNELS, opt)
    g = torch.Generator(device="cuda").manual_seed(1)
    A = torch.randn((N, D), device="cuda", generator=g)
    params = mad.Params(torch.randint(0, D, (C, 4), dtype=torch.int32, device="cuda", generator=g),
                        torch.randn((C, 16), device="cuda", generator=g))
    luts = torch.randint(0, 256, (C, 16, M), dtype=torch.uint8, device="cuda", generator=g)
    out = torch.empty((N, ldo), device="cuda")
    mad.maddness_encode_scan(params, A, luts, torch.ones(M, device="cuda"), torch.zeros(M, device="cuda"), out=out[:, :M])
    got = mad.maddness_last_kernel()
    torch.cuda.synchronize()
    assert got.startswith(kernel), got
    mad.maddness_encode_scan(params, A[:0], luts, torch.ones(M, device="cuda"), torch.zeros(M, device="cuda"))
    assert mad.maddness_last_kernel() == ""     # nothing launched


def _sampled_rows(rng, N, n_random):
    edge = np.concatenate([np.arange(0, 300), np.arange(N - 300, N)])
    return np.unique(np.concatenate([edge, rng.integers(0, N, n_random)]))


def test_parity_throughput_workload_full_size(mad):
    """Workload 4 at its full size (the launch that bench.py times): every code,
    accumulator and output of ~20000 sampled rows, against the oracle."""
    import torch
    from paper_2106_10860_amd.learn import learn
    w = wl.get_workload(4)
    model = learn(wl.make_A_train(w), w.subspaces)
    B = wl.make_B(w)
    print("workload", w.name, "learned", flush=True)
    A_d = torch.empty((w.N, w.D), dtype=torch.float32, device="cuda")
    rng = np.random.default_rng(4)
    rows = _sampled_rows(rng, w.N, 20000)
    A_rows = np.empty((rows.size, w.D), dtype=np.float32)
    for i in range(wl.n_chunks(w)):
        lo, hi = wl.chunk_rows(w, i)
        chunk = wl.make_A_chunk(w, i)
        A_d[lo:hi] = torch.from_numpy(chunk).cuda()
        sel = (rows >= lo) & (rows < hi)
        A_rows[sel] = chunk[rows[sel] - lo]
    print("A resident", flush=True)
    ref = oracle_pipeline(A_rows, model.split_dims, model.thresholds, model.prototypes, B)
    params = mad.Params.from_model(model)
    luts_d, scale_d, offset_d = mad.maddness_build_luts(params, dev(B))
    torch.cuda.synchronize()
    flips = compare_luts(luts_d.cpu().numpy(), scale_d.cpu().numpy(), offset_d.cpu().numpy(), ref,
                         model.prototypes, B)
    print("table bytes on a rounding boundary:", flips, flush=True)
    luts, scale, offset = dev(ref["luts"]), dev(ref["scale"]), dev(ref["offset"])
    out = torch.empty((w.N, w.M), dtype=torch.float32, device="cuda")
    acc = acc_buf(w.N, w.M)
    codes = torch.empty((w.N, w.C // 2), dtype=torch.uint8, device="cuda")
    mad.maddness_encode_scan(params, A_d, luts, scale, offset, out=out, acc=acc, codes=codes)
    torch.cuda.synchronize()
    idx = torch.from_numpy(rows).cuda()
    assert (codes[idx].cpu().numpy() == ref["packed"]).all()
    assert (acc_np(acc[idx]) == ref["acc"]).all()
    assert (out[idx].cpu().numpy() == ref["out"]).all()
    # the launch bench.py times: out only
    out2 = torch.empty_like(out)
    mad.maddness_encode_scan(params, A_d, luts, scale, offset, out=out2)
    assert mad.maddness_last_kernel().startswith("fused_mfma_kernel, A by rows")
    torch.cuda.synchronize()
    assert torch.equal(out, out2)
    # and the launch bench.py times beside it: the same call with the matrix-core kernels switched off
    # (tables in LDS, lookups and integer additions on the vector ALUs)
    mad.maddness_set_option(mad.MADDNESS_OPT_KERNELS, mad.MADDNESS_KERNELS_NO_MATRIX_CORES)
    try:
        out2.fill_(-1.0)
        mad.maddness_encode_scan(params, A_d, luts, scale, offset, out=out2)
        assert mad.maddness_last_kernel().startswith("rows_kernel")
        torch.cuda.synchronize()
        assert torch.equal(out, out2)
        out2.fill_(-1.0)
        codes_v = mad.maddness_encode(params, A_d)
        mad.maddness_scan(w.C, codes_v, luts, scale, offset, out=out2)
        assert mad.maddness_last_kernel().startswith("rows_kernel")
        torch.cuda.synchronize()
        assert torch.equal(out, out2) and torch.equal(codes_v, codes)
    finally:
        mad.maddness_set_option(mad.MADDNESS_OPT_KERNELS, mad.MADDNESS_KERNELS_AUTO)
    # properties that hold for every row: alpha acc + beta, and accumulator range
    assert int(acc.max()) <= 255 * w.C
    # (acc * scale is exact for a power-of-two scale, so mul-then-add rounds once, like an fma)
    recon = acc.to(torch.float32) * scale[None, :] + offset[None, :]
    assert torch.equal(recon, out)
    # the two-call path gives the same bits on all rows
    codes_b = mad.maddness_encode(params, A_d)
    out_b, _ = mad.maddness_scan(w.C, codes_b, luts, scale, offset)
    torch.cuda.synchronize()
    assert torch.equal(codes_b, codes) and torch.equal(out_b, out)
    # the error measure is the same number from both paths (same bytes in)
    Y = oracle.matmul_f64(A_rows, B)
    assert oracle.nmse(out[idx].cpu().numpy(), Y) == oracle.nmse(ref["out"], Y)


def test_parity_stress_workload_chunks(mad):
    """Workload 5's D, M, C (tables four times the size of LDS) on four of its 64
    chunks plus a ragged tail; the training set is cut to 8192 rows to keep the
    CPU set-up short."""
    import torch
    from paper_2106_10860_amd.learn import learn
    w = wl.get_workload(5)
    model = learn(wl.make_A_train(w)[:8192], w.subspaces)
    B = wl.make_B(w)
    print("workload", w.name, "learned", flush=True)
    chunks = [0, 63, 17, 42]
    parts = [wl.make_A_chunk(w, i) for i in chunks]
    parts.append(wl.make_A_chunk(w, 5)[:777])
    A = np.concatenate(parts)
    rng = np.random.default_rng(5)
    rows = _sampled_rows(rng, A.shape[0], 6000)
    ref = oracle_pipeline(A[rows], model.split_dims, model.thresholds, model.prototypes, B)
    params = mad.Params.from_model(model)
    luts_d, scale_d, offset_d = mad.maddness_build_luts(params, dev(B))
    torch.cuda.synchronize()
    compare_luts(luts_d.cpu().numpy(), scale_d.cpu().numpy(), offset_d.cpu().numpy(), ref,
                 model.prototypes, B)
    luts, scale, offset = dev(ref["luts"]), dev(ref["scale"]), dev(ref["offset"])
    A_d = dev(A)
    N = A.shape[0]
    out = torch.empty((N, w.M), dtype=torch.float32, device="cuda")
    acc = acc_buf(N, w.M)
    codes = torch.empty((N, w.C // 2), dtype=torch.uint8, device="cuda")
    mad.maddness_encode_scan(params, A_d, luts, scale, offset, out=out, acc=acc, codes=codes)
    torch.cuda.synchronize()
    idx = torch.from_numpy(rows).cuda()
    assert (codes[idx].cpu().numpy() == ref["packed"]).all()
    assert (acc_np(acc[idx]) == ref["acc"]).all()
    assert (out[idx].cpu().numpy() == ref["out"]).all()
    codes_b = mad.maddness_encode(params, A_d)
    out_b, _ = mad.maddness_scan(w.C, codes_b, luts, scale, offset)
    torch.cuda.synchronize()
    assert torch.equal(codes_b, codes) and torch.equal(out_b, out)


def _resident_A(w, sinks, rows):
    """Fills device tensors chunk by chunk from the workload's seeded generator (a few chunks
    drawn ahead on host threads).  sinks: list of (tensor [N][D], host conversion of an fp32
    chunk).  Returns the fp32 host rows `rows` (sorted row numbers)."""
    import torch
    from concurrent.futures import ThreadPoolExecutor
    A_rows = np.empty((rows.size, w.D), dtype=np.float32)
    n = wl.n_chunks(w)
    with ThreadPoolExecutor(4) as pool:
        pending = {i: pool.submit(wl.make_A_chunk, w, i) for i in range(min(6, n))}
        for i in range(n):
            chunk = pending.pop(i).result()
            if i + 6 < n:
                pending[i + 6] = pool.submit(wl.make_A_chunk, w, i + 6)
            lo, hi = wl.chunk_rows(w, i)
            for tensor, convert in sinks:
                tensor[lo:hi] = typed_dev(convert(chunk), "bf16" if tensor.dtype == torch.bfloat16 else "")
            sel = (rows >= lo) & (rows < hi)
            A_rows[sel] = chunk[rows[sel] - lo]
            if i % 8 == 7:
                print("  chunks resident:", i + 1, "of", n, flush=True)
    return A_rows


def _assert_dequantised(acc, scale, offset, out, bias=0):
    """out == fma(acc - bias, scale, offset) on every row, block by block ((acc - bias) * scale is
    exact for a power-of-two scale, so multiply-then-add rounds once, like the fma)."""
    import torch
    for lo in range(0, out.shape[0], 1 << 18):
        a = acc[lo:lo + (1 << 18)].to(torch.int32) & 0xFFFF
        recon = (a - bias).to(torch.float32) * scale[None, :] + offset[None, :]
        assert torch.equal(recon, out[lo:lo + (1 << 18)]), f"alpha acc + beta != out in rows from {lo}"


def test_parity_stress_workload_full_size(mad):
    """Workload 5 at its stated size, one launch of 2^22 rows (16 GiB in, 8 GiB out, byte offsets
    beyond 2^32 on both sides, several regions of the phased kernel): codes, accumulators and
    outputs of sampled rows of chunks 0, 17, 42 and 63 (and of random rows anywhere) against the
    oracle, and on ALL rows the identities out = alpha acc + beta and fused = encode then scan."""
    import torch
    from paper_2106_10860_amd.learn import learn
    w = wl.get_workload(5)
    model = learn(wl.make_A_train(w), w.subspaces)
    B = wl.make_B(w)
    print("workload", w.name, "learned", flush=True)
    rng = np.random.default_rng(55)
    picks = [np.arange(0, 300), np.arange(w.N - 300, w.N), rng.integers(0, w.N, 3000)]
    for c in (0, 17, 42, 63):
        lo, hi = wl.chunk_rows(w, c)
        picks += [rng.integers(lo, hi, 2500), np.arange(lo, lo + 40), np.arange(hi - 40, hi)]
    rows = np.unique(np.concatenate(picks))
    A_d = torch.empty((w.N, w.D), dtype=torch.float32, device="cuda")
    A_rows = _resident_A(w, [(A_d, lambda c: c)], rows)
    ref = oracle_pipeline(A_rows, model.split_dims, model.thresholds, model.prototypes, B)
    print("oracle done on", rows.size, "rows", flush=True)
    params = mad.Params.from_model(model)
    luts_d, scale_d, offset_d = mad.maddness_build_luts(params, dev(B))
    torch.cuda.synchronize()
    flips = compare_luts(luts_d.cpu().numpy(), scale_d.cpu().numpy(), offset_d.cpu().numpy(), ref,
                         model.prototypes, B)
    print("table bytes on a rounding boundary:", flips, flush=True)
    luts, scale, offset = dev(ref["luts"]), dev(ref["scale"]), dev(ref["offset"])
    out = torch.empty((w.N, w.M), dtype=torch.float32, device="cuda")
    acc = acc_buf(w.N, w.M)
    codes = torch.empty((w.N, w.C // 2), dtype=torch.uint8, device="cuda")
    mad.maddness_encode_scan(params, A_d, luts, scale, offset, out=out, acc=acc, codes=codes)
    torch.cuda.synchronize()
    idx = torch.from_numpy(rows).cuda()
    assert (codes[idx].cpu().numpy() == ref["packed"]).all()
    assert (acc_np(acc[idx]) == ref["acc"]).all()
    assert (out[idx].cpu().numpy() == ref["out"]).all()
    print("sampled rows agree with the oracle", flush=True)
    _assert_dequantised(acc, scale, offset, out)
    # the launch bench.py times: out only
    out2 = torch.empty_like(out)
    mad.maddness_encode_scan(params, A_d, luts, scale, offset, out=out2)
    torch.cuda.synchronize()
    assert torch.equal(out, out2)
    # the two-call path gives the same bits on all rows
    codes_b = mad.maddness_encode(params, A_d)
    mad.maddness_scan(w.C, codes_b, luts, scale, offset, out=out2)
    torch.cuda.synchronize()
    assert torch.equal(codes_b, codes) and torch.equal(out2, out)
    Y = oracle.matmul_f64(A_rows, B)
    assert oracle.nmse(out[idx].cpu().numpy(), Y) == oracle.nmse(ref["out"], Y)
    del A_d, out, out2, acc, codes, codes_b
    torch.cuda.empty_cache()


def test_parity_input_variants_and_averaged_full_size(mad):
    """The launches bench.py times beside the headline at N = 2^20 (workload 4): narrow element
    types by rows, A stored by columns, and the aggregation by pairwise averages.  Sampled rows
    against the oracle on the same bytes; on all rows fused = encode then scan and
    out = alpha acc + beta."""
    import torch
    from paper_2106_10860_amd.learn import learn
    w = wl.get_workload(4)
    model = learn(wl.make_A_train(w), w.subspaces)
    B = wl.make_B(w)
    print("workload", w.name, "learned", flush=True)
    rng = np.random.default_rng(44)
    rows = _sampled_rows(rng, w.N, 12000)
    to_host = {"f32": lambda c: c, "f16": lambda c: c.astype(np.float16),
               "bf16": lambda c: (c.view(np.uint32) >> 16).astype(np.uint16),
               "u8": lambda c: np.clip(np.rint(c * 32.0), 0, 255).astype(np.uint8)}
    tdt = {"f32": torch.float32, "f16": torch.float16, "bf16": torch.bfloat16, "u8": torch.uint8}
    A_dev = {k: torch.empty((w.N, w.D), dtype=tdt[k], device="cuda") for k in to_host}
    A_rows = _resident_A(w, [(A_dev[k], to_host[k]) for k in to_host], rows)
    luts_h, scale_h, offset_h, _, _ = oracle.quantize_luts(oracle.build_luts_f64(model.prototypes, B))
    luts, scale, offset = dev(luts_h), dev(scale_h), dev(offset_h)
    params = mad.Params.from_model(model)
    idx = torch.from_numpy(rows).cuda()
    out = torch.empty((w.N, w.M), dtype=torch.float32, device="cuda")
    out_b = torch.empty_like(out)
    acc = acc_buf(w.N, w.M)
    for dtype, col_major in (("f16", False), ("bf16", False), ("u8", False), ("f32", True), ("f16", True)):
        what = f"{dtype} {'by columns' if col_major else 'by rows'}"
        print("variant", what, flush=True)
        typed_rows = to_host[dtype](A_rows)
        want_codes = oracle.pack(oracle.encode_typed(typed_rows, dtype, False, model.split_dims, model.thresholds))
        want_out, want_acc, ov = oracle.scan(want_codes, w.C, luts_h, scale_h, offset_h)
        assert ov == 0
        X = A_dev[dtype].t().contiguous() if col_major else A_dev[dtype]
        codes = torch.zeros((w.N, w.C // 2), dtype=torch.uint8, device="cuda")
        out.fill_(-1.0)
        mad.maddness_encode_scan_typed(params, X, luts, scale, offset, col_major=col_major, out=out, acc=acc, codes=codes)
        torch.cuda.synchronize()
        assert (codes[idx].cpu().numpy() == want_codes).all(), f"{what}: codes differ"
        assert (acc_np(acc[idx]) == want_acc).all(), f"{what}: accumulators differ"
        assert (out[idx].cpu().numpy() == want_out).all(), f"{what}: out not bit-identical"
        _assert_dequantised(acc, scale, offset, out)
        # what bench.py times: out only; and encode alone, then scan
        mad.maddness_encode_scan_typed(params, X, luts, scale, offset, col_major=col_major, out=out_b)
        torch.cuda.synchronize()
        assert torch.equal(out, out_b), f"{what}: out-only launch differs"
        codes_b = mad.maddness_encode_typed(params, X, col_major=col_major)
        mad.maddness_scan(w.C, codes_b, luts, scale, offset, out=out_b)
        torch.cuda.synchronize()
        assert torch.equal(codes_b, codes) and torch.equal(out_b, out), f"{what}: two calls differ from the fused one"
        del X
    # aggregation by pairwise averages (Appendix D) on the fp32 rows
    print("variant averaged", flush=True)
    want_codes = oracle.pack(oracle.encode(A_rows, model.split_dims, model.thresholds))
    want_out, want_usum = oracle.scan_averaged(want_codes, w.C, luts_h, scale_h, offset_h)
    codes = torch.zeros((w.N, w.C // 2), dtype=torch.uint8, device="cuda")
    mad.maddness_encode_scan_averaged(params, A_dev["f32"], luts, scale, offset, out=out, acc=acc, codes=codes)
    torch.cuda.synchronize()
    assert (codes[idx].cpu().numpy() == want_codes).all()
    assert (acc_np(acc[idx]) == want_usum).all(), "averaged: 16 x sum of block averages differs"
    assert (out[idx].cpu().numpy() == want_out).all(), "averaged: out not bit-identical"
    _assert_dequantised(acc, scale, offset, out, bias=w.C)
    mad.maddness_scan_averaged(w.C, codes, luts, scale, offset, out=out_b)
    torch.cuda.synchronize()
    assert torch.equal(out, out_b), "averaged: scan of the codes differs from the fused call"
    mad.maddness_encode_scan_averaged(params, A_dev["f32"], luts, scale, offset, out=out_b)
    torch.cuda.synchronize()
    assert torch.equal(out, out_b), "averaged: out-only launch differs"
    del A_dev, out, out_b, acc
    torch.cuda.empty_cache()


# ---------------------------------------------------------------------------
# aggregation by pairwise averages (Appendix D)
# ---------------------------------------------------------------------------

# (N, D, M, C): every kernel that has an averaged form - row kernels (C = 16 / 32,
# 64 < M <= 256), the column-tiled kernel (C = 64), the general kernel (the rest:
# narrow or ragged M, C = 48 / 256, unaligned rows).
AVG_SHAPES = [
    (515, 512, 256, 32),
    (4099, 256, 128, 32),
    (1000, 64, 200, 16),
    (777, 128, 100, 32),
    (300, 27, 10, 16),
    (200, 96, 70, 48),
    (600, 1024, 512, 64),
    (450, 64, 400, 64),
    (130, 40, 64, 256),
    (1030, 512, 1030, 32),
]


@pytest.mark.parametrize("shape", AVG_SHAPES, ids=lambda s: "N%d_D%d_M%d_C%d" % s)
@pytest.mark.parametrize("general_only", [False, True], ids=["auto", "general"])
def test_parity_averaged(mad, shape, general_only, options):
    import torch
    N, D, M, C = shape
    print("case averaged", shape, general_only, flush=True)
    if general_only:
        options(mad.MADDNESS_OPT_KERNELS, mad.MADDNESS_KERNELS_GENERAL)
    rng = np.random.default_rng(N + 3 * C)
    _, A, B = wl.random_problem(N * 5 + M, N, D, M, latent=min(8, D), N_train=4)
    sd, th = random_trees(rng, A, C)
    P = rng.standard_normal((C, 16, D)).astype(np.float32)
    ref = oracle_pipeline(A, sd, th, P, B)
    # full-range bytes as well as the learned-looking tables: the rounding of the
    # averages depends on the low bits
    for luts_h in (ref["luts"], rng.integers(0, 256, size=ref["luts"].shape, dtype=np.uint8)):
        want_out, want_usum = oracle.scan_averaged(ref["packed"], C, luts_h, ref["scale"], ref["offset"])
        luts, scale, offset = dev(luts_h), dev(ref["scale"]), dev(ref["offset"])
        params = mad.Params(dev(sd), dev(th), dev(P))
        out, acc = mad.maddness_scan_averaged(C, dev(ref["packed"]), luts, scale, offset, acc=acc_buf(N, M))
        torch.cuda.synchronize()
        assert (acc_np(acc) == want_usum).all(), "averaged scan: 16 x sum of block averages differs"
        assert (out.cpu().numpy() == want_out).all(), "averaged scan: out not bit-identical"
        acc2 = acc_buf(N, M)
        codes2 = torch.zeros((N, (C + 1) // 2), dtype=torch.uint8, device="cuda")
        out2 = mad.maddness_encode_scan_averaged(params, dev(A), luts, scale, offset, acc=acc2, codes=codes2)
        torch.cuda.synchronize()
        assert (codes2.cpu().numpy() == ref["packed"]).all(), "averaged fused: codes differ"
        assert (acc_np(acc2) == want_usum).all(), "averaged fused: 16 x sum of block averages differs"
        assert (out2.cpu().numpy() == want_out).all(), "averaged fused: out not bit-identical"
        # without the optional outputs
        out3 = mad.maddness_encode_scan_averaged(params, dev(A), luts, scale, offset)
        torch.cuda.synchronize()
        assert (out3.cpu().numpy() == want_out).all()


def test_averaged_rejects_partial_blocks(mad):
    import torch
    N, D, M, C = 64, 32, 16, 24
    rng = np.random.default_rng(5)
    A = rng.standard_normal((N, D)).astype(np.float32)
    sd, th = random_trees(rng, A, C)
    params = mad.Params(dev(sd), dev(th))
    luts = torch.zeros((C, 16, M), dtype=torch.uint8, device="cuda")
    scale = torch.ones(M, device="cuda")
    offset = torch.zeros(M, device="cuda")
    codes = torch.zeros((N, C // 2), dtype=torch.uint8, device="cuda")
    with pytest.raises(mad.MaddnessError) as e:
        mad.maddness_scan_averaged(C, codes, luts, scale, offset)
    assert e.value.status == mad.MADDNESS_E_UNSUPPORTED
    with pytest.raises(mad.MaddnessError) as e:
        mad.maddness_encode_scan_averaged(params, dev(A), luts, scale, offset)
    assert e.value.status == mad.MADDNESS_E_UNSUPPORTED


# ---------------------------------------------------------------------------
# narrow element types and inputs stored by columns (Section 4.1; Appendix E.6)
# ---------------------------------------------------------------------------

def typed_copy(A32, dtype, rng):
    """The same matrix in a narrower storage type: (host array for the oracle, torch dtype view)."""
    if dtype == "f32":
        return A32.copy()
    if dtype == "f16":
        return A32.astype(np.float16)
    if dtype == "bf16":
        return (A32.view(np.uint32) >> 16).astype(np.uint16)          # bit patterns, truncated
    return np.clip(np.rint(A32 * 40.0 + rng.integers(0, 3, size=A32.shape)), 0, 255).astype(np.uint8)


def typed_dev(a, dtype):
    import torch
    if dtype == "bf16":
        return torch.from_numpy(a.view(np.int16)).cuda().view(torch.bfloat16)
    return torch.from_numpy(a).cuda()


# (N, D, M, C, pad): rows of 16-byte pieces with C = 32 (row kernels for narrow types), many rows
# (column kernels: a wavefront takes 64 rows), and shapes only the general kernels take.
TYPED_SHAPES = [
    (70001, 64, 128, 32, 3),      # by columns: N % 4 = 1 with a column stride of 70004
    (65600, 48, 256, 16, 4),
    (66000, 32, 8, 64, 0),
    (5000, 512, 256, 32, 0),
    (20000, 512, 256, 32, 0),     # narrow rows, many: phased kernel with the scan on the matrix cores
    (66000, 32, 300, 64, 0),      # C = 64, two passes of 256 columns, by rows and by columns
    (17000, 1024, 100, 64, 0),    # C = 64, rows of 2 KiB (fp16) / 1 KiB (uint8)
    (16500, 1024, 200, 32, 16),
    (16400, 2048, 68, 64, 0),     # rows of 8 KiB (fp32), 4 KiB (fp16) and 2 KiB (uint8)
    (16400, 4096, 36, 32, 0),     # uint8 rows of 4 KiB; wider types: the general kernels
    (4500, 1024, 200, 32, 16),
    (777, 27, 10, 5, 3),
    (300, 40, 300, 33, 0),
]


# every shape with the library's own choice of kernels (run 0); the run length of the column kernels on the
# vector ALUs (1, 2, 4 rows per lane) only where it matters: many rows, tables in LDS
TYPED_CASES = [pytest.param(s, r, id="N%d_D%d_M%d_C%d_p%d-%s" % (*s, "run%d" % r if r else "auto"))
               for s in TYPED_SHAPES for r in (0, 1, 2, 4) if r == 0 or (s[0] >= 65536 and s[2] > 64)]


@pytest.mark.parametrize("shape,run", TYPED_CASES)
@pytest.mark.parametrize("dtype", ["f32", "f16", "bf16", "u8"])
def test_parity_typed_and_column_major(mad, shape, dtype, run, options):
    import torch
    N, D, M, C, pad = shape
    print("case typed", shape, dtype, run, flush=True)
    # "auto": the library's own choice (many rows: the scan on the matrix cores); "runN": the
    # column kernels on the vector ALUs with N rows per lane
    if run:
        options(mad.MADDNESS_OPT_COLS_RUN, run)
        options(mad.MADDNESS_OPT_KERNELS, mad.MADDNESS_KERNELS_NO_MATRIX_CORES)
    rng = np.random.default_rng(N + D + C)
    _, A32, B = wl.random_problem(N + 11 * D, N, D, M, latent=min(8, D), N_train=4)
    A_h = typed_copy(A32, dtype, rng)
    values = oracle.widen(A_h, dtype)
    sd, th = random_trees(rng, values, C)
    P = rng.standard_normal((C, 16, D)).astype(np.float32)
    want_codes = oracle.pack(oracle.encode_typed(A_h, dtype, False, sd, th))
    assert (want_codes == oracle.pack(oracle.encode(values, sd, th))).all()
    luts_h, scale_h, offset_h, _, _ = oracle.quantize_luts(oracle.build_luts_f64(P, B))
    want_out, want_acc, ov = oracle.scan(want_codes, C, luts_h, scale_h, offset_h)
    assert ov == 0
    params = mad.Params(dev(sd), dev(th), dev(P))
    luts, scale, offset = dev(luts_h), dev(scale_h), dev(offset_h)
    for col_major in (False, True):
        # leading dimension with padding: rows of D + pad, or columns of N + pad elements
        host = np.ascontiguousarray(A_h.T) if col_major else A_h
        full = torch.zeros((host.shape[0], host.shape[1] + pad), dtype=typed_dev(host[:1, :1], dtype).dtype,
                           device="cuda")
        full[:, :host.shape[1]] = typed_dev(host, dtype)
        A_d = full[:, :host.shape[1]]
        what = f"{shape} {dtype} {'by columns' if col_major else 'by rows'}"
        codes = mad.maddness_encode_typed(params, A_d, col_major=col_major)
        torch.cuda.synchronize()
        assert (codes.cpu().numpy() == want_codes).all(), f"{what}: codes differ"
        acc = acc_buf(N, M)
        codes2 = torch.zeros_like(codes)
        out = mad.maddness_encode_scan_typed(params, A_d, luts, scale, offset, col_major=col_major, acc=acc,
                                             codes=codes2)
        torch.cuda.synchronize()
        assert (codes2.cpu().numpy() == want_codes).all(), f"{what}: fused codes differ"
        assert (acc_np(acc) == want_acc).all(), f"{what}: fused accumulators differ"
        assert (out.cpu().numpy() == want_out).all(), f"{what}: fused out not bit-identical"
        out3 = mad.maddness_encode_scan_typed(params, A_d, luts, scale, offset, col_major=col_major)
        torch.cuda.synchronize()
        assert (out3.cpu().numpy() == want_out).all(), f"{what}: fused out without acc/codes differs"


@pytest.mark.parametrize("shape", [(70001, 64, 128, 32, 3), (66000, 32, 300, 64, 0), (20000, 512, 256, 32, 0)],
                         ids=lambda s: "N%d_D%d_M%d_C%d_p%d" % s)
@pytest.mark.parametrize("dtype", ["f32", "f16", "u8"])
def test_parity_typed_phased_kernel_many_blocks(mad, shape, dtype, options):
    """The phased kernel on narrow rows and on A stored by columns with three workgroups and the
    fewest rows per region: every workgroup takes many blocks in turn (codes area reused, the
    barrier after the scan), the last block is ragged and some wavefronts get no rows in it."""
    import torch
    N, D, M, C, pad = shape
    print("case typed blocks", shape, dtype, flush=True)
    options(mad.MADDNESS_OPT_MAX_WORKGROUPS, 3)
    rng = np.random.default_rng(N + D + C + 1)
    _, A32, B = wl.random_problem(N + 13 * D, N, D, M, latent=min(8, D), N_train=4)
    A_h = typed_copy(A32, dtype, rng)
    values = oracle.widen(A_h, dtype)
    sd, th = random_trees(rng, values, C)
    P = rng.standard_normal((C, 16, D)).astype(np.float32)
    want_codes = oracle.pack(oracle.encode_typed(A_h, dtype, False, sd, th))
    luts_h, scale_h, offset_h, _, _ = oracle.quantize_luts(oracle.build_luts_f64(P, B))
    want_out, want_acc, ov = oracle.scan(want_codes, C, luts_h, scale_h, offset_h)
    assert ov == 0
    params = mad.Params(dev(sd), dev(th), dev(P))
    luts, scale, offset = dev(luts_h), dev(scale_h), dev(offset_h)
    for col_major in (False, True):
        # by rows: 6 rows per wavefront and region; by columns: 256 (the unit of that encoder)
        options(mad.MADDNESS_OPT_PHASED_ROWS, 256 if col_major else 6)
        host = np.ascontiguousarray(A_h.T) if col_major else A_h
        full = torch.zeros((host.shape[0], host.shape[1] + pad), dtype=typed_dev(host[:1, :1], dtype).dtype,
                           device="cuda")
        full[:, :host.shape[1]] = typed_dev(host, dtype)
        A_d = full[:, :host.shape[1]]
        what = f"{shape} {dtype} {'by columns' if col_major else 'by rows'}"
        acc = acc_buf(N, M)
        codes = torch.zeros((N, C // 2), dtype=torch.uint8, device="cuda")
        out = mad.maddness_encode_scan_typed(params, A_d, luts, scale, offset, col_major=col_major, acc=acc,
                                             codes=codes)
        torch.cuda.synchronize()
        assert (codes.cpu().numpy() == want_codes).all(), f"{what}: fused codes differ"
        assert (acc_np(acc) == want_acc).all(), f"{what}: fused accumulators differ"
        assert (out.cpu().numpy() == want_out).all(), f"{what}: fused out not bit-identical"
        out3 = mad.maddness_encode_scan_typed(params, A_d, luts, scale, offset, col_major=col_major)
        torch.cuda.synchronize()
        assert (out3.cpu().numpy() == want_out).all(), f"{what}: fused out without acc/codes differs"


def test_typed_every_bit_pattern(mad):
    """All 65536 binary16 and bfloat16 patterns and all bytes through the encoder (subnormals,
    infinities, NaNs, signed zeros), thresholds drawn from the same patterns."""
    import torch
    rng = np.random.default_rng(99)
    for dtype, count in (("f16", 65536), ("bf16", 65536), ("u8", 256)):
        bits = np.arange(count, dtype=np.uint16 if count > 256 else np.uint8)
        D, C = 16, 32
        N = 65536        # enough rows for the column kernels (a wavefront takes 64 rows)
        A_h = rng.permutation(np.tile(bits, N * D // count)).reshape(N, D)
        if dtype == "f16":
            A_h = A_h.view(np.float16)
        values = oracle.widen(A_h, dtype)
        sd = rng.integers(0, D, size=(C, 4)).astype(np.int32)
        th = values[rng.integers(0, N, size=(C, 16)), rng.integers(0, D, size=(C, 16))].astype(np.float32)
        th[np.isnan(th)] = 0.0
        want = oracle.pack(oracle.encode_typed(A_h, dtype, False, sd, th))
        params = mad.Params(dev(sd), dev(th))
        for col_major in (False, True):
            host = np.ascontiguousarray(A_h.T) if col_major else A_h
            got = mad.maddness_encode_typed(params, typed_dev(host, dtype), col_major=col_major)
            torch.cuda.synchronize()
            assert (got.cpu().numpy() == want).all(), (dtype, col_major)


def test_typed_rejects_bad_arguments(mad):
    import torch
    import ctypes
    N, D, C = 64, 32, 8
    rng = np.random.default_rng(6)
    A = rng.standard_normal((N, D)).astype(np.float32)
    sd, th = random_trees(rng, A, C)
    params = mad.Params(dev(sd), dev(th))
    A_d = dev(A)
    codes = torch.zeros((N, C // 2), dtype=torch.uint8, device="cuda")
    p = params.c_struct(D)
    L = mad.lib()
    assert L.maddness_encode_typed(ctypes.byref(p), A_d.data_ptr(), 7, 0, N, D, codes.data_ptr(), None) == mad.MADDNESS_E_INVAL
    assert L.maddness_encode_typed(ctypes.byref(p), A_d.data_ptr(), 0, 2, N, D, codes.data_ptr(), None) == mad.MADDNESS_E_INVAL
    # stored by columns: the leading dimension is the column stride and must cover N
    assert L.maddness_encode_typed(ctypes.byref(p), A_d.data_ptr(), 0, 1, N, N - 1, codes.data_ptr(), None) == mad.MADDNESS_E_INVAL
    # binary16 data at an odd address
    assert L.maddness_encode_typed(ctypes.byref(p), A_d.data_ptr() + 1, 1, 0, N, D, codes.data_ptr(), None) == mad.MADDNESS_E_ALIGN


# ---------------------------------------------------------------------------
# the exact scan on the matrix cores (many rows, C a multiple of 8 up to 64)
# ---------------------------------------------------------------------------

MFMA_SHAPES = [
    (16384, 4, 8), (20001, 100, 16), (16400, 256, 24), (30000, 256, 32), (17000, 300, 32), (16385, 64, 32),
    (16500, 130, 40), (18000, 512, 48), (16390, 34, 56), (20000, 512, 64), (16384, 1000, 64), (70000, 16, 16),
    (16400, 200, 64),   # an odd number of 16-row groups where two are taken per step
    # any other shape of many rows: the same kernel padded to 16 / 32 / 64 codebooks, codes and tables read byte by
    # byte, rows written with 4-byte stores
    (20000, 250, 30), (16400, 257, 31), (16390, 130, 5), (17000, 18, 33), (16500, 1030, 17), (16385, 66, 63),
    (262144 + 3, 100, 12),
]


@pytest.mark.parametrize("shape", MFMA_SHAPES, ids=lambda s: "N%d_M%d_C%d" % s)
@pytest.mark.parametrize("vector_only", [False, True], ids=["matrix", "vector"])
def test_scan_on_matrix_cores(mad, shape, vector_only, options):
    """Random codes and full-range table bytes: the int8 matrix-core scan (and, with the
    switch set, the vector-ALU kernels on the same inputs) against the oracle's exact sum."""
    import torch
    N, M, C = shape
    print("case matrix-core scan", shape, vector_only, flush=True)
    if vector_only:
        options(mad.MADDNESS_OPT_KERNELS, mad.MADDNESS_KERNELS_NO_MATRIX_CORES)
    rng = np.random.default_rng(N + M + C)
    packed = oracle.pack(rng.integers(0, 16, size=(N, C), dtype=np.uint8))
    luts_h = rng.integers(0, 256, size=(C, 16, M), dtype=np.uint8)
    luts_h[:, :, 0] = 255                       # the largest possible sums in one column
    if M > 1:
        luts_h[:, :, 1] = 0
    scale_h = (2.0 ** rng.integers(-6, 3, size=M)).astype(np.float32)
    offset_h = rng.standard_normal(M).astype(np.float32)
    want_out, want_acc, ov = oracle.scan(packed, C, luts_h, scale_h, offset_h)
    assert ov == 0
    ldo = M + (4 - M % 4) % 4 + 4 if (C % 8 == 0 and M % 4 == 0) else M + 1
    full = torch.full((N, ldo), -3.0, dtype=torch.float32, device="cuda")
    view = full[:, :M]
    acc = acc_buf(N, M)
    mad.maddness_scan(C, dev(packed), dev(luts_h), dev(scale_h), dev(offset_h), out=view, acc=acc)
    torch.cuda.synchronize()
    assert (acc_np(acc) == want_acc).all(), "accumulators differ"
    assert (view.cpu().numpy() == want_out).all(), "out not bit-identical"
    assert (full[:, M:] == -3.0).all(), "wrote outside the output columns"
    if not vector_only:
        assert "mfma_scan_kernel" in mad.maddness_last_kernel()
    out2, _ = mad.maddness_scan(C, dev(packed), dev(luts_h), dev(scale_h), dev(offset_h))
    torch.cuda.synchronize()
    assert (out2.cpu().numpy() == want_out).all()
    _, acc3 = mad.maddness_scan(C, dev(packed), dev(luts_h), dev(scale_h), dev(offset_h), acc=acc_buf(N, M), want_out=False)
    torch.cuda.synchronize()
    assert (acc_np(acc3) == want_acc).all(), "accumulators without fp32 output differ"


@pytest.mark.parametrize("seed", [11, 12, 13])
def test_selected_kernels_against_general_kernels_on_random_shapes(mad, seed, options):
    """Many random valid shapes (sizes around the kernels' switch points, strides, optional outputs,
    element types, storage orders): whatever kernel the library selects gives the bits of its general
    kernels, which the tests above hold against the oracle."""
    import torch
    rng = np.random.default_rng(seed)
    dtypes = [torch.float32, torch.float32, torch.float16, torch.bfloat16, torch.uint8]
    for case in range(120):
        C = int(rng.choice([8, 16, 24, 32, 40, 48, 56, 64, 12, 30]))
        D = int(rng.choice([64, 96, 128, 256, 320, 512, 516, 1000, 1024, 2048, 130]))
        D = max(D, 4 * C)
        M = int(rng.choice([4, 16, 36, 64, 100, 128, 132, 200, 256, 260, 300, 448, 452, 512, 516, 640, 1000, 1024]))
        N = int(rng.choice([16384, 16385 + int(rng.integers(0, 5000)), 70000 + int(rng.integers(0, 3)),
                            262144 + int(rng.integers(0, 40))]))
        if N * (D + M) > 3e8:
            N = 16384 + int(rng.integers(0, 3000))
        dt = dtypes[int(rng.integers(0, len(dtypes)))]
        col = bool(rng.random() < 0.3)
        if col:
            N -= N % 4 if rng.random() < 0.5 else 0
        ldo = M + int(rng.choice([0, 0, 4, 28, 60]))
        if rng.random() < 0.3:
            ldo = (M + 31) // 32 * 32
        want_acc, want_codes = bool(rng.random() < 0.5), bool(rng.random() < 0.5)
        print("case", seed, case, N, D, M, C, dt, col, ldo, want_acc, want_codes, flush=True)
        g = torch.Generator(device="cuda").manual_seed(int(rng.integers(0, 1 << 30)))
        pad = int(rng.choice([0, 16]))
        base = torch.randn((D, N + pad) if col else (N, D + pad), device="cuda", generator=g)
        if dt == torch.uint8:
            base = (base * 40 + 128).clamp(0, 255)
        base = base.to(dt)
        A = base[:, :N] if col else base[:, :D]
        sd = torch.randint(0, D, (C, 4), dtype=torch.int32, device="cuda", generator=g)
        th = torch.randn((C, 16), device="cuda", generator=g) * 0.7 + (128 if dt == torch.uint8 else 0)
        luts = torch.randint(0, 256, (C, 16, M), dtype=torch.uint8, device="cuda", generator=g)
        scale = 2.0 ** torch.randint(-5, 3, (M,), device="cuda", generator=g).float()
        offset = torch.randn(M, device="cuda", generator=g)
        params = mad.Params(sd, th)

        def run():
            out = torch.full((N, ldo), -5.0, device="cuda")
            acc = acc_buf(N, M) if want_acc else None
            codes = torch.zeros((N, (C + 1) // 2), dtype=torch.uint8, device="cuda") if want_codes else None
            mad.maddness_encode_scan_typed(params, A, luts, scale, offset, col_major=col, out=out[:, :M], acc=acc, codes=codes)
            enc = mad.maddness_encode_typed(params, A, col_major=col)
            out_s = torch.full((N, ldo), -5.0, device="cuda")
            mad.maddness_scan(C, enc, luts, scale, offset, out=out_s[:, :M])
            out_a = out_sa = None
            if C % 16 == 0 and dt == torch.float32 and not col:   # the averaged aggregation
                out_a = torch.full((N, ldo), -5.0, device="cuda")
                mad.maddness_encode_scan_averaged(params, A, luts, scale, offset, out=out_a[:, :M])
                out_sa = torch.full((N, ldo), -5.0, device="cuda")
                mad.maddness_scan_averaged(C, enc, luts, scale, offset, out=out_sa[:, :M])
            torch.cuda.synchronize()
            return out, acc, codes, enc, out_s, out_a, out_sa

        options(mad.MADDNESS_OPT_KERNELS, mad.MADDNESS_KERNELS_AUTO)
        got = run()
        options(mad.MADDNESS_OPT_KERNELS, mad.MADDNESS_KERNELS_GENERAL)
        want = run()
        options(mad.MADDNESS_OPT_KERNELS, mad.MADDNESS_KERNELS_AUTO)
        for name, x, y in zip(("fused out", "acc", "fused codes", "codes", "scan out", "averaged fused out",
                               "averaged scan out"), got, want):
            if x is not None:
                assert torch.equal(x.view(torch.int32) if x.dtype == torch.float32 else x,
                                   y.view(torch.int32) if y.dtype == torch.float32 else y), f"{name} differs"
        assert torch.equal(got[0].view(torch.int32), got[4].view(torch.int32)), "fused and two-call outputs differ"



def _random_many_row_shapes(n, seed):
    """Seeded shapes of many rows off every grid: D, M, C, pitches and the alignment of `out` drawn at random."""
    rng = np.random.default_rng(seed)
    shapes = []
    for _ in range(n):
        C = int(rng.integers(1, 65))
        D = int(rng.integers(max(128, C), 1200))
        M = int(rng.choice([rng.integers(17, 130), rng.integers(130, 520), rng.integers(520, 1100)]))
        N = int(rng.integers(16384, 21000))
        lda_pad = int(rng.choice([0, 0, 1, 2, 3, 5]))
        ldo_pad = int(rng.choice([0, 0, 0, 1, 3, 6]))
        out_off = int(rng.integers(0, 4))        # floats: `out` starts on any 4-byte boundary
        shapes.append((N, D, M, C, lda_pad, ldo_pad, out_off))
    return shapes


@pytest.mark.parametrize("shape", _random_many_row_shapes(20, 2024), ids=lambda s: "N%d_D%d_M%d_C%d_p%d_%d_o%d" % s)
def test_parity_random_shapes_of_many_rows(mad, shape):
    """The any-shape forms of the phased and the scan kernel (and whatever else the library picks) on drawn
    shapes, with `out` at any 4-byte alignment inside a buffer whose other floats must stay untouched."""
    import torch
    N, D, M, C, lda_pad, ldo_pad, out_off = shape
    print("case random many rows", shape, flush=True)
    rng = np.random.default_rng(N + D + M + C)
    _, A, B = wl.random_problem(N + D, N, D, M, latent=8, N_train=4)
    sd, th = random_trees(rng, A, C)
    luts_h = rng.integers(0, 256, size=(C, 16, M)).astype(np.uint8)
    scale_h = np.ldexp(np.ones(M, np.float32), rng.integers(-6, 3, size=M)).astype(np.float32)
    offset_h = rng.standard_normal(M).astype(np.float32)
    want_out, want_acc, want_packed = oracle.encode_scan(A, sd, th, luts_h, scale_h, offset_h)
    A_d = torch.zeros((N, D + lda_pad), dtype=torch.float32, device="cuda")
    A_d[:, :D] = dev(A)
    params = mad.Params(dev(sd), dev(th))
    luts, scale, offset = dev(luts_h), dev(scale_h), dev(offset_h)
    ldo = M + ldo_pad
    guard = 64

    def fresh():
        flat = torch.full((guard + out_off + N * ldo + guard,), -7.0, dtype=torch.float32, device="cuda")
        view = flat[guard + out_off: guard + out_off + N * ldo].view(N, ldo)[:, :M]
        return flat, view

    def check(flat, view, what):
        torch.cuda.synchronize()
        assert (view.cpu().numpy() == want_out).all(), f"{shape}: {what} out not bit-identical"
        body = flat[guard + out_off: guard + out_off + N * ldo].view(N, ldo)
        assert (flat[:guard + out_off] == -7.0).all() and (flat[guard + out_off + N * ldo:] == -7.0).all(), \
            f"{shape}: {what} wrote before or after `out`"
        if ldo_pad:
            assert (body[:, M:] == -7.0).all(), f"{shape}: {what} wrote into the padding of `out`"

    flat, view = fresh()
    codes = torch.zeros((N, (C + 1) // 2), dtype=torch.uint8, device="cuda")
    mad.maddness_encode_scan(params, A_d[:, :D], luts, scale, offset, out=view, codes=codes)
    check(flat, view, f"fused ({mad.maddness_last_kernel()})")
    assert (codes.cpu().numpy() == want_packed).all(), f"{shape}: fused codes differ"
    flat, view = fresh()
    acc = acc_buf(N, M)
    mad.maddness_scan(C, codes, luts, scale, offset, out=view, acc=acc)
    check(flat, view, f"scan ({mad.maddness_last_kernel()})")
    assert (acc_np(acc) == want_acc).all(), f"{shape}: scan accumulators differ"
