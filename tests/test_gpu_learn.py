"""GPU parity of the learning step (maddness_learn_trees / maddness_learn_prototypes, called
through the C ABI) against the oracle's plain statement of Algorithms 2-4 and of the ridge
step on the same seeded training matrices.  Split columns and training codes are integers
and must be equal; thresholds are fp32 midpoints of two data values and must be equal; the
prototypes come out of an fp64 Cholesky solve whose operations run in the oracle's order
and are compared to 1e-6 relative (of the largest entry), with the number of entries that
differ at all reported."""
import ctypes

import numpy as np
import pytest

import oracle
import workloads as wl

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def mad():
    import torch
    import paper_2106_10860_amd as m
    assert torch.cuda.is_available()
    m.lib()
    return m


def dev(x):
    import torch
    return torch.from_numpy(np.ascontiguousarray(x)).cuda()


def check_against_oracle(mad, A, subspaces, label, lda_pad=0, lam=1.0):
    import torch
    N, D = A.shape
    full = torch.zeros((N, D + lda_pad), dtype=torch.float32, device="cuda")
    full[:, :D] = dev(A)
    A_d = full[:, :D]
    sd, th, codes = mad.maddness_learn_trees(A_d, subspaces)
    torch.cuda.synchronize()
    want_sd, want_th, want_codes, _ = oracle.learn_trees(A, subspaces)
    assert (sd.cpu().numpy() == want_sd).all(), f"{label}: split columns differ\n{sd.cpu().numpy()}\n{want_sd}"
    assert (th.cpu().numpy() == want_th).all(), f"{label}: thresholds differ"
    assert (codes.cpu().numpy() == want_codes).all(), f"{label}: training codes differ"
    for ridge in (True, False):
        P = mad.maddness_learn_prototypes(codes, A_d, subspaces, ridge=ridge, lam=lam)
        torch.cuda.synchronize()
        want = oracle.ridge_prototypes(want_codes, A, lam) if ridge else oracle.bucket_means(want_codes, A, subspaces)
        got = P.cpu().numpy()
        tol = 1e-6 * max(np.abs(want).max(), 1e-30)
        assert np.abs(got - want).max() <= tol, f"{label}: prototypes (ridge={ridge}) differ by {np.abs(got - want).max()}"
        print(f"{label}: ridge={ridge}: {(got != want.astype(np.float32)).sum()} of {got.size} prototype entries "
              "differ from the oracle's fp32 rounding", flush=True)
    return sd, th, codes


def even(D, C):
    w = D // C
    return [(c * w, (c + 1) * w) for c in range(C)]


SMALL = [
    # (seed, N, D, subspaces, kind, lda_pad)
    (1, 300, 24, [(0, 8), (8, 16), (16, 24)], "relu", 0),
    (2, 1000, 27, [(0, 7), (7, 14), (14, 21), (21, 27)], "integers", 5),      # the image workload's subspaces
    (3, 65, 10, [(0, 2), (2, 3), (3, 5), (5, 10)], "integers", 0),            # widths 2, 1, 2, 5; one tile + 1 row
    (4, 4097, 64, even(64, 8), "relu", 0),                                    # a row more than a power of two
    (5, 8192, 32, even(32, 2), "normal", 3),                                  # exactly one sort chunk
    (6, 20000, 128, even(128, 2), "relu", 0),                                 # subspaces 64 columns wide, keys in 4 chunks
    (7, 700, 128, [(0, 128)], "normal", 0),                                   # the widest subspace the learner takes
    (8, 50, 5, [(0, 2), (2, 3), (3, 5)], "few_values", 0),                    # buckets that cannot be split, empty buckets
    (9, 1, 4, [(0, 4)], "normal", 0),                                         # one training row
    (10, 9, 2, [(0, 2)], "constant", 0),
    (11, 3000, 48, [(0, 48), (0, 16), (8, 40)], "relu", 0),                   # overlapping subspaces are allowed
    (12, 2000, 100, [(0, 100)], "normal", 0),                                 # the widest kind whose tiles stay in bucket order
    (13, 1500, 66, [(0, 33), (33, 66)], "relu", 1),                           # an odd width, tiles of 128 positions
    (14, 5000, 40, [(0, 3), (3, 40)], "integers", 0),                         # many equal values: ties among the candidate splits
    (15, 600, 224, even(224, 224), "normal", 0),                              # 224 codebooks: a factor of 3584 rows, the substitution kernel for large factors
]


def training_matrix(seed, N, D, kind):
    rng = np.random.default_rng(seed)
    if kind == "relu":
        _, A, _ = wl.random_problem(seed, N, D, 4, latent=min(8, D), N_train=4)
        return A
    if kind == "integers":
        return rng.integers(0, 256, size=(N, D)).astype(np.float32)
    if kind == "few_values":
        return rng.integers(0, 4, size=(N, D)).astype(np.float32)
    if kind == "constant":
        return np.full((N, D), 3.0, dtype=np.float32)
    return rng.standard_normal((N, D)).astype(np.float32)


@pytest.mark.parametrize("case", SMALL, ids=lambda c: "seed%d_N%d_D%d_%s" % (c[0], c[1], c[2], c[4]))
def test_learner_small_cases(mad, case):
    seed, N, D, subspaces, kind, pad = case
    print("case learn", case, flush=True)
    A = training_matrix(seed, N, D, kind)
    sd, th, codes = check_against_oracle(mad, A, subspaces, str(case), lda_pad=pad, lam=1.0 if seed % 2 else 0.5)
    # the learned parameters drive the library's encoder to the same leaves
    import torch
    params = mad.Params(sd, th)
    packed = mad.maddness_encode(params, dev(A))
    torch.cuda.synchronize()
    assert (packed.cpu().numpy() == oracle.pack(codes.cpu().numpy())).all()


def test_learner_random_small_problems(mad):
    """Forty seeded problems of mixed shapes: 1 to 33 codebooks (both launch shapes of the split search), subspaces 1
    to 69 columns wide, 1 to 5000 rows around the tile sizes, continuous data and data with many ties; trees, training
    codes, ridge prototypes and bucket means all equal to the oracle's, to the bit."""
    import torch
    rng = np.random.default_rng(2106)
    for case in range(40):
        C = int(rng.choice([1, 2, 3, 5, 8, 15, 16, 17, 20, 33]))
        widths = rng.integers(1, 12, size=C)
        if rng.random() < 0.2:
            widths[rng.integers(0, C)] = int(rng.integers(30, 70))
        D = int(widths.sum())
        starts = np.concatenate([[0], np.cumsum(widths)[:-1]])
        subspaces = [(int(s), int(s + w)) for s, w in zip(starts, widths)]
        N = int(rng.choice([1, 2, 7, 63, 64, 65, 255, 256, 257, 511, 1000, 2049, 5000]))
        kind = str(rng.choice(["normal", "integers", "few_values"]))
        A = training_matrix(int(rng.integers(1 << 30)), N, D, kind)
        pad = int(rng.integers(0, 4))
        lam = float(rng.choice([1.0, 0.5, 3.0]))
        label = f"case {case}: N={N} D={D} C={C} {kind} pad={pad} lambda={lam}"
        print(label, flush=True)
        full = torch.zeros((N, D + pad), dtype=torch.float32, device="cuda")
        full[:, :D] = dev(A)
        A_d = full[:, :D]
        sd, th, codes = mad.maddness_learn_trees(A_d, subspaces)
        torch.cuda.synchronize()
        want_sd, want_th, want_codes, _ = oracle.learn_trees(A, subspaces)
        assert (sd.cpu().numpy() == want_sd).all(), label
        assert (th.cpu().numpy() == want_th).all(), label
        assert (codes.cpu().numpy() == want_codes).all(), label
        P = mad.maddness_learn_prototypes(codes, A_d, subspaces, ridge=True, lam=lam)
        Pm = mad.maddness_learn_prototypes(codes, A_d, subspaces, ridge=False)
        torch.cuda.synchronize()
        assert (P.cpu().numpy() == oracle.ridge_prototypes(want_codes, A, lam).astype(np.float32)).all(), label
        assert (Pm.cpu().numpy() == oracle.bucket_means(want_codes, A, subspaces).astype(np.float32)).all(), label


@pytest.mark.parametrize("cfg", [1, 2, 3, 4, 5, 6])
def test_learner_on_the_workloads(mad, cfg):
    """The training sets of all six workloads at their full sizes."""
    w = wl.get_workload(cfg)
    print("workload", w.name, flush=True)
    A = wl.make_A_train(w)
    check_against_oracle(mad, A, list(w.subspaces), w.name)


def test_learn_on_device_feeds_the_inference_calls(mad):
    """Learn on the device, build the tables, run the fused call: equal to the oracle fed with the
    oracle-learned parameters."""
    import torch
    w = wl.get_workload(2)
    At, A, B = wl.make_A_train(w), wl.make_A(w), wl.make_B(w)
    params = mad.learn_on_device(dev(At), list(w.subspaces))
    luts, scale, offset = mad.maddness_build_luts(params, dev(B))
    out = mad.maddness_encode_scan(params, dev(A), luts, scale, offset)
    torch.cuda.synchronize()
    sd, th, codes, _ = oracle.learn_trees(At, list(w.subspaces))
    P = oracle.ridge_prototypes(codes, At, 1.0).astype(np.float32)
    assert (params.prototypes.cpu().numpy() == P).all() or np.abs(params.prototypes.cpu().numpy() - P).max() <= 1e-6 * np.abs(P).max()
    want, _, _ = oracle.encode_scan(A, sd, th, luts.cpu().numpy(), scale.cpu().numpy(), offset.cpu().numpy())
    assert (out.cpu().numpy() == want).all()


def test_learner_rejects_bad_arguments(mad):
    import torch
    L = mad.lib()
    A = torch.zeros((100, 300), dtype=torch.float32, device="cuda")
    out_i = torch.zeros((1, 4), dtype=torch.int32, device="cuda")
    out_f = torch.zeros((1, 16), dtype=torch.float32, device="cuda")
    ws = torch.zeros(1 << 22, dtype=torch.uint8, device="cuda")

    def trees(bounds, N=100, D=300, C=1, lda=300):
        b = (ctypes.c_int32 * len(bounds))(*bounds)
        return L.maddness_learn_trees(A.data_ptr(), N, lda, D, C, b, out_i.data_ptr(), out_f.data_ptr(), None,
                                      ws.data_ptr(), ws.numel(), None)
    assert trees([0, 16]) == mad.MADDNESS_OK
    assert trees([0, 129]) == mad.MADDNESS_E_UNSUPPORTED and "128" in L.maddness_last_error().decode()
    assert trees([5, 5]) == mad.MADDNESS_E_INVAL
    assert trees([-1, 4]) == mad.MADDNESS_E_INVAL
    assert trees([290, 301]) == mad.MADDNESS_E_INVAL
    assert trees([0, 16], N=0) == mad.MADDNESS_E_INVAL
    assert trees([0, 16], lda=299) == mad.MADDNESS_E_INVAL
    b = (ctypes.c_int32 * 2)(0, 16)
    assert L.maddness_learn_trees(A.data_ptr(), 100, 300, 300, 1, b, out_i.data_ptr(), out_f.data_ptr(), None, ws.data_ptr(), 64,
                                  None) == mad.MADDNESS_E_UNSUPPORTED
    codes = torch.zeros((100, 1), dtype=torch.uint8, device="cuda")
    P = torch.zeros((1, 16, 300), dtype=torch.float32, device="cuda")
    assert L.maddness_learn_prototypes(codes.data_ptr(), A.data_ptr(), 100, 300, 300, 1, b, 1, 0.0, P.data_ptr(), ws.data_ptr(),
                                       ws.numel(), None) == mad.MADDNESS_E_INVAL
    assert L.maddness_learn_prototypes(None, A.data_ptr(), 100, 300, 300, 1, b, 1, 1.0, P.data_ptr(), ws.data_ptr(),
                                       ws.numel(), None) == mad.MADDNESS_E_INVAL
    torch.cuda.synchronize()
