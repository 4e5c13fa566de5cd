"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle on
the same seeded inputs.  Maps must match bit for bit; C must satisfy
|C - C_ref| <= 1e-5 * (|A| x |B|) + 1e-6 in fp32 (1e-2 for bf16 inputs), and be
bit-exact where every product and partial sum is an exact integer."""
import numpy as np
import pytest
import torch

import mmm_synth as synth
import oracle
import paper_2402_14118_amd as mm
from hip_harness import HipRun, assert_close

pytestmark = pytest.mark.gpu


@pytest.fixture(autouse=True)
def _auto_options():
    mm.mmm_set_option("matmul_variant", -1)
    mm.mmm_set_option("split_k", 0)
    mm.mmm_set_option("matmul_path", -1)
    yield
    mm.mmm_set_option("matmul_variant", -1)
    mm.mmm_set_option("split_k", 0)
    mm.mmm_set_option("matmul_path", -1)


@pytest.fixture(params=[mm.MMM_PATH_MATRIX, mm.MMM_PATH_PAIRS], ids=["matrix", "pairs"])
def path(request):
    """Runs a test once per multiplication kernel."""
    mm.mmm_set_option("matmul_path", request.param)
    return request.param


def derived_from_bits(ab, bb, M, K, NB):
    """Column-any words per 32-row tile and the transposed B map, from the oracle's bitmaps."""
    a = synth.unpack_bits(ab, K)
    pad = (-M) % 32
    a = np.concatenate([a, np.zeros((pad, K), bool)]) if pad else a
    colany = synth.pack_bits(a.reshape(-1, 32, K).any(axis=1))
    bt = synth.pack_bits(synth.unpack_bits(bb, NB).T)
    return colany, bt


def live_rows(w):
    """The k that keep_rows leaves on (row-compacted mode numbers them k' = 0, 1, ...), or None without keep_rows."""
    if w.keep_rows is None:
        return None
    return np.nonzero(synth.unpack_bits(w.keep_rows.reshape(1, -1), w.K)[0])[0]


def check_lists(run, ab, w, what):
    """The blocked non-zero lists of A against the oracle's bitmap and the input values: per 64 x 128 block the
    same set of {slab offset, value bits} words (their order is the library's own), then the stated padding.  With
    keep_rows the blocks are over the live columns only."""
    counts, ents = run.lists_host()
    keep = synth.unpack_bits(ab, w.K)
    xbits = np.ascontiguousarray(w.X, dtype=np.float32).view(np.uint32)
    live = live_rows(w)
    if live is not None:
        keep, xbits = keep[:, live], xbits[:, live]
    kcols = keep.shape[1]
    MB, KB = (w.M + 63) // 64, (w.K + 127) // 128
    assert counts.shape == (MB, KB), what
    for bm in range(MB):
        for bk in range((kcols + 127) // 128):
            kp = keep[bm * 64:(bm + 1) * 64, bk * 128:(bk + 1) * 128]
            r, c = np.nonzero(kp)
            want = (xbits[bm * 64 + r, bk * 128 + c].astype(np.uint64) << np.uint64(32)) | (272 * c + 16 * (r % 16) + 4 * (r // 16)).astype(np.uint64)
            got = ents[bm * KB + bk]
            n = int(counts[bm, bk])
            assert n == len(want), f"{what}: block ({bm},{bk}) count {n} want {len(want)}"
            np.testing.assert_array_equal(np.sort(got[:n]), np.sort(want), err_msg=f"{what}: block ({bm},{bk}) entries")
            assert (got[n:] == np.uint64(34816)).all(), f"{what}: block ({bm},{bk}) padding"


def check_compacted(run, ab, bb, w, what):
    """Row-compacted mode: the numbering of the live rows and the maps over it, against copies derived from the
    oracle's bitmaps and the keep_rows input."""
    comp = run.eng.compacted()
    live = live_rows(w)
    if live is None or w.dtype == synth.DT_F64:     # double inputs do not use the mode
        assert comp is None, what
        return
    assert comp is not None, what
    torch.cuda.synchronize()
    count, kmap, colany_c, btc = (t.cpu().numpy() for t in comp)
    assert int(count[0]) == len(live), what
    np.testing.assert_array_equal(kmap[: len(live)], live, err_msg=f"{what}: kmap")
    words = (len(live) + 127) // 128 * 2          # the words the multiplication looks at
    if words == 0:
        return
    a = synth.unpack_bits(ab, w.K)[:, live]
    pad = (-w.M) % 32
    a = np.concatenate([a, np.zeros((pad, len(live)), bool)]) if pad else a
    exp_c = synth.pack_bits(np.pad(a.reshape(-1, 32, len(live)).any(axis=1), ((0, 0), (0, words * 64 - len(live)))))
    exp_b = synth.pack_bits(np.pad(synth.unpack_bits(bb, w.N // w.bw)[live].T, ((0, 0), (0, words * 64 - len(live)))))
    have = min(words, (w.K + 63) // 64)          # a short K has fewer words than a whole step
    np.testing.assert_array_equal(colany_c.view(np.uint64)[:, :have], exp_c[:, :have], err_msg=f"{what}: a_colany over k'")
    np.testing.assert_array_equal(btc.view(np.uint64)[:, :have], exp_b[:, :have], err_msg=f"{what}: bt_bits over k'")


def check_k_lists(run, ab, bb, w, what):
    """The per-tile active-k lists the matrix kernel walks, as its own list construction writes them out: for every row
    tile of 64, 16-column group and step of 128 the ascending k with (some non-zero of A in the tile's column k) and
    (the group's block(s) of B occupied in row k) -- over the live rows k' when keep_rows is given.  Expected lists
    come from the oracle's bitmaps alone."""
    got = run.eng.k_lists().cpu().numpy()
    NB, bw = w.N // w.bw, w.bw
    a = synth.unpack_bits(ab, w.K)
    b = synth.unpack_bits(bb, NB)
    live = live_rows(w)
    if live is not None:
        a, b = a[:, live], b[live]
    kk = a.shape[1]
    tm, groups, steps = got.shape[:3]
    assert tm == (w.M + 63) // 64 and groups == 16 * ((w.N + 255) // 256) and steps == (w.K + 127) // 128, what
    pad = (-w.M) % 64
    a64 = np.concatenate([a, np.zeros((pad, kk), bool)]) if pad else a
    colany = a64.reshape(tm, 64, kk).any(axis=1)                      # [tile, k]
    for G in range(groups):
        if G * 16 >= w.N:
            occ = np.zeros(kk, bool)
        elif bw == 16:
            occ = b[:, G]
        elif bw == 32:
            occ = b[:, G // 2]
        else:
            occ = b[:, 2 * G] | (b[:, 2 * G + 1] if 2 * G + 1 < NB else False)
        for t in range(tm):
            active = colany[t] & occ
            for c in range((kk + 127) // 128):                        # steps past the last live one are not written
                want = np.nonzero(active[128 * c: 128 * c + 128])[0]
                rec = got[t, G, c]
                n = int(rec[:4].view(np.uint32)[0])
                assert n == len(want), f"{what}: k list of tile {t} group {G} step {c}: {n} entries, want {len(want)}"
                np.testing.assert_array_equal(rec[4: 4 + n], want.astype(np.uint8), err_msg=f"{what}: k list ({t},{G},{c})")


def check_workload(w, what, exact=False, **ld):
    print(f"case {what}: M={w.M} K={w.K} N={w.N} bw={w.bw} dtype={w.dtype}", flush=True)
    ab, bb, C_ref, mag = oracle.run_workload(w)
    run = HipRun(w, **ld)
    a_hip, b_hip, C = run.run()
    np.testing.assert_array_equal(a_hip, ab, err_msg=f"{what}: a_bits")
    np.testing.assert_array_equal(b_hip, bb, err_msg=f"{what}: b_bits")
    colany, bt = run.derived_host()
    exp_colany, exp_bt = derived_from_bits(ab, bb, w.M, w.K, w.N // w.bw)
    np.testing.assert_array_equal(colany, exp_colany, err_msg=f"{what}: a_colany")
    np.testing.assert_array_equal(bt, exp_bt, err_msg=f"{what}: bt_bits")
    check_compacted(run, ab, bb, w, what)
    if w.M * w.K <= 1 << 22 and w.dtype != synth.DT_F64:     # double inputs have no blocked lists
        check_lists(run, ab, w, what)
        if w.M * w.K * (w.N // 16) <= 1 << 26:
            check_k_lists(run, ab, bb, w, what)
    assert run.eng.stats() == oracle.counts(ab, bb, w.M, w.K, w.N, w.bw), what
    if exact:
        np.testing.assert_array_equal(C, C_ref, err_msg=what)
    else:
        assert_close(C, C_ref, mag, w.dtype, what)
    assert not np.isnan(run.Cbuf[:, : w.N].cpu().numpy()).any()
    return run, (ab, bb, C_ref, mag, C)


# ---- small sizes, element by element: several tiles and ragged tails ------------------------
SHAPES = [
    (1, 1, 8, 8), (1, 1, 16, 16), (1, 1, 32, 32),
    (5, 7, 24, 8),              # N not a multiple of 16 with bw 8: half a column group
    (33, 65, 48, 16),           # one row / one k past a tile edge
    (70, 200, 272, 16),         # ragged in every dimension
    (100, 130, 96, 32),
    (64, 128, 256, 16),         # exactly one tile of the default variant
    (129, 257, 520, 8),
    (200, 1000, 320, 32),
]


@pytest.mark.parametrize("M,K,N,bw", SHAPES)
def test_small_shapes_exact_integers(M, K, N, bw, path):
    w = synth.random_masked(M, K, N, bw, 0.3, 0.4, 500 + M + K, dist="smallint", p_rows=0.8)
    check_workload(w, f"int {M}x{K}x{N} bw{bw}", exact=True)


@pytest.mark.parametrize("M,K,N,bw", SHAPES[3:])
def test_small_shapes_float(M, K, N, bw, path):
    w = synth.random_masked(M, K, N, bw, 0.25, 0.3, 900 + N, dist="normal")
    check_workload(w, f"f32 {M}x{K}x{N} bw{bw}")


@pytest.mark.parametrize("variant", range(mm.mmm_matmul_variant_count()))
@pytest.mark.parametrize("split", [1, 3])
def test_every_variant_and_split(variant, split):
    mm.mmm_set_option("matmul_variant", variant)
    mm.mmm_set_option("split_k", split)
    short = mm.mmm_matmul_variant_name(variant).startswith("R2")     # kernels for at most 32 rows
    w = synth.random_masked(30 if short else 150, 700, 400, 16, 0.3, 0.3, 77, dist="smallint")
    run, _ = check_workload(w, f"variant {variant} split {split}", exact=True)
    v, s, _ = run.eng.plan()
    assert v == variant and s == split
    # the same with rows of B switched off: the kernel walks the live rows only and shares them out over the splits
    for p_rows in (0.5, 0.02):
        w = synth.random_masked(30 if short else 150, 1500, 400, 16, 0.3, 0.5, 78, dist="smallint", p_rows=p_rows)
        check_workload(w, f"variant {variant} split {split} rows {p_rows}", exact=True)


@pytest.mark.parametrize("variant", range(mm.mmm_matmul_variant_count()))
@pytest.mark.parametrize("bw,p_a,p_b", [(16, 0.9, 0.95), (8, 0.15, 0.5), (32, 0.5, 0.1)])
def test_long_k_dense_lists(variant, bw, p_a, p_b):
    """K long enough for several list windows in every variant; dense A (blocks with more entries than one round of the
    workgroup) and dense B (k lists of many batches)."""
    mm.mmm_set_option("matmul_variant", variant)
    mm.mmm_set_option("split_k", 1)
    short = mm.mmm_matmul_variant_name(variant).startswith("R2")
    w = synth.random_masked(30 if short else 70, 2500, 96, bw, p_a, p_b, 4242 + variant, dist="smallint")
    check_workload(w, f"long K variant {variant} bw {bw}", exact=True)


@pytest.mark.parametrize("bw", [8, 16, 32])
def test_column_structured_a(bw, path):
    """Whole columns of A and the same rows of B switched off: the k lists shrink to the shared set."""
    w = synth.column_sparse(130, 1000, 320, bw, 0.15, 0.7, 0.8, 600 + bw)
    run, (ab, bb, *_rest) = check_workload(w, f"column sparse bw {bw}")
    selected = synth.unpack_bits(w.keep_rows.reshape(1, -1), w.K)[0]
    assert not (synth.unpack_bits(ab, w.K).any(axis=0) & ~selected).any()
    assert not (synth.unpack_bits(bb, w.N // bw).any(axis=1) & ~selected).any()


def test_padded_leading_dimensions_and_unaligned_rows(path):
    w = synth.random_masked(70, 203, 80, 16, 0.3, 0.5, 31, dist="smallint")
    check_workload(w, "ld padded", exact=True, ldx=209, ldy=83, ldc=91)


def test_predicates_and_special_values():
    rng = np.random.default_rng(12)
    M, K, N, bw = 40, 96, 64, 16
    X = rng.standard_normal((M, K)).astype(np.float32)
    X[0, :8] = [0.0, -0.0, 1e-45, -1e-40, 3e-39, -2.0, 0.5, 1.0]     # zeros and denormals
    X[1, 5] = np.nan                                                   # NaN is dropped by > and |.| >
    Y = rng.standard_normal((K, N)).astype(np.float32)
    Y[3, 16:32] = 0.0
    Y[3, 20] = -0.0                                                    # all-zero block: unoccupied
    Y[4, 32:48] = 0.0
    Y[4, 40] = 1e-45                                                   # denormal occupies its block
    for pred, thr in [(synth.PRED_GT, 0.0), (synth.PRED_GT, -0.5), (synth.PRED_ABS_GT, 0.7),
                      (synth.PRED_ABS_GT, -1.0), (synth.PRED_GT, 1e-40)]:
        w = synth.Workload("pred", M, K, N, bw, synth.DT_F32, X, Y, pred=pred, threshold=thr)
        ab = oracle.a_bits(X, pred, thr)
        bb = oracle.b_bits(Y, bw)
        run = HipRun(w)
        run.build()
        a_hip, b_hip = run.maps_host()
        np.testing.assert_array_equal(a_hip, ab, err_msg=f"pred {pred} thr {thr}")
        np.testing.assert_array_equal(b_hip, bb)
    # NONZERO keeps the NaN: checked on maps only (the product would be NaN on both sides)
    ab = oracle.a_bits(X)
    w = synth.Workload("nz", M, K, N, bw, synth.DT_F32, X, Y)
    run = HipRun(w)
    run.build()
    np.testing.assert_array_equal(run.maps_host()[0], ab)


@pytest.mark.parametrize("dtype", [synth.DT_F32, synth.DT_BF16, synth.DT_F16])
@pytest.mark.parametrize("bw,N", [(8, 136), (16, 128), (32, 160)])
def test_masked_positions_may_hold_anything(bw, N, dtype, path):
    """Masked-out X elements and switched-off Y blocks never reach the arithmetic.  With bw = 8 a 16-column group of
    the multiplier spans two blocks (and N = 136 leaves half a group at the edge), with bw = 32 a block spans two
    groups."""
    w = synth.random_masked(64, 256, N, bw, 0.3, 0.3, 5 + bw, dist="smallint", dtype=dtype)
    ab, bb, C_ref, _ = oracle.run_workload(w)
    keepa = synth.unpack_bits(w.keep_a, w.K)
    keepb = np.repeat(synth.unpack_bits(w.keep_blocks, w.N // w.bw), w.bw, axis=1)
    w.X = np.where(keepa, w.X, np.float32(np.nan))
    w.Y = np.where(keepb, w.Y, np.float32(np.inf))
    if dtype == synth.DT_BF16:
        w.X_bits, w.Y_bits = synth.round_to_bf16(w.X)[0], synth.round_to_bf16(w.Y)[0]
    elif dtype == synth.DT_F16:
        w.X_bits, w.Y_bits = synth.round_to_f16(w.X)[0], synth.round_to_f16(w.Y)[0]
    a_hip, b_hip, C = HipRun(w).run()
    np.testing.assert_array_equal(a_hip, ab)
    np.testing.assert_array_equal(b_hip, bb)
    np.testing.assert_array_equal(C, C_ref)


@pytest.mark.parametrize("bw", [8, 16, 32])
def test_non_finite_value_inside_an_occupied_block(bw, path):
    """The stated contract for a kept Inf in Y: only its column of C is affected; rows whose element of A at that k is
    non-zero get a non-finite result, the other rows of that column the exact value or NaN."""
    w = synth.random_masked(100, 300, 160, bw, 0.3, 0.5, 41 + bw, dist="smallint")
    bb0 = oracle.b_bits(w.Y, bw, w.keep_rows, w.keep_blocks)
    k, jb = [int(v[0]) for v in np.nonzero(synth.unpack_bits(bb0, w.N // bw))]      # some occupied block
    j = jb * bw + 3
    w.Y[k, j] = np.inf
    ab, bb, C_ref, _ = oracle.run_workload(w)
    np.testing.assert_array_equal(bb, bb0)
    a_hip, b_hip, C = HipRun(w).run()
    np.testing.assert_array_equal(a_hip, ab)
    np.testing.assert_array_equal(b_hip, bb)
    other = np.arange(w.N) != j
    np.testing.assert_array_equal(C[:, other], C_ref[:, other])
    hit = synth.unpack_bits(ab, w.K)[:, k]
    assert hit.any() and not hit.all()
    assert not np.isfinite(C_ref[hit, j]).any() and np.isfinite(C_ref[~hit, j]).all()     # what the definition gives
    assert not np.isfinite(C[hit, j]).any()
    rest = C[~hit, j]
    assert np.all(np.isnan(rest) | (rest == C_ref[~hit, j]))


def test_rebuilding_a_row_compacted_b_side_alone_leaves_a_unbuilt():
    mm.mmm_set_option("matmul_path", mm.MMM_PATH_MATRIX)
    w = synth.random_masked(70, 400, 96, 16, 0.3, 0.5, 61, dist="smallint", p_rows=0.3)
    _, _, C_ref, _ = oracle.run_workload(w)
    run = HipRun(w)
    run.build()
    run.build(a=False, b=True)             # the numbering of the live rows was made anew: the lists of A are void
    with pytest.raises(mm.MmmError) as e:
        run.matmul()
    assert e.value.status == mm.binding.MMM_ERR_MAPS_MISMATCH
    run.build(a=True, b=False)
    run.matmul()
    torch.cuda.synchronize()
    np.testing.assert_array_equal(run.C.cpu().numpy(), C_ref)
    # other rows switched on, B rebuilt together with A
    w2 = synth.random_masked(70, 400, 96, 16, 0.3, 0.5, 62, dist="smallint", p_rows=0.6)
    w2.X, w2.keep_a = w.X, w.keep_a
    _, _, C2_ref, _ = oracle.run_workload(w2)
    run.Y.copy_(torch.from_numpy(w2.Y))
    run.keep_rows.copy_(torch.from_numpy(w2.keep_rows.view(np.int64)))
    run.keep_blocks.copy_(torch.from_numpy(w2.keep_blocks.view(np.int64)))
    run.build()
    run.matmul()
    torch.cuda.synchronize()
    np.testing.assert_array_equal(run.C.cpu().numpy(), C2_ref)


def test_matmul_refuses_another_x_than_the_one_built_from():
    w = synth.random_masked(40, 100, 64, 16, 0.3, 0.3, 77, dist="smallint")
    run = HipRun(w)
    run.build()
    X2 = run.X.clone()
    with pytest.raises(mm.MmmError) as e:
        run.eng.matmul(X2, run.Y, run.C)
    assert e.value.status == mm.binding.MMM_ERR_MAPS_MISMATCH
    run.matmul()          # the X it was built from is accepted


def test_identity_zero_and_full_masks(path):
    n, bw = 96, 16
    rng = np.random.default_rng(2)
    Y = rng.standard_normal((n, n)).astype(np.float32)
    eye = np.eye(n, dtype=np.float32)
    kb = synth.pack_bits(rng.random((n, n // bw)) < 0.5)
    w = synth.Workload("I*Y", n, n, n, bw, synth.DT_F32, eye, Y, keep_blocks=kb)
    _, _, C = HipRun(w).run()
    np.testing.assert_array_equal(C, np.where(np.repeat(synth.unpack_bits(kb, n // bw), bw, axis=1), Y, 0))
    ka = synth.pack_bits(rng.random((n, n)) < 0.3)
    w = synth.Workload("X*I", n, n, n, bw, synth.DT_F32, Y, eye, keep_a=ka)
    _, _, C = HipRun(w).run()
    np.testing.assert_array_equal(C, np.where(synth.unpack_bits(ka, n), Y, 0))
    for pa, pb in [(0.0, 0.5), (0.5, 0.0)]:
        w = synth.random_masked(50, 130, 64, 16, pa, pb, 8)
        run, (_, _, _, _, C) = check_workload(w, f"zero mask {pa},{pb}", exact=True)
        assert not C.any() and not np.signbit(C).any()
        assert run.eng.stats()[2] == 0
    w = synth.random_masked(48, 100, 64, 16, 1.0, 1.0, 9, dist="normal")     # nothing masked: plain GEMM
    _, (_, _, _, mag, C) = check_workload(w, "all keep")
    ref = w.X.astype(np.float64) @ w.Y.astype(np.float64)
    assert np.all(np.abs(C - ref) <= 1e-5 * mag + 1e-6)


def test_accumulate_and_cached_b_map(path):
    w = synth.random_masked(90, 300, 160, 16, 0.3, 0.3, 21, dist="smallint")
    ab, bb, C_ref, _ = oracle.run_workload(w)
    run = HipRun(w)
    run.build()
    run.matmul()
    run.matmul(accumulate=True)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(run.C.cpu().numpy(), 2 * C_ref)
    # new activations against the cached B map: only the A side is rebuilt
    w2 = synth.random_masked(90, 300, 160, 16, 0.5, 0.3, 22, dist="smallint")
    w2.Y, w2.keep_blocks = w.Y, w.keep_blocks
    ab2, bb2, C2_ref, _ = oracle.run_workload(w2)
    run.X.copy_(torch.from_numpy(w2.X))
    run.keep_a.copy_(torch.from_numpy(w2.keep_a.view(np.int64)))
    run.build(a=True, b=False)
    run.matmul()
    a_hip, b_hip = run.maps_host()
    np.testing.assert_array_equal(a_hip, ab2)
    np.testing.assert_array_equal(b_hip, bb)
    np.testing.assert_array_equal(run.C.cpu().numpy(), C2_ref)


@pytest.mark.parametrize("variant", [0, 1, 5])
def test_accumulate_with_split_k_and_padded_c(variant):
    """C += A x B through the split-K path (partials reduced, then added), rows of C padded: the padding stays."""
    mm.mmm_set_option("matmul_variant", variant)
    mm.mmm_set_option("split_k", 3)
    short = mm.mmm_matmul_variant_name(variant).startswith("R2")
    w = synth.random_masked(30 if short else 90, 900, 176, 16, 0.3, 0.3, 23 + variant, dist="smallint")
    _, _, C_ref, _ = oracle.run_workload(w)
    run = HipRun(w, ldc=w.N + 5)
    run.build()
    run.matmul()
    run.matmul(accumulate=True)
    run.matmul(accumulate=True)
    torch.cuda.synchronize()
    assert run.eng.plan()[1] == 3
    np.testing.assert_array_equal(run.C.cpu().numpy(), 3 * C_ref)
    assert torch.isnan(run.Cbuf[:, w.N:]).all()


@pytest.mark.parametrize("variant", range(mm.mmm_matmul_variant_count()))
@pytest.mark.parametrize("dtype", [synth.DT_BF16, synth.DT_F16])
def test_16_bit_inputs_every_variant(variant, dtype):
    mm.mmm_set_option("matmul_variant", variant)
    mm.mmm_set_option("split_k", 1)
    short = mm.mmm_matmul_variant_name(variant).startswith("R2")
    w = synth.random_masked(30 if short else 100, 1500, 160, 32, 0.3, 0.4, 300 + variant, dist="smallint", dtype=dtype)
    check_workload(w, f"dtype {dtype} variant {variant}", exact=True)


# ---- the kernel over exactly the surviving products (vector FMAs) -----------------------------
@pytest.mark.parametrize("bw,p_a,p_b", [(16, 0.9, 0.95), (8, 0.15, 0.5), (32, 0.5, 0.1), (8, 1.0, 1.0)])
@pytest.mark.parametrize("M,N", [(5, 96), (300, 2048)])
def test_pairs_long_k_dense_lists(bw, p_a, p_b, M, N):
    """K beyond one range of the row copy in LDS; lists far longer than one pass holds (dense A and B); both workgroup
    shapes (few rows: every range of k is split over four waves; many rows: eight waves side by side)."""
    mm.mmm_set_option("matmul_path", mm.MMM_PATH_PAIRS)
    w = synth.random_masked(M, 20000, N, bw, p_a, p_b, 5150 + bw + M, dist="smallint")
    check_workload(w, f"pairs long K bw {bw} M {M}", exact=True)


def test_automatic_path():
    """Few rows: the pair kernel.  Many rows: the matrix kernel until the statistics show a very sparse A."""
    w = synth.random_masked(40, 300, 64, 16, 0.3, 0.3, 1)
    run = HipRun(w)
    run.build()
    assert run.eng.path() == mm.MMM_PATH_PAIRS
    run.eng.set_plan(0, 1)
    assert run.eng.path() == mm.MMM_PATH_MATRIX       # a tile variant was asked for
    run.eng.set_plan()
    for p_a, p_b, want in [(0.02, 0.3, mm.MMM_PATH_PAIRS), (0.02, 0.02, mm.MMM_PATH_MATRIX), (0.2, 0.3, mm.MMM_PATH_MATRIX)]:
        w = synth.random_masked(1024, 600, 2048, 16, p_a, p_b, 2, dist="smallint")
        run = HipRun(w)
        run.build()
        assert run.eng.path() == mm.MMM_PATH_MATRIX   # nothing counted yet
        run.eng.stats()
        assert run.eng.path() == want
        run.build()                                    # the estimate survives a rebuild
        assert run.eng.path() == want
        run.matmul()
        torch.cuda.synchronize()
        np.testing.assert_array_equal(run.C.cpu().numpy(), oracle.run_workload(w)[2])
        run.eng.set_path(mm.MMM_PATH_MATRIX)
        assert run.eng.path() == mm.MMM_PATH_MATRIX
        run.eng.set_path()
    # a small problem with short lists: latency-bound, the pair kernel (once the densities are known)
    w = synth.random_masked(200, 600, 128, 16, 0.2, 0.3, 3, dist="smallint")
    run = HipRun(w)
    run.build()
    assert run.eng.path() == mm.MMM_PATH_MATRIX
    run.eng.stats()
    assert run.eng.path() == mm.MMM_PATH_PAIRS


FUSED_CASES = [(synth.PRED_NONZERO, 0.0, True), (synth.PRED_GT, 0.0, False), (synth.PRED_GT, -0.5, True),
               (synth.PRED_ABS_GT, 0.7, False), (synth.PRED_GT, 1e-40, False)]


@pytest.mark.parametrize("pred,thr,with_keep", FUSED_CASES)
@pytest.mark.parametrize("dtype", [synth.DT_F32, synth.DT_BF16, synth.DT_F16])
def test_fused_mask_evaluation(pred, thr, with_keep, dtype):
    """mmm_matmul_fused: M is evaluated inside the multiplication (predicate, keep bitmap, non-zero test), only the B
    side of the maps is built.  Special values in X as in the builder's test; C against the oracle."""
    rng = np.random.default_rng(77)
    M, K, N, bw = 37, 9000, 208, 16
    w = synth.random_masked(M, K, N, bw, 0.4, 0.4, 4040, dist="normal", dtype=dtype)
    w.X[0, :8] = [0.0, -0.0, 1e-45, -1e-40, 3e-39, -2.0, 0.5, 1.0]
    w.X[1, 5] = np.nan if pred != synth.PRED_NONZERO else 1.0
    if dtype == synth.DT_BF16:
        w.X_bits, w.X = synth.round_to_bf16(w.X)
    elif dtype == synth.DT_F16:
        w.X_bits, w.X = synth.round_to_f16(w.X)
    w.pred, w.threshold = pred, thr
    if not with_keep:
        w.keep_a = None
    ab, bb, C_ref, mag = oracle.run_workload(w)
    run = HipRun(w)
    run.build(a=False, b=True)
    run.eng.matmul_fused(run.X, run.Y, run.C, pred, thr, run.keep_a)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(run.maps_host()[1], bb)
    assert_close(run.C.cpu().numpy(), C_ref, mag, dtype, f"fused pred {pred} thr {thr}")
    run.eng.matmul_fused(run.X, run.Y, run.C, pred, thr, run.keep_a, accumulate=True)
    torch.cuda.synchronize()
    assert_close(run.C.cpu().numpy(), 2 * C_ref, 2 * mag, dtype, "fused accumulate")


def test_row_stride_of_y_beyond_the_pair_kernels_reach():
    """The pair kernel forms 32-bit offsets inside 4096 rows of Y; with a row stride of 2^18 floats and more the matrix
    kernel multiplies whatever was asked for, and the fused entry (pair kernel only) refuses."""
    w = synth.random_masked(40, 200, 64, 16, 0.3, 0.5, 88, dist="smallint")
    _, _, C_ref, _ = oracle.run_workload(w)
    run = HipRun(w, ldy=(1 << 18) + 8)
    mm.mmm_set_option("matmul_path", mm.MMM_PATH_PAIRS)
    run.build()
    run.matmul()
    torch.cuda.synchronize()
    np.testing.assert_array_equal(run.C.cpu().numpy(), C_ref)
    with pytest.raises(mm.MmmError) as e:
        run.eng.matmul_fused(run.X, run.Y, run.C, w.pred, w.threshold, run.keep_a)
    assert e.value.status == mm.binding.MMM_ERR_SHAPE


def test_fused_exact_and_argument_checks():
    w = synth.random_masked(70, 700, 144, 8, 0.3, 0.4, 99, dist="smallint")
    _, _, C_ref, _ = oracle.run_workload(w)
    run = HipRun(w, ldx=711, ldy=150, ldc=149)
    with pytest.raises(mm.MmmError) as e:
        run.eng.matmul_fused(run.X, run.Y, run.C, w.pred, w.threshold, run.keep_a)      # B side not built
    assert e.value.status == mm.binding.MMM_ERR_MAPS_MISMATCH
    run.build(a=False, b=True)
    run.eng.matmul_fused(run.X, run.Y, run.C, w.pred, w.threshold, run.keep_a)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(run.C.cpu().numpy(), C_ref)
    assert torch.isnan(run.Cbuf[:, w.N:]).all()
    with pytest.raises(mm.MmmError) as e:
        run.eng.matmul_fused(run.X, run.Y, run.C, 3, 0.0, None)
    assert e.value.status == mm.binding.MMM_ERR_INVALID_ARG


# ---- double-precision inputs (pair kernel only) -----------------------------------------------
@pytest.mark.parametrize("M,K,N,bw", SHAPES)
def test_f64_small_shapes(M, K, N, bw):
    w = synth.random_masked(M, K, N, bw, 0.3, 0.4, 700 + M + K, dist="smallint", p_rows=0.8, dtype=synth.DT_F64)
    run, _ = check_workload(w, f"f64 int {M}x{K}x{N} bw{bw}", exact=True)
    assert run.eng.path() == mm.MMM_PATH_PAIRS and run.C.dtype == torch.float64
    w = synth.random_masked(M, K, N, bw, 0.25, 0.3, 800 + N, dist="normal", dtype=synth.DT_F64)
    check_workload(w, f"f64 {M}x{K}x{N} bw{bw}", ldx=K + 3, ldy=N + 5, ldc=N + 1)


@pytest.mark.parametrize("bw,p_a,p_b,M,N", [(16, 0.9, 0.95, 5, 96), (8, 0.15, 0.5, 300, 2048), (32, 0.5, 0.1, 40, 160)])
def test_f64_long_k(bw, p_a, p_b, M, N):
    w = synth.random_masked(M, 9000, N, bw, p_a, p_b, 5250 + bw, dist="normal", dtype=synth.DT_F64)
    check_workload(w, f"f64 long K bw {bw}")


def test_f64_predicates_special_values_and_fused():
    """Values float cannot hold: double denormals are non-zero, 1e300 passes the predicates; junk at masked positions;
    the fused entry evaluates the same predicates on doubles."""
    M, K, N, bw = 37, 700, 208, 16
    for pred, thr, with_keep in FUSED_CASES:
        w = synth.random_masked(M, K, N, bw, 0.4, 0.4, 4141, dist="normal", dtype=synth.DT_F64)
        w.X[0, :8] = [0.0, -0.0, 1e-310, -1e-320, 4.9e-324, -2.0, 0.5, 1e300]
        w.X[1, 5] = np.nan if pred != synth.PRED_NONZERO else 1.0
        w.Y[3, 16:32] = 0.0
        w.Y[3, 20] = 4.9e-324                    # a denormal occupies its block
        w.pred, w.threshold = pred, thr
        if not with_keep:
            w.keep_a = None
        ab, bb, C_ref, mag = oracle.run_workload(w)
        keepb = np.repeat(synth.unpack_bits(w.keep_blocks, N // bw), bw, axis=1)
        w.Y = np.where(keepb, w.Y, np.inf)       # switched-off blocks may hold anything
        run = HipRun(w)
        a_hip, b_hip, C = run.run()
        np.testing.assert_array_equal(a_hip, ab, err_msg=f"f64 pred {pred} thr {thr}")
        np.testing.assert_array_equal(b_hip, bb)
        assert_close(C, C_ref, mag, w.dtype, f"f64 pred {pred} thr {thr}")
        run.Cbuf.fill_(float("nan"))
        run.eng.matmul_fused(run.X, run.Y, run.C, pred, thr, run.keep_a)
        torch.cuda.synchronize()
        assert_close(run.C.cpu().numpy(), C_ref, mag, w.dtype, f"f64 fused pred {pred} thr {thr}")


def test_f64_config2_shape_full():
    """The 2048^3 configuration in double precision, element by element."""
    w = synth.random_masked(2048, 2048, 2048, 16, 0.1, 0.1, 1002, "normal", 0.0, 1.0, name="cfg2_f64", dtype=synth.DT_F64)
    check_workload(w, "config 2 shape, f64")


def test_autotune_fixes_a_plan_and_keeps_the_result():
    w = synth.random_masked(130, 900, 384, 16, 0.2, 0.2, 808, dist="smallint")
    _, _, C_ref, _ = oracle.run_workload(w)
    run = HipRun(w)
    run.build()
    timed = run.eng.autotune(run.X, run.Y, run.C, splits=(0, 2), reps=3)
    assert len(timed) >= 4 and timed == sorted(timed)
    assert run.eng.plan()[:2] == (timed[0][1], timed[0][2])
    run.matmul()
    torch.cuda.synchronize()
    np.testing.assert_array_equal(run.C.cpu().numpy(), C_ref)
    run.eng.set_plan()   # back to the automatic choice


def test_run_to_run_bitwise_reproducible():
    w = synth.config(2, scale=4)
    run = HipRun(w)
    _, _, C1 = run.run()
    run.Cbuf.fill_(float("nan"))
    _, _, C2 = run.run()
    np.testing.assert_array_equal(C1, C2)
    mm.mmm_set_option("split_k", 4)
    _, _, C3 = run.run()
    _, _, C4 = run.run()
    np.testing.assert_array_equal(C3, C4)


@pytest.mark.parametrize("dtype", [synth.DT_BF16, synth.DT_F16])
def test_16_bit_inputs_small(dtype, path):
    w = synth.random_masked(32, 520, 96, 16, 0.3, 0.3, 17, dist="normal", dtype=dtype)
    check_workload(w, f"dtype {dtype} small")
    w = synth.random_masked(45, 260, 64, 8, 0.3, 0.3, 18, dist="smallint", dtype=dtype)
    check_workload(w, f"dtype {dtype} int", exact=True)


def test_f16_predicates_and_tiny_values(path):
    """Half-precision denormals are non-zero and widen exactly; ReLU-style and magnitude predicates act on the value."""
    rng = np.random.default_rng(5)
    M, K, N, bw = 40, 200, 64, 16
    X = rng.standard_normal((M, K)).astype(np.float16)
    X[0, :6] = np.array([0.0, -0.0, 6e-8, -6e-8, 6.1e-5, -65504.0], dtype=np.float16)
    Y = rng.standard_normal((K, N)).astype(np.float16)
    Y[3, 16:32] = 0.0
    Y[3, 20] = np.float16(6e-8)          # a denormal occupies its block
    for pred, thr in [(synth.PRED_NONZERO, 0.0), (synth.PRED_GT, 0.0), (synth.PRED_ABS_GT, 0.5)]:
        w = synth.Workload("f16 pred", M, K, N, bw, synth.DT_F16, X.astype(np.float32), Y.astype(np.float32), pred=pred,
                           threshold=thr)
        w.X_bits, w.Y_bits = X.view(np.uint16), Y.view(np.uint16)
        check_workload(w, f"f16 pred {pred} thr {thr}")


def test_random_shapes_sweep():
    """Many small random cases (shape, block width, densities, dtype, variant, split, leading dimensions), exact on
    integer inputs; each case is printed before it runs."""
    rng = np.random.default_rng(2024)
    nv = mm.mmm_matmul_variant_count()
    for it in range(250):
        bw = int(rng.choice([8, 16, 32]))
        M, K, N = int(rng.integers(1, 200)), int(rng.integers(1, 3000)), bw * int(rng.integers(1, 40))
        if rng.random() < 0.3:
            M = int(rng.integers(1, 33))
        p_a, p_b = (float(rng.choice([0.02, 0.1, 0.3, 0.7, 1.0])) for _ in range(2))
        dtype = int(rng.choice([synth.DT_F32, synth.DT_BF16, synth.DT_F16]))
        variant, split = int(rng.integers(-1, nv)), int(rng.integers(0, 5))
        path, fused = int(rng.integers(-1, 2)), bool(rng.random() < 0.25)
        if variant >= 0 and mm.mmm_matmul_variant_name(variant).startswith("R2") and M > 32:
            variant = -1
        ld = dict(ldx=K + int(rng.integers(0, 9)), ldy=N + int(rng.integers(0, 9)), ldc=N + int(rng.integers(0, 9)))
        p_rows = [None, None, 0.0, 0.1, 0.5, 1.0][int(rng.integers(0, 6))]     # whole rows of B switched off
        what = (f"sweep {it}: M={M} K={K} N={N} bw={bw} p_a={p_a} p_b={p_b} dtype={dtype} variant={variant} split={split} "
                f"path={path} fused={fused} rows={p_rows} {ld}")
        print(what, flush=True)
        mm.mmm_set_option("matmul_variant", variant)
        mm.mmm_set_option("split_k", split)
        mm.mmm_set_option("matmul_path", path)
        w = synth.random_masked(M, K, N, bw, p_a, p_b, 20000 + it, dist="smallint", dtype=dtype, p_rows=p_rows)
        ab, bb, C_ref, _ = oracle.run_workload(w)
        run = HipRun(w, **ld)
        a_hip, b_hip, C = run.run()
        np.testing.assert_array_equal(a_hip, ab, err_msg=what)
        np.testing.assert_array_equal(b_hip, bb, err_msg=what)
        np.testing.assert_array_equal(C, C_ref, err_msg=what)
        assert torch.isnan(run.Cbuf[:, N:]).all(), what
        if fused:
            run.Cbuf.fill_(float("nan"))
            run.eng.matmul_fused(run.X, run.Y, run.C, w.pred, w.threshold, run.keep_a)
            torch.cuda.synchronize()
            np.testing.assert_array_equal(run.C.cpu().numpy(), C_ref, err_msg=what + " (fused)")
            assert torch.isnan(run.Cbuf[:, N:]).all(), what


# ---- the benchmark configurations at full size ------------------------------------------------
def test_config1_full(path):
    check_workload(synth.config(1), "config 1")


def test_config2_full(path):
    run, _ = check_workload(synth.config(2), "config 2")
    print("plan", run.eng.plan())


def test_config5_full_bf16_decode(path):
    run, _ = check_workload(synth.config(5), "config 5")
    print("plan", run.eng.plan())


@pytest.mark.parametrize("ip", range(len(synth.SWEEP_P)))
def test_config3_full(ip, path):
    """Every point of the sparsity sweep at full size, in the launch configuration the benchmark times, element by
    element against the oracle."""
    run, _ = check_workload(synth.config(3, ip), f"config 3 p={synth.SWEEP_P[ip]}")
    print("plan", run.eng.plan(), flush=True)


def test_config4_full(path):
    run, _ = check_workload(synth.config(4), "config 4")
    print("plan", run.eng.plan(), flush=True)
