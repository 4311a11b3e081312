"""Parity of the HIP path with the fp64 CPU oracle, element by element, through the C ABI.

Error measure (per level k): e_k = ||G_k - O_k||_2 / ||O_k||_2 with the norm taken over
all paths and stream positions of that level.  Bars: fp32 e_k <= 1e-4, fp64 e_k <= 1e-10.
"""
import functools

import numpy as np
import pytest

import paper_2001_00706_amd as sig
from oracle import sig_oracle as orc
from paper_2001_00706_amd.inputs import WORKLOADS, brownian_paths, uniform_paths, workload_paths

pytestmark = pytest.mark.gpu

TOL = {np.float32: 1e-4, np.float64: 1e-10}
# worst single path may sit somewhat above the batch-wide figure
TOL_SINGLE = {np.float32: 5e-4, np.float64: 5e-10}


def torch_mod():
    import torch
    return torch


def gpu_signature(x, N, stream=False, basepoint=False, variant=sig.SIG_VARIANT_AUTO, poison=True):
    torch = torch_mod()
    xt = torch.from_numpy(np.ascontiguousarray(x)).to("cuda:0")
    B, L, d = x.shape
    S = sig.sig_signature_channels(d, N)
    n_inc = L if basepoint else L - 1
    shape = (B, n_inc, S) if stream else (B, S)
    out = torch.full(shape, float("nan"), dtype=xt.dtype, device=xt.device) if poison else None
    got = sig.sig_forward(xt, N, stream=stream, basepoint=basepoint, out=out, variant=variant)
    torch.cuda.synchronize()
    return got.cpu().numpy()


def level_errors(got, want, d, N, elementwise=False):
    """Batch-wide and worst-single-path relative L2 error of every level; with `elementwise` also the worst
    single element of a path's level, relative to the largest element of that level of that path."""
    got = np.asarray(got, dtype=np.float64)
    B = got.shape[0]
    batch, single, element = [], [], []
    for sl in orc.level_slices(d, N):
        g, w = got[..., sl].reshape(B, -1), want[..., sl].reshape(B, -1)
        den = np.linalg.norm(w)
        batch.append(np.linalg.norm(g - w) / (den if den > 0 else 1.0))
        dens = np.linalg.norm(w, axis=1)
        dens[dens == 0] = 1.0
        single.append(float(np.max(np.linalg.norm(g - w, axis=1) / dens)))
        tops = np.max(np.abs(w), axis=1)
        tops[tops == 0] = 1.0
        element.append(float(np.max(np.max(np.abs(g - w), axis=1) / tops)))
    if elementwise:
        return np.array(batch), np.array(single), np.array(element)
    return np.array(batch), np.array(single)


def served(x, N, stream, basepoint, variant):
    B, L, d = x.shape
    dtype = sig.SIG_F32 if x.dtype == np.float32 else sig.SIG_F64
    return sig.sig_variant_name(B, L, d, N, stream, basepoint, dtype, variant) != "unsupported"


def check(x, N, stream=False, basepoint=False, variant=sig.SIG_VARIANT_AUTO, sample=None, want=None):
    """Runs the HIP path and compares with the oracle (or with `want`, an oracle result computed earlier for the
    same input); returns None (nothing compared) when the forced kernel family does not serve the shape."""
    if not served(x, N, stream, basepoint, variant):
        return None
    dt = x.dtype.type
    got = gpu_signature(x, N, stream, basepoint, variant)
    assert np.all(np.isfinite(got)), "output not fully written"
    idx = np.arange(x.shape[0]) if sample is None else np.asarray(sample)
    if want is None:
        want = orc.signature(x[idx], N, stream=stream, basepoint=basepoint)
    batch, single, element = level_errors(got[idx], want, x.shape[2], N, elementwise=True)
    assert np.all(batch <= TOL[dt]), f"per-level rel L2 {batch}"
    assert np.all(single <= TOL_SINGLE[dt]), f"worst single-path rel L2 {single}"
    # element by element: max |G - O| <= c * max |O| over the same level of the same path (and stream position set)
    assert np.all(element <= TOL[dt]), f"worst element, relative to the level's largest {element}"
    return got


VARIANTS = [sig.SIG_VARIANT_AUTO, sig.SIG_VARIANT_GENERIC, sig.SIG_VARIANT_MFMA, sig.SIG_VARIANT_MFMA_SHARD,
            sig.SIG_VARIANT_SMALL, sig.SIG_VARIANT_TREE, sig.SIG_VARIANT_MFMA_STREAM, sig.SIG_VARIANT_ROW_STREAM,
            sig.SIG_VARIANT_WIDE, sig.SIG_VARIANT_DEPTH2]
VARIANT_IDS = ["auto", "generic", "mfma", "mfma_shard", "small", "tree", "mfma_stream", "row_stream", "wide", "depth2"]
MODES = [(False, False), (False, True), (True, False), (True, True)]     # (stream, basepoint)


def serving_variants(B, L, d, N, dtype, modes):
    """The kernel families that serve this shape in at least one of `modes`, as pytest parameters; asked of the
    library itself (`sig_variant_name` is a host function), so that no case is generated only to be skipped."""
    code = sig.SIG_F32 if dtype == np.float32 else sig.SIG_F64
    return [pytest.param(v, id=name) for v, name in zip(VARIANTS, VARIANT_IDS)
            if any(sig.sig_variant_name(B, L, d, N, st, bp, code, v) != "unsupported" for st, bp in modes)]


# ------------------------------------------------------------------ benchmark workloads
@functools.lru_cache(maxsize=2)
def workload_oracle(index):
    """The oracle's signatures of every path of a workload (the fp64 input is the exact widening of the fp32 one,
    so one result serves both precisions)."""
    w = WORKLOADS[index - 1]
    return orc.signature(workload_paths(w), w.N, stream=w.stream, basepoint=w.basepoint)


WORKLOAD_CASES = [pytest.param(w, dtype, v.values[0], id=f"{w.name}-{np.dtype(dtype).name}-{v.id}")
                  for w in WORKLOADS for dtype in (np.float32, np.float64)
                  for v in serving_variants(w.B, w.L, w.d, w.N, dtype, [(w.stream, w.basepoint)])]


@pytest.mark.parametrize("w,dtype,variant", WORKLOAD_CASES)
def test_benchmark_workloads_full_size_every_path(w, dtype, variant):
    """The five workloads at full size, in the launch configuration bench.py times and under every kernel family
    that serves them, in fp32 and in fp64 (the fp64 input is the exact widening of the fp32 one): every element of
    every path, and of every prefix in stream mode, is compared with the oracle."""
    x = workload_paths(w).astype(dtype)
    assert check(x, w.N, stream=w.stream, basepoint=w.basepoint, variant=variant, want=workload_oracle(w.index)) is not None


# ------------------------------------------------------------------------ shape sweep
SWEEP = [
    # (B, L, d, N); the last rows sit at the limits of the small-state family (S = 510, 363, 512 / d = 64)
    (2, 70, 2, 8), (3, 9, 3, 5), (1, 5, 22, 2), (2, 4, 64, 1), (2, 130, 2, 4),
    (1, 2, 1, 1), (3, 2, 1, 5), (2, 5, 2, 1), (5, 3, 2, 2), (4, 17, 3, 4), (2, 9, 5, 3),
    (3, 6, 7, 3), (2, 33, 2, 7), (1, 4, 6, 4), (7, 12, 4, 4), (2, 5, 9, 2), (3, 70, 3, 5),
    (2, 11, 4, 6), (5, 19, 8, 3), (2, 7, 16, 3), (1, 3, 33, 2),
]


SWEEP_CASES = [pytest.param(B, L, d, N, dtype, v.values[0], id=f"{B}-{L}-{d}-{N}-{np.dtype(dtype).name}-{v.id}")
               for (B, L, d, N) in SWEEP for dtype in (np.float32, np.float64)
               for v in serving_variants(B, L, d, N, dtype, MODES)]


@pytest.mark.parametrize("B,L,d,N,dtype,variant", SWEEP_CASES)
def test_shape_sweep(B, L, d, N, dtype, variant):
    x = uniform_paths(B, L, d, seed=1000 + 7 * L + d, lo=-0.5, hi=0.5).astype(dtype)
    ran = [check(x, N, stream=stream, basepoint=basepoint, variant=variant) is not None for stream, basepoint in MODES]
    assert any(ran)


@pytest.mark.parametrize("variant", VARIANTS[:2], ids=VARIANT_IDS[:2])
def test_state_too_large_for_lds(variant):
    # d = 16, N = 4: 69904 scalars per path, several tiles of every level and ragged tails
    x = brownian_paths(3, 9, 16, seed=77)
    check(x, 4, variant=variant)
    check(x.astype(np.float64), 4, variant=variant)
    x = brownian_paths(2, 6, 11, seed=78)   # 11^4: not a multiple of the workgroup size
    check(x, 4, variant=variant)
    check(x, 4, stream=True, variant=variant)


# ----------------------------------------------------- matrix-core kernels, d = 4
D4_SHAPES = [
    # (B, L, N): odd and even increment counts, one increment, tile and chunk boundaries
    (3, 2, 4), (2, 3, 5), (3, 2, 6), (2, 5, 6), (5, 6, 6), (2, 64, 6), (3, 65, 6), (2, 66, 5), (1, 129, 6),
    (2, 130, 5), (2, 257, 6), (1, 258, 4), (2, 300, 6), (7, 31, 5), (4, 70, 4),
]


def d4_modes(L):
    return [m for m in MODES if not (m[0] and L > 140)]


D4_CASES = [pytest.param(B, L, N, v.values[0], id=f"{B}-{L}-{N}-{v.id}")
            for (B, L, N) in D4_SHAPES
            for v in serving_variants(B, L, 4, N, np.float32, d4_modes(L)) if v.id in ("mfma", "mfma_shard", "mfma_stream")]


@pytest.mark.parametrize("B,L,N,variant", D4_CASES)
def test_d4_matrix_core_kernels(B, L, N, variant):
    x = uniform_paths(B, L, 4, seed=2000 + 3 * L + N, lo=-0.5, hi=0.5)
    if L > 40:
        x = brownian_paths(B, L, 4, seed=2000 + 3 * L + N)
    ran = [check(x, N, stream=stream, basepoint=bp, variant=variant) is not None for stream, bp in d4_modes(L)]
    assert any(ran)


def test_large_stream_outputs_take_the_run_assembling_kernel():
    """Beyond the last-level cache (about 300 MB of output) sig_forward hands stream mode at d = 4 to the kernel
    that assembles whole runs in LDS; the shape below (B = 1024 of the stream workload's 128) is compared with the
    oracle on every prefix of a sample of paths and checked for complete, finite coverage on the rest."""
    torch = torch_mod()
    w = WORKLOADS[3]
    B = 1024
    assert sig.sig_variant_name(B, w.L, w.d, w.N, True, False) == "mfma_d4_stream"
    assert sig.sig_variant_name(w.B, w.L, w.d, w.N, True, False) == "mfma_d4_shard"
    x = brownian_paths(B, w.L, w.d, seed=w.seed + 50)
    out = torch.full((B, w.L - 1, w.channels), float("nan"), device="cuda:0")
    sig.sig_forward(torch.from_numpy(x).to("cuda:0"), w.N, stream=True, out=out)
    torch.cuda.synchronize()
    assert bool(torch.isfinite(out).all())
    forced = sig.sig_forward(torch.from_numpy(x).to("cuda:0"), w.N, stream=True, variant=sig.SIG_VARIANT_MFMA_SHARD)
    torch.cuda.synchronize()
    # every element of every path against the independent four-wavefront kernel (same arithmetic per word: same bits)
    assert torch.equal(out, forced)
    del forced
    idx = np.unique(np.concatenate([[0, 1, B - 1], np.random.default_rng(5).choice(B, size=29, replace=False)]))
    want = orc.signature(x[idx], w.N, stream=True)
    batch, single, element = level_errors(out[torch.from_numpy(idx).to("cuda:0")].cpu().numpy(), want, w.d, w.N, elementwise=True)
    assert np.all(batch <= 1e-4) and np.all(single <= 5e-4) and np.all(element <= 1e-4), (batch, single, element)


MANY_SHORT = [
    # (B, L, N): more wavefronts than SIMDs (several wavefronts share a SIMD), rounds of four increments and tails
    (700, 8, 6), (400, 30, 6), (1300, 9, 6), (2000, 5, 6), (700, 8, 5), (1300, 9, 4), (300, 8, 7), (500, 5, 7),
]
MANY_SHORT_CASES = [pytest.param(B, L, N, v.values[0], id=f"{B}-{L}-{N}-{v.id}")
                    for (B, L, N) in MANY_SHORT
                    for v in serving_variants(B, L, 4, N, np.float32, [(True, False)])
                    if v.id in ("auto", "mfma_shard", "mfma_stream")]


@pytest.mark.parametrize("B,L,N,variant", MANY_SHORT_CASES)
def test_d4_stream_mode_many_short_paths(B, L, N, variant):
    """Stream mode at d = 4 with hundreds to thousands of short paths, every path and prefix against the oracle, three
    launches each.  With more than 128 paths a SIMD holds several wavefronts of the four-wavefront kernel; at depth
    6 and 7 the first prefix signature of a round of four increments then came out, now and then, with one register
    of a level that was transposed in the lane quads before its store wrong in lanes 12..15 of every row of 16 lanes
    (stream mode stores those levels untransposed now)."""
    x = (0.2 * np.random.Generator(np.random.PCG64(B + L + N)).standard_normal((B, L, 4))).astype(np.float32)
    want = orc.signature(x, N, stream=True)
    for _ in range(3):
        assert check(x, N, stream=True, variant=variant, want=want) is not None


MANY_FINAL = [
    # (B, L, d, N): every matrix-core family in final mode with several wavefronts per SIMD
    (2500, 30, 4, 6), (2500, 9, 4, 5), (3000, 6, 4, 4), (1500, 12, 4, 7), (200, 20, 8, 5), (150, 9, 8, 6), (300, 70, 8, 4),
    (700, 12, 16, 4),
]
MANY_FINAL_CASES = [pytest.param(B, L, d, N, v.values[0], id=f"{B}-{L}-{d}-{N}-{v.id}")
                    for (B, L, d, N) in MANY_FINAL
                    for v in serving_variants(B, L, d, N, np.float32, [(False, False)])
                    if v.id in ("auto", "mfma", "mfma_shard")]


@pytest.mark.parametrize("B,L,d,N,variant", MANY_FINAL_CASES)
def test_matrix_core_kernels_with_several_wavefronts_per_simd(B, L, d, N, variant):
    """Final mode on the matrix-core families with more wavefronts than the device has SIMDs (the benchmark workloads
    put at most two on one): every path against the oracle, two launches each."""
    x = (0.2 * np.random.Generator(np.random.PCG64(B + L + d + N)).standard_normal((B, L, d))).astype(np.float32)
    want = orc.signature(x, N)
    for _ in range(2):
        assert check(x, N, variant=variant, want=want) is not None


def test_d4_depth_seven():
    x = brownian_paths(3, 21, 4, seed=707)
    check(x, 7)
    check(x, 7, stream=True, basepoint=True)
    assert sig.sig_variant_name(3, 21, 4, 7, False, False) == "mfma_d4_shard"


@pytest.mark.parametrize("B,L", [(1, 2), (2, 3), (3, 9), (2, 128), (1, 129), (2, 130), (1, 300)])
def test_d16_matrix_core_kernel(B, L):
    x = brownian_paths(B, L, 16, seed=1600 + L) if L > 20 else uniform_paths(B, L, 16, seed=1600 + L, lo=-0.3, hi=0.3)
    assert sig.sig_variant_name(B, L, 16, 4, False, False, variant=sig.SIG_VARIANT_MFMA) == "mfma_d16"
    for bp in (False, True):
        check(x, 4, basepoint=bp, variant=sig.SIG_VARIANT_MFMA)


@pytest.mark.parametrize("B,L,N", [(1, 2, 4), (2, 3, 5), (1, 4, 6), (3, 9, 5), (2, 64, 5), (1, 65, 6), (2, 66, 4),
                                   (2, 130, 5), (1, 200, 5)])
def test_d8_matrix_core_kernel(B, L, N):
    x = brownian_paths(B, L, 8, seed=800 + L) if L > 20 else uniform_paths(B, L, 8, seed=800 + L, lo=-0.4, hi=0.4)
    assert sig.sig_variant_name(B, L, 8, N, False, False, variant=sig.SIG_VARIANT_MFMA) == "mfma_d8_shard"
    for bp in (False, True):
        check(x, N, basepoint=bp, variant=sig.SIG_VARIANT_MFMA)


def test_unaligned_buffers_fall_back_to_the_generic_kernel():
    torch = torch_mod()
    w = WORKLOADS[1]
    x = workload_paths(w)[:4]
    want = orc.signature(x, w.N)
    big = torch.zeros(x.size + 1, dtype=torch.float32, device="cuda:0")
    xt = big[1:].view(x.shape)                      # 4-byte aligned only
    xt.copy_(torch.from_numpy(x))
    obig = torch.full((want.size + 1,), float("nan"), dtype=torch.float32, device="cuda:0")
    ot = obig[1:].view(want.shape)
    sig.sig_forward(xt, w.N, out=ot)
    torch.cuda.synchronize()
    batch, _ = level_errors(ot.cpu().numpy(), want, w.d, w.N)
    assert np.all(batch <= 1e-4)
    with pytest.raises(sig.SigError):
        sig.sig_forward(xt, w.N, out=ot, variant=sig.SIG_VARIANT_MFMA)


# -------------------------------------------------------------------------- edge cases
def test_single_increment_with_and_without_basepoint():
    x = uniform_paths(4, 2, 3, seed=5)
    check(x, 4)
    check(x[:, :1], 4, basepoint=True)
    check(x[:, :1], 4, basepoint=True, stream=True)


def test_zero_increments_leave_the_identity():
    x = np.ones((3, 6, 4), dtype=np.float32) * 0.37
    got = gpu_signature(x, 4)
    assert np.all(got == 0.0)
    got = gpu_signature(x, 4, stream=True)
    assert np.all(got == 0.0)


def test_repeated_points_do_not_change_the_result():
    x = brownian_paths(3, 10, 3, seed=9)
    y = np.repeat(x, 2, axis=1)
    a, b = gpu_signature(x, 4), gpu_signature(y, 4)
    np.testing.assert_array_equal(a, b)


def test_empty_batch():
    torch = torch_mod()
    x = torch.zeros((0, 5, 3), dtype=torch.float32, device="cuda:0")
    assert tuple(sig.sig_forward(x, 3).shape) == (0, 39)
    assert tuple(sig.sig_forward(x, 3, stream=True).shape) == (0, 4, 39)


@pytest.mark.parametrize("variant", [sig.SIG_VARIANT_GENERIC, sig.SIG_VARIANT_SMALL], ids=["generic", "small"])
def test_many_paths_more_than_one_grid_pass(variant):
    # more paths than the launch has workgroups: the grid-stride loop over paths
    B = (1 << 20) + 37
    x = uniform_paths(B, 2, 1, seed=3)
    got = gpu_signature(x, 2, variant=variant)
    dz = (x[:, 1, 0].astype(np.float64) - x[:, 0, 0])
    np.testing.assert_allclose(got[:, 0], dz, rtol=1e-6, atol=1e-7)
    np.testing.assert_allclose(got[:, 1], dz * dz / 2, rtol=1e-5, atol=1e-7)


def test_stream_last_entry_equals_final_result():
    for w in (WORKLOADS[0], WORKLOADS[3]):
        x = workload_paths(w)[:8]
        fin = gpu_signature(x, w.N)
        st = gpu_signature(x, w.N, stream=True)
        # the two modes may be served by different kernels: equal up to fp32 rounding
        batch, _ = level_errors(st[:, -1], fin.astype(np.float64), w.d, w.N)
        assert np.all(batch <= 1e-5), batch
        same = gpu_signature(x, w.N, variant=sig.SIG_VARIANT_GENERIC)
        st_g = gpu_signature(x, w.N, stream=True, variant=sig.SIG_VARIANT_GENERIC)
        np.testing.assert_array_equal(st_g[:, -1], same)   # same kernel, same arithmetic


def test_runs_are_bit_identical():
    for w in WORKLOADS[:4]:
        x = workload_paths(w)[:16]
        a = gpu_signature(x, w.N, stream=w.stream)
        b = gpu_signature(x, w.N, stream=w.stream)
        np.testing.assert_array_equal(a, b)


def test_errors_leave_the_output_untouched():
    torch = torch_mod()
    x = torch.zeros((2, 1, 3), dtype=torch.float32, device="cuda:0")
    out = torch.full((2, 39), 7.0, dtype=torch.float32, device="cuda:0")
    st = sig.sig_forward_raw(x.data_ptr(), 2, 1, 3, 3, 0, 0, sig.SIG_F32, out.data_ptr(),
                             torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    assert st == sig.SIG_ERR_INVALID_ARG
    assert bool(torch.all(out == 7.0))
    with pytest.raises(sig.SigError):
        sig.sig_forward(x, 3)
    with pytest.raises(sig.SigError):
        sig.sig_forward(torch.zeros((2, 4, 3), device="cuda:0"), 3, variant=sig.SIG_VARIANT_MFMA)


def test_work_is_enqueued_on_the_callers_stream():
    torch = torch_mod()
    w = WORKLOADS[0]
    x = torch.from_numpy(workload_paths(w)).to("cuda:0")
    ref = sig.sig_forward(x, w.N)
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        got = sig.sig_forward(x, w.N)
    side.synchronize()
    assert torch.equal(ref, got)


def test_long_paths_cross_many_tiles():
    # every family with a staged tile: several tiles, ragged last tile
    check(brownian_paths(2, 1000, 4, seed=31), 6)                                  # mfma_d4, 64-increment tiles
    check(brownian_paths(1, 333, 4, seed=32), 5, stream=True)                      # mfma_d4_shard
    for N, L in [(4, 301), (5, 333), (6, 140)]:                                     # mfma_d4_stream: 128-increment tiles,
        x = brownian_paths(3, L, 4, seed=40 + N)                                    # runs of 16 / 4 / 1 prefix signatures
        assert check(x, N, stream=True, variant=sig.SIG_VARIANT_MFMA_STREAM) is not None
        assert check(x, N, stream=True, basepoint=True, variant=sig.SIG_VARIANT_MFMA_STREAM) is not None
    check(brownian_paths(1, 333, 4, seed=32), 7, basepoint=True)                   # mfma_d4_shard, depth 7
    check(brownian_paths(1, 450, 8, seed=33), 5)                                   # mfma_d8_shard
    check(brownian_paths(1, 700, 16, seed=34), 4)                                  # mfma_d16, 128-increment tiles
    check(brownian_paths(2, 3000, 2, seed=35), 4, stream=True)                     # small
    check(brownian_paths(1, 2500, 3, seed=36).astype(np.float64), 6)               # generic, fp64


def test_calls_can_be_captured_in_a_graph_and_replayed():
    # nothing in the library allocates, synchronises or memsets, so a call can sit in a HIP graph
    torch = torch_mod()
    for w in (WORKLOADS[0], WORKLOADS[1], WORKLOADS[3]):
        x_host = workload_paths(w)[:16]
        x = torch.from_numpy(x_host).to("cuda:0")
        eager = sig.sig_forward(x, w.N, stream=w.stream)
        torch.cuda.synchronize()
        out = torch.zeros_like(eager)
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            sig.sig_forward(x, w.N, stream=w.stream, out=out)      # warm-up on the capture stream
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            sig.sig_forward(x, w.N, stream=w.stream, out=out)
        for rep in range(3):
            out.fill_(float("nan"))
            x.copy_(torch.from_numpy(x_host * (rep + 1)).to("cuda:0"))
            torch.cuda.synchronize()
            graph.replay()
            torch.cuda.synchronize()
            want = sig.sig_forward(x, w.N, stream=w.stream)
            torch.cuda.synchronize()
            assert torch.equal(out, want), (w.name, rep)


def test_two_streams_at_once():
    torch = torch_mod()
    wa, wb = WORKLOADS[1], WORKLOADS[3]
    xa = torch.from_numpy(workload_paths(wa)[:256]).to("cuda:0")
    xb = torch.from_numpy(workload_paths(wb)[:32]).to("cuda:0")
    ra = sig.sig_forward(xa, wa.N)
    rb = sig.sig_forward(xb, wb.N, stream=True)
    torch.cuda.synchronize()
    sa, sb = torch.cuda.Stream(), torch.cuda.Stream()
    outs = []
    for _ in range(4):
        with torch.cuda.stream(sa):
            ga = sig.sig_forward(xa, wa.N)
        with torch.cuda.stream(sb):
            gb = sig.sig_forward(xb, wb.N, stream=True)
        outs.append((ga, gb))
    sa.synchronize()
    sb.synchronize()
    for ga, gb in outs:
        assert torch.equal(ga, ra) and torch.equal(gb, rb)


# ------------------------------------------------------------------ group product
@pytest.mark.parametrize("dtype", [np.float32, np.float64])
@pytest.mark.parametrize("B,d,N", [(3, 1, 4), (2, 2, 1), (5, 2, 7), (4, 3, 4), (2, 4, 6), (1, 8, 4), (2, 16, 3)])
def test_combine_matches_the_oracle_group_product(B, d, N, dtype):
    torch = torch_mod()
    xa = uniform_paths(B, 5, d, seed=300 + d, lo=-0.6, hi=0.6)
    xb = uniform_paths(B, 4, d, seed=400 + N, lo=-0.6, hi=0.6)
    a64, b64 = orc.signature(xa, N), orc.signature(xb, N)
    a, b = a64.astype(dtype), b64.astype(dtype)
    want = np.stack([orc.group_mul(a[i].astype(np.float64), b[i].astype(np.float64), d, N) for i in range(B)])
    out = torch.full((B, a.shape[1]), float("nan"), dtype=torch.from_numpy(a).dtype, device="cuda:0")
    got = sig.sig_combine(torch.from_numpy(a).to("cuda:0"), torch.from_numpy(b).to("cuda:0"), d, N, out=out)
    torch.cuda.synchronize()
    batch, single = level_errors(got.cpu().numpy(), want, d, N)
    assert np.all(batch <= TOL[dtype]) and np.all(single <= TOL_SINGLE[dtype]), (batch, single)


def test_chunked_scan_plus_combine_equals_the_whole_scan():
    # Chen's identity on the GPU path: scan two halves that share the middle point, then join them
    torch = torch_mod()
    w = WORKLOADS[1]
    x = workload_paths(w)[:64]
    xt = torch.from_numpy(x).to("cuda:0")
    whole = sig.sig_forward(xt, w.N)
    left = sig.sig_forward(xt[:, :65].contiguous(), w.N)
    right = sig.sig_forward(xt[:, 64:].contiguous(), w.N)
    joined = sig.sig_combine(left, right, w.d, w.N)
    torch.cuda.synchronize()
    batch, _ = level_errors(joined.cpu().numpy(), whole.cpu().numpy().astype(np.float64), w.d, w.N)
    assert np.all(batch <= 1e-5), batch
    want = orc.signature(x[:8], w.N)
    batch, _ = level_errors(joined[:8].cpu().numpy(), want, w.d, w.N)
    assert np.all(batch <= 1e-4), batch


# ------------------------------------------------------------- scan as a parallel reduction over L
@pytest.mark.parametrize("dtype", [np.float32, np.float64])
@pytest.mark.parametrize("B,L,d,N,chunks", [
    (3, 130, 4, 6, 4),     # one wavefront per path family (B * chunks small -> four per path), ragged last chunk
    (600, 40, 4, 5, 2),    # B * chunks >= 512: one wavefront per chunk
    (2, 128, 8, 5, 8),     # 127 increments in 8 chunks of 16 (the last one 15)
    (2, 300, 16, 4, 4),
    (3, 50, 2, 6, 16),     # small-state family
    (2, 33, 5, 3, 4),      # fallback family
    (2, 5, 3, 4, 8),       # more chunks than increments: empty chunks are the identity
    (1, 2, 4, 4, 2),
    # depth 2: the stretches' sums are added (no products); ragged and empty last stretches, many channels, stretches of
    # several tiles
    (3, 1000, 3, 2, 16), (2, 40, 20, 2, 64), (1, 700, 64, 2, 4), (5, 2, 6, 2, 2), (2, 2000, 8, 2, 8),
    # beyond 16 channels: the stretches on the kernel for many channels (several share a workgroup; ragged and empty ones)
    (2, 150, 20, 3, 8), (1, 70, 17, 4, 4), (3, 9, 33, 3, 16),
])
def test_chunked_scan_equals_the_plain_scan(B, L, d, N, chunks, dtype):
    torch = torch_mod()
    x = brownian_paths(B, L, d, seed=L + d + chunks).astype(dtype)
    want = orc.signature(x, N)
    got = sig.sig_forward_chunked(torch.from_numpy(x).to("cuda:0"), N, chunks)
    torch.cuda.synchronize()
    batch, single = level_errors(got.cpu().numpy(), want, d, N)
    assert np.all(batch <= TOL[dtype]), batch
    # with a basepoint by value
    bp = uniform_paths(B, 1, d, seed=3)[:, 0].astype(dtype)
    want = orc.signature(np.concatenate([bp[:, None], x], axis=1), N)
    got = sig.sig_forward_chunked(torch.from_numpy(x).to("cuda:0"), N, chunks, basepoint=torch.from_numpy(bp).to("cuda:0"))
    torch.cuda.synchronize()
    batch, single = level_errors(got.cpu().numpy(), want, d, N)
    assert np.all(batch <= TOL[dtype]), batch


def test_chunked_scan_argument_checks():
    torch = torch_mod()
    x = torch.zeros((2, 9, 4), device="cuda:0")
    for bad in (0, 1, 3, 6, 1 << 17):
        with pytest.raises(sig.SigError) as e:
            sig.sig_forward_chunked(x, 4, bad)
        assert e.value.status == sig.SIG_ERR_INVALID_ARG
    need = sig.sig_forward_chunked_workspace_bytes(2, 9, 4, 4, False, 4)
    assert need == 6 * 2 * 340 * 4
    with pytest.raises(sig.SigError):
        sig.sig_forward_chunked(x, 4, 4, workspace=torch.empty(need - 4, dtype=torch.uint8, device="cuda:0"))


# ------------------------------------------------------------------ stream mode cut into chunks
# From 128 increments on (and up to 512 paths) the small-state and prefix-tree families cut a stream-mode scan into
# chunks: chunk signatures at the chunk ends, a running product along them, every chunk scanned again from the row
# before it.  Shapes: several paths per workgroup (d = 3, 8, 6), several workgroups per path (d = 5, N = 6), one level
# below a thread's word (d = 12), the one-wavefront kernel (d = 2, 3, 20), the kernel for many channels (d = 17, 20, 32);
# lengths that leave a ragged last chunk, a
# last chunk of one increment (n_inc = 129 in 4 chunks of 33) and many chunks (n_inc = 1100: 16 chunks).
@pytest.mark.parametrize("B,L,d,N", [
    (3, 130, 3, 5), (2, 257, 8, 3), (5, 200, 6, 3), (1, 130, 5, 6), (2, 140, 12, 3), (3, 1101, 3, 4), (17, 129, 7, 2),
    (4, 130, 2, 5), (2, 300, 3, 3), (3, 129, 20, 1), (2, 513, 2, 8), (4, 130, 2, 3), (2, 200, 8, 4), (3, 131, 16, 2),
    (2, 150, 20, 3), (3, 130, 17, 2), (1, 140, 32, 3), (2, 129, 9, 7 - 2),   # beyond 16 channels: the kernel for many channels
    (40, 1100, 1, 1), (3, 130, 1, 1), (2, 300, 1, 4), (5, 131, 2, 1),   # one channel, a signature of one scalar (divisions by 1)
])
@pytest.mark.parametrize("dtype", [np.float32, np.float64])
def test_stream_mode_cut_into_chunks(B, L, d, N, dtype):
    x = (brownian_paths(B, L, d, seed=L + d + N) + 0.1).astype(dtype)
    for basepoint in (False, True):
        got = check(x, N, stream=True, basepoint=basepoint)
        assert got is not None
        # the last prefix signature is the signature of the whole path, which the final-mode call computes unchunked
        final = gpu_signature(x, N, False, basepoint, sig.SIG_VARIANT_AUTO)
        batch, _ = level_errors(got[:, -1], final.astype(np.float64), d, N)
        assert np.all(batch <= 10 * TOL[dtype])


def test_chunked_stream_with_initial_and_inverse():
    # what follows the scan works on the rows in place, whichever way they were produced
    import torch
    B, L, d, N = 2, 200, 3, 4
    x = brownian_paths(B, L, d, seed=77).astype(np.float64)
    y = brownian_paths(B, 9, d, seed=78).astype(np.float64)
    y += x[:, :1] - y[:, -1:]
    initial = orc.signature(y, N)
    to_dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to("cuda:0")
    got = sig.sig_signature(to_dev(x), N, stream=True, initial=to_dev(initial), inverse=True)
    torch.cuda.synchronize()
    whole = np.concatenate([y, x[:, 1:]], axis=1)
    for j in (0, 57, L - 2):
        want = orc.signature(whole[:, :9 + j + 1][:, ::-1], N)   # inverse = the signature of the reversed path
        np.testing.assert_allclose(got[:, j].cpu().numpy(), want, rtol=1e-9, atol=1e-12)


# ------------------------------------------------------------------ depth 2 without a scan
@pytest.mark.parametrize("B,L,d", [(3, 2, 5), (2, 3, 1), (37, 9, 2), (4, 40, 32), (1, 300, 7), (2, 9, 100), (20, 17, 16), (2, 130, 64),
                                   (1, 70, 300), (5, 65, 3),
                                   # enough paths that several share a workgroup, over two tiles and a ragged last group
                                   (5000, 140, 2), (2100, 20, 4), (1100, 33, 6),
                                   # fp32 on the matrix cores: 4, 5, 8 and 16 tiles per side, several staged tiles, a
                                   # last step of 1, 2 and 3 increments
                                   (3, 50, 60), (2, 14, 75), (1, 40, 128), (2, 7, 250), (300, 6, 64)])
@pytest.mark.parametrize("dtype", [np.float32, np.float64])
def test_depth_two_as_a_contraction_over_the_increments(B, L, d, dtype):
    x = (brownian_paths(B, L, d, seed=L + d) + 0.3).astype(dtype)
    for basepoint in (False, True):
        assert check(x, 2, basepoint=basepoint, variant=sig.SIG_VARIANT_DEPTH2) is not None
    assert sig.sig_variant_name(B, L, d, 2, False, False, sig.SIG_F32 if dtype == np.float32 else sig.SIG_F64) == "depth2"
    # a basepoint given by value
    import torch
    bp = uniform_paths(B, 1, d, seed=d + 1)[:, 0].astype(dtype)
    got = sig.sig_signature(torch.from_numpy(x).to("cuda:0"), 2, basepoint=torch.from_numpy(bp).to("cuda:0"))
    torch.cuda.synchronize()
    want = orc.signature(np.concatenate([bp[:, None], x], axis=1).astype(np.float64), 2)
    batch, _ = level_errors(got.cpu().numpy(), want, d, 2)
    assert np.all(batch <= TOL[dtype])


@pytest.mark.parametrize("B,L,d", [(4, 300, 3), (3, 200, 12), (2, 150, 64), (2, 120, 40)])
def test_depth_two_far_from_the_origin(B, L, d):
    # the signature does not see where a path lies (section 2.1: it is built from increments): a path around 10 000 must
    # come out as exactly as one around 0, which rules out forming midpoints before subtracting the first point
    x = (brownian_paths(B, L, d, seed=L + d) + 10000.0).astype(np.float32)
    for basepoint in (False, True):
        if basepoint:   # a basepoint at the origin would make the first increment 10 000 long
            import torch
            bp = np.full((B, d), 10000.0, dtype=np.float32)
            got = sig.sig_signature(torch.from_numpy(x).to("cuda:0"), 2, basepoint=torch.from_numpy(bp).to("cuda:0"))
            torch.cuda.synchronize()
            want = orc.signature(np.concatenate([bp[:, None], x], axis=1).astype(np.float64), 2)
            batch, _ = level_errors(got.cpu().numpy(), want, d, 2)
            assert np.all(batch <= TOL[np.float32]), batch
        else:
            assert check(x, 2, variant=sig.SIG_VARIANT_DEPTH2) is not None


@pytest.mark.parametrize("shift,dtype", [(1, np.float32), (2, np.float32), (1, np.float64)])   # 4, 8 and 8 bytes off
def test_depth_two_on_a_path_that_starts_off_a_16_byte_boundary(shift, dtype):
    # the staging loads are 16 bytes wide only where every point starts on such a boundary
    import torch
    _depth_two_off_boundary(6, 50, 8, shift, dtype)
    _depth_two_off_boundary(3, 11, 64, shift, dtype)   # fp32: the matrix-core kernel
    _depth_two_off_boundary(2, 7, 250, shift, dtype)   # ... which steps aside where scalar loads leave no room for a tile


def _depth_two_off_boundary(B, L, d, shift, dtype):
    import torch
    x = (brownian_paths(B, L, d, seed=3) - 0.1).astype(dtype)
    flat = torch.empty(B * L * d + shift, dtype=torch.from_numpy(x).dtype, device="cuda:0")
    dev = flat[shift:].view(B, L, d)
    dev.copy_(torch.from_numpy(x))
    assert dev.data_ptr() % 16 != 0 and dev.is_contiguous()
    got = sig.sig_forward(dev, 2, variant=sig.SIG_VARIANT_DEPTH2)
    torch.cuda.synchronize()
    batch, _ = level_errors(got.cpu().numpy(), orc.signature(x.astype(np.float64), 2), d, 2)
    assert np.all(batch <= TOL[dtype])


# ------------------------------------------------------------------ many channels at low depth
@pytest.mark.parametrize("B,L,d,N", [
    (3, 9, 20, 2), (2, 40, 32, 2), (37, 6, 18, 2),      # several paths per workgroup, a ragged last workgroup
    (1, 4, 64, 2), (2, 35, 100, 2),                     # 256 and 700 threads per path
    (5, 7, 17, 3), (2, 5, 33, 3), (2, 70, 24, 3),       # a last block of 1 letter, 3267 threads per path, several tiles
    (1, 5, 20, 4), (2, 3, 18, 4),                       # depth 4: 16 000 and 11 664 threads per path
    (3, 9, 5, 3), (2, 6, 16, 2),                        # channel counts the other families serve as well
    (2, 5, 17, 5), (1, 3, 9, 7), (1, 4, 3, 9),          # deeper: beyond 16 channels, and where no other family goes
])
@pytest.mark.parametrize("dtype", [np.float32, np.float64])
def test_wide_channel_family(B, L, d, N, dtype):
    x = (brownian_paths(B, L, d, seed=B + L + d + N) + 0.2).astype(dtype)
    code = sig.SIG_F32 if dtype == np.float32 else sig.SIG_F64
    for stream in (False, True):
        for basepoint in (False, True):
            assert check(x, N, stream=stream, basepoint=basepoint, variant=sig.SIG_VARIANT_WIDE) is not None
    if N >= 7 and d >= 9:
        assert sig.sig_variant_name(B, L, d, N, False, False, code) == "wide"
    if d > 16:   # ... and it is what serves these shapes
        assert sig.sig_variant_name(B, L, d, N, False, False, code) == ("depth2" if N == 2 else "wide")
        assert sig.sig_variant_name(B, L, d, N, True, False, code) == "wide"


# ------------------------------------------------------------------ prefix-tree family
@pytest.mark.parametrize("B,L,d,N", [
    (3, 9, 7, 7),      # 16 807 words per path over 66 workgroups; 960 799 scalars per signature
    (2, 20, 4, 9), (2, 12, 4, 8), (3, 15, 5, 7), (2, 10, 6, 7), (5, 40, 3, 7), (4, 70, 2, 9),
    (37, 6, 3, 4),     # 9 words per path: 16 paths share a workgroup, the last workgroup is ragged
    (5, 5, 8, 2), (3, 7, 6, 3), (1, 2, 2, 2),
    # 9 to 16 channels: one level of d scalars per thread below its word, depths 2..6
    (3, 9, 9, 2), (20, 7, 16, 2), (2, 40, 16, 3), (3, 9, 10, 4), (2, 6, 16, 4), (2, 5, 11, 5), (1, 4, 9, 6), (2, 70, 13, 3),
    (2, 6, 12, 4), (1, 5, 14, 3), (1, 5, 15, 3),
])
@pytest.mark.parametrize("dtype", [np.float32, np.float64])
def test_prefix_tree_family(B, L, d, N, dtype):
    x = brownian_paths(B, L, d, seed=B + L + d + N).astype(dtype)
    for basepoint in (False, True):
        assert check(x, N, basepoint=basepoint, variant=sig.SIG_VARIANT_TREE) is not None
    if d ** N * L * B < 3_000_000:   # every prefix signature written (kept small for the oracle's sake)
        assert check(x, N, stream=True, variant=sig.SIG_VARIANT_TREE) is not None
        assert check(x, N, stream=True, basepoint=True, variant=sig.SIG_VARIANT_TREE) is not None
