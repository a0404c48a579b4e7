"""GPU parity, stage by stage: each HIP kernel gets the oracle's own inputs and is compared
element by element with the oracle's output for that stage.
Bars: int32 accumulators and GEMM epilogues bit-exact; scan fp32 output <= 1e-3 and Hadamard
fp32 output <= 1e-5 of the tensor's absmax; requantized int8 within 1 LSB on <= 0.1 %."""
import numpy as np
import pytest
import torch

import oracle as O
import paper_2410_13229_amd as Q
import workloads as W
from gpu_util import (assert_lsb, dev, empty, host, oracle_setup, rel_err, workspace)

pytestmark = pytest.mark.gpu


# ------------------------------------------------------------------ quantize
@pytest.mark.parametrize("n", [8, 2048, 2048 * 3 + 8, 1000003])
def test_quantize_f16_exact(n):
    rng = np.random.default_rng(n)
    x = (rng.standard_normal(n) * 40).astype(np.float16)
    x[: min(n, 6)] = np.array([0.5, 1.5, 2.5, -0.5, 300.0, -300.0], dtype=np.float16)[: min(n, 6)]
    inv = np.float32(1.0 / 0.37)
    q = empty((n,), torch.int8)
    Q.quamba_quantize_f16(dev(x), q, n, inv)
    assert np.array_equal(host(q), O.quantize(x.astype(np.float32), inv))


# ------------------------------------------------------------------ GEMM
GEMM_SHAPES = [
    # M, N, K, lda_pad, label
    (64, 64, 64, 0), (1, 4, 16, 0), (200, 192, 160, 32), (129, 260, 48, 0), (257, 80, 1536, 0),
    (64, 10240, 2560, 0), (512, 2560, 5120, 0), (300, 5120, 160, 32), (2048, 192, 5120, 0),
    (64, 2560, 5120, 0), (1000, 288, 8192, 0), (333, 1280, 1024, 0), (2048, 80, 1536, 0),
    # the widest tiles (256 x 320, eight waves) and the two-workgroups-per-CU 128 x 160 tiles, ragged in M and N
    (1100, 14000, 256, 0), (1500, 5408, 128, 0), (4000, 4096, 128, 0),  # the last: 256 x 256 tiles
    # few rows (generation): the streaming kernel without matrix tiles
    (1, 10240, 2560, 0), (4, 2560, 5120, 0), (8, 192, 5120, 0), (3, 5120, 160, 32), (2, 12, 48, 0), (7, 768, 1536, 0),
    # more than 512 tiles of 64 x 64 with deep K (the 128-byte-slice form), as in the 1024- and 256-token prefills
    (1024, 2560, 5120, 0), (256, 10240, 2560, 0),
    # in_proj and out_proj of the 2.8B layer at 2048 tokens, exactly as the benchmark launches them: 256 x 320
    # tiles over a ring that wraps 20 times, and 128 x 160 tiles with two K groups and 256-byte slices
    (2048, 10240, 2560, 0), (2048, 2560, 5120, 0),
    # few rows with the deepest K whose rows still fit the streaming kernel's LDS (2 rows) and one that no
    # longer does (3 rows: matrix tiles)
    (2, 64, 16384, 0), (3, 64, 16384, 0),
    # 65 to 255 rows (short prompts, generation with many sequences) at the 2.8B widths: 32 x 32 tiles with four K
    # groups for the narrower outputs, 64 x 64 tiles for the wide one
    (128, 2560, 5120, 0), (200, 10240, 2560, 0), (96, 192, 5120, 0), (255, 2560, 5120, 16),
]


def _random_gemm_shapes(count, seed=2024):
    """Seeded shapes inside the documented limits (K a multiple of 16, N of 4): every kernel choice has
    ragged neighbours among them."""
    rng = np.random.default_rng(seed)
    out = []
    for _ in range(count):
        M = int(rng.choice([rng.integers(1, 9), rng.integers(9, 80), rng.integers(80, 400)]))
        N = 4 * int(rng.choice([rng.integers(1, 20), rng.integers(20, 120), rng.integers(120, 360)]))
        K = 16 * int(rng.choice([rng.integers(1, 8), rng.integers(8, 40), rng.integers(40, 96)]))
        out.append((M, N, K, int(rng.choice([0, 16, 48]))))
    return out


GEMM_SHAPES += _random_gemm_shapes(28)


@pytest.mark.parametrize("M,N,K,pad", GEMM_SHAPES)
def test_gemm_acc_and_requant_bit_exact(M, N, K, pad):
    rng = np.random.default_rng(M * 7 + N * 3 + K)
    lda = K + pad
    A = rng.integers(-128, 128, (M, lda), dtype=np.int8)
    Wt = rng.integers(-128, 128, (N, K), dtype=np.int8)
    A[0, :K] = -128
    Wt[0, :] = -128  # largest possible accumulator
    acc_ref = O.int_matmul(A[:, :K], Wt)
    e0, e1 = (N // 4) // 4 * 4, (N // 2) // 4 * 4
    mult = np.array([3.1e-5, 7.7e-5, 1.9e-4], dtype=np.float32) * np.float32(5120.0 / K)
    cols = np.arange(N)
    mcol = np.where(cols < e0, mult[0], np.where(cols < e1, mult[1], mult[2])).astype(np.float32)
    want_i8 = np.clip(np.rint(acc_ref.astype(np.float32) * mcol[None, :]), -128, 127).astype(np.int8)
    for k, m in ((0, mult[0]), (1, mult[1]), (2, mult[2])):  # the oracle's own requant, per range
        sel = (cols < e0) if k == 0 else ((cols >= e0) & (cols < e1) if k == 1 else cols >= e1)
        assert np.array_equal(want_i8[:, sel], O.requant_acc(acc_ref[:, sel], m))
    ldo = N + 16
    acc = empty((M, N), torch.int32)
    out = torch.zeros((M, ldo), dtype=torch.int8, device="cuda:0")
    dA, dW = dev(A), dev(Wt)
    Q.quamba_gemm_i8(dA, lda, dW, K, M, N, K, e0, e1, mult, out, None, ldo, acc)
    assert np.array_equal(host(acc), acc_ref)
    # same call with a workspace: skinny shapes take the split-K path, the result must not change
    out2 = torch.zeros((M, ldo), dtype=torch.int8, device="cuda:0")
    acc2 = empty((M, N), torch.int32)
    ws = workspace(Q.quamba_gemm_workspace_bytes(M, N, K))
    Q.quamba_gemm_i8(dA, lda, dW, K, M, N, K, e0, e1, mult, out2, None, ldo, acc2, ws)
    assert np.array_equal(host(acc2), acc_ref)
    assert torch.equal(out, out2)
    got = host(out)
    assert np.array_equal(got[:, :N], want_i8)
    assert not got[:, N:].any()  # nothing written past N
    # without the raw sums the epilogue may restage rows through LDS: same codes
    out3 = torch.zeros((M, ldo), dtype=torch.int8, device="cuda:0")
    Q.quamba_gemm_i8(dA, lda, dW, K, M, N, K, e0, e1, mult, out3, None, ldo, None, ws)
    assert torch.equal(out, out3)
    # fp16 epilogue
    outh = torch.zeros((M, ldo), dtype=torch.float16, device="cuda:0")
    Q.quamba_gemm_i8(dA, lda, dW, K, M, N, K, N, N, mult, None, outh, ldo, None, ws)
    want_h = (acc_ref.astype(np.float32) * mult[0]).astype(np.float16)
    goth = host(outh)
    assert np.array_equal(goth[:, :N].view(np.uint16), want_h.view(np.uint16))
    assert not goth[:, N:].any()


def _random_large_gemm_shapes(count, seed=77):
    """Seeded row counts between the benchmark's sizes at the model widths: whatever tile form, row split and
    K split the planner takes for them must give the oracle's numbers."""
    rng = np.random.default_rng(seed)
    widths = [(10240, 2560), (2560, 5120), (192, 5120), (16384, 4096), (4096, 8192), (3072, 768)]
    return [(int(rng.integers(400, 7000)),) + widths[i % len(widths)] for i in range(count)]


@pytest.mark.parametrize("M,N,K", _random_large_gemm_shapes(12) + [
                                   (16384, 10240, 2560), (16384, 2560, 5120),  # the 2.8B layer at 4 x 4096 tokens
                                   (16384, 16384, 4096), (16384, 4096, 8192),  # the Jamba-shaped layer at 16384 tokens
                                   (16384, 320, 8192), (16384, 8192, 256),     # its x_proj and dt_proj
                                   # row counts that leave a nearly empty last round of tiles: the launcher runs the
                                   # rows that fill whole rounds and the rest as two launches
                                   (2304, 10240, 2560), (2049, 10240, 2560), (2600, 2560, 5120), (4500, 4096, 8192)])
def test_gemm_large_shapes_sampled_rows(M, N, K):
    """The big projections at their full sizes: raw sums and both epilogues on sampled rows against the oracle
    (which computes those rows one by one), and the row-staged epilogue (no raw sums asked for) against the
    direct one on every element."""
    rng = np.random.default_rng(M + N * 3 + K)
    A = rng.integers(-128, 128, (M, K), dtype=np.int8)
    Wt = rng.integers(-128, 128, (N, K), dtype=np.int8)
    A[0] = -128
    Wt[0] = -128
    rows = np.unique(np.concatenate([[0, 1, 255, 256, M // 2, M - 257, M - 1], rng.integers(0, M, 57),
                                     np.array([r for r in (2047, 2048, 2049, 2303, 2559, 2560, 4095, 4096) if r < M],
                                              dtype=np.int64)]).astype(np.int64))
    acc_ref = O.int_matmul(A[rows], Wt)
    e0, e1 = (N // 4) // 4 * 4, (N // 2) // 4 * 4
    mult = np.array([3.1e-5, 7.7e-5, 1.9e-4], dtype=np.float32) * np.float32(5120.0 / K)
    want = np.concatenate([O.requant_acc(acc_ref[:, :e0], mult[0]), O.requant_acc(acc_ref[:, e0:e1], mult[1]),
                           O.requant_acc(acc_ref[:, e1:], mult[2])], axis=1)
    dA, dW, drows = dev(A), dev(Wt), dev(rows)
    ws = workspace(Q.quamba_gemm_workspace_bytes(M, N, K))
    acc = empty((M, N), torch.int32)
    out = torch.zeros((M, N), dtype=torch.int8, device="cuda:0")
    Q.quamba_gemm_i8(dA, K, dW, K, M, N, K, e0, e1, mult, out, None, N, acc, ws)
    assert np.array_equal(host(acc[drows]), acc_ref)
    assert np.array_equal(host(out[drows]), want)
    del acc
    out3 = torch.zeros((M, N), dtype=torch.int8, device="cuda:0")
    Q.quamba_gemm_i8(dA, K, dW, K, M, N, K, e0, e1, mult, out3, None, N, None, ws)
    torch.cuda.synchronize()
    assert torch.equal(out, out3)
    outh = torch.zeros((M, N), dtype=torch.float16, device="cuda:0")
    Q.quamba_gemm_i8(dA, K, dW, K, M, N, K, N, N, mult, None, outh, N, None, ws)
    want_h = (acc_ref.astype(np.float32) * mult[0]).astype(np.float16)
    assert np.array_equal(host(outh[drows]).view(np.uint16), want_h.view(np.uint16))


@pytest.mark.parametrize("kind", [7, 11, 12, 13])
@pytest.mark.parametrize("M,N,K", [(64, 2560, 5120), (37, 204, 512), (64, 96, 256), (5, 1000, 1280)])
def test_gemm_generation_step_kinds_forced(kind, M, N, K):
    """The tile forms the planner reserves for generation-step shapes (64 x 32 and 32 x 32 tiles with two or
    four K groups, 64 x 64 with two), forced onto ragged shapes through the tuning hook: raw sums, codes and
    the half-precision epilogue against the oracle."""
    rng = np.random.default_rng(kind * 1000 + M + N + K)
    A = rng.integers(-128, 128, (M, K), dtype=np.int8)
    Wt = rng.integers(-128, 128, (N, K), dtype=np.int8)
    A[0] = -128
    Wt[0] = -128
    acc_ref = O.int_matmul(A, Wt)
    mult = np.array([3.1e-5, 7.7e-5, 1.9e-4], dtype=np.float32) * np.float32(5120.0 / K)
    e0, e1 = (N // 4) // 4 * 4, (N // 2) // 4 * 4
    want = np.concatenate([O.requant_acc(acc_ref[:, :e0], mult[0]), O.requant_acc(acc_ref[:, e0:e1], mult[1]),
                           O.requant_acc(acc_ref[:, e1:], mult[2])], axis=1)
    dA, dW = dev(A), dev(Wt)
    Q.quamba_debug_set_gemm_variant(kind)
    try:
        acc = empty((M, N), torch.int32)
        out = torch.zeros((M, N), dtype=torch.int8, device="cuda:0")
        Q.quamba_gemm_i8(dA, K, dW, K, M, N, K, e0, e1, mult, out, None, N, acc)
        out2 = torch.zeros((M, N), dtype=torch.int8, device="cuda:0")
        Q.quamba_gemm_i8(dA, K, dW, K, M, N, K, e0, e1, mult, out2, None, N, None)  # row-staged epilogue
        outh = torch.zeros((M, N), dtype=torch.float16, device="cuda:0")
        Q.quamba_gemm_i8(dA, K, dW, K, M, N, K, N, N, mult, None, outh, N, None)
    finally:
        Q.quamba_debug_set_gemm_variant(-1)
    assert np.array_equal(host(acc), acc_ref)
    assert np.array_equal(host(out), want)
    assert torch.equal(out, out2)
    want_h = (acc_ref.astype(np.float32) * mult[0]).astype(np.float16)
    assert np.array_equal(host(outh).view(np.uint16), want_h.view(np.uint16))


@pytest.mark.parametrize("kind", [2, 4, 8, 9, 10])
@pytest.mark.parametrize("M,N,K", [(300, 700, 256), (130, 164, 512), (257, 332, 768), (40, 64, 1280)])
def test_gemm_ring_of_two_kinds_forced(kind, M, N, K):
    """The tile forms with a ring of two stages (256 x 320, 256 x 256, 128 x 160 with and without K groups, 64 x 64
    with 256-byte slices) keep their per-slice barrier in front of the last sub-slice and run the last slice in a
    copy of the loop body; forced onto ragged shapes whose K is one, two, three, five or ten slices: raw sums, codes
    and the half-precision epilogue against the oracle."""
    rng = np.random.default_rng(kind * 977 + M + N + K)
    A = rng.integers(-128, 128, (M, K), dtype=np.int8)
    Wt = rng.integers(-128, 128, (N, K), dtype=np.int8)
    A[-1] = -128
    Wt[-1] = -128
    acc_ref = O.int_matmul(A, Wt)
    mult = np.array([3.1e-5, 7.7e-5, 1.9e-4], dtype=np.float32) * np.float32(5120.0 / K)
    e0, e1 = (N // 4) // 4 * 4, (N // 2) // 4 * 4
    want = np.concatenate([O.requant_acc(acc_ref[:, :e0], mult[0]), O.requant_acc(acc_ref[:, e0:e1], mult[1]),
                           O.requant_acc(acc_ref[:, e1:], mult[2])], axis=1)
    dA, dW = dev(A), dev(Wt)
    Q.quamba_debug_set_gemm_variant(kind)
    try:
        acc = empty((M, N), torch.int32)
        out = torch.zeros((M, N), dtype=torch.int8, device="cuda:0")
        Q.quamba_gemm_i8(dA, K, dW, K, M, N, K, e0, e1, mult, out, None, N, acc)
        out2 = torch.zeros((M, N), dtype=torch.int8, device="cuda:0")
        Q.quamba_gemm_i8(dA, K, dW, K, M, N, K, e0, e1, mult, out2, None, N, None)  # row-staged epilogue
        outh = torch.zeros((M, N), dtype=torch.float16, device="cuda:0")
        Q.quamba_gemm_i8(dA, K, dW, K, M, N, K, N, N, mult, None, outh, N, None)
    finally:
        Q.quamba_debug_set_gemm_variant(-1)
    assert np.array_equal(host(acc), acc_ref)
    assert np.array_equal(host(out), want)
    assert torch.equal(out, out2)
    want_h = (acc_ref.astype(np.float32) * mult[0]).astype(np.float16)
    assert np.array_equal(host(outh).view(np.uint16), want_h.view(np.uint16))


def test_gemm_rejects_bad_arguments():
    a = torch.zeros((16, 32), dtype=torch.int8, device="cuda:0")
    o = torch.zeros((16, 16), dtype=torch.int8, device="cuda:0")
    with pytest.raises(Q.QuambaError):
        Q.quamba_gemm_i8(a, 32, a, 32, 16, 16, 24, 16, 16, [1, 1, 1], o, None, 16, None)  # K % 16
    with pytest.raises(Q.QuambaError):
        Q.quamba_gemm_i8(a, 32, a, 32, 16, 16, 32, 16, 16, [1, 1, 1], None, None, 16, None)  # no output
    with pytest.raises(Q.QuambaError):
        Q.quamba_gemm_i8(None, 32, a, 32, 16, 16, 32, 16, 16, [1, 1, 1], o, None, 16, None)  # NULL


# ------------------------------------------------------------------ conv
@pytest.mark.parametrize("Bt,L,Di", [(1, 1, 64), (2, 3, 128), (3, 37, 192), (1, 256, 1536), (2, 100, 5120),
                                     (2, 21, 36), (1, 7, 100),  # channel counts that only the 4-channel form serves
                                     (1, 2048, 5120), (3, 1000, 208)])
def test_conv_prefill(Bt, L, Di):
    rng = np.random.default_rng(Bt * 1000 + L)
    ldx = 2 * Di
    xz = rng.integers(-128, 128, (Bt, L, ldx), dtype=np.int8)
    wq = rng.integers(-128, 128, (Di, 4), dtype=np.int8)
    b = (rng.standard_normal(Di) * 0.2).astype(np.float32)
    sc = {"m_conv": np.float32(2.3e-4), "inv_s_x": np.float32(1 / 0.011), "s_xpre": np.float32(0.031)}
    want = O.q_conv_prefill(xz[..., :Di], wq, b, sc)
    xq = empty((Bt, L, Di), torch.int8)
    cs = empty((Bt, Di, 3), torch.float16)
    Q.quamba_conv_silu_quant(dev(xz), ldx, dev(wq), dev(b), Bt, L, Di, sc["m_conv"], sc["inv_s_x"], sc["s_xpre"],
                             xq, cs)
    assert_lsb(host(xq), want, "x_q")
    hist = np.zeros((Bt, 3, Di), dtype=np.float32)
    take = min(L, 3)
    hist[:, 3 - take:] = sc["s_xpre"] * xz[:, L - take:, :Di].astype(np.float32)
    assert np.array_equal(host(cs), hist.transpose(0, 2, 1).astype(np.float16))


@pytest.mark.parametrize("Bt,Di", [(1, 64), (5, 192), (64, 5120)])
def test_conv_step(Bt, Di):
    rng = np.random.default_rng(Bt + Di)
    ldx = 2 * Di
    xz = rng.integers(-128, 128, (Bt, ldx), dtype=np.int8)
    wq = rng.integers(-128, 128, (Di, 4), dtype=np.int8)
    b = (rng.standard_normal(Di) * 0.2).astype(np.float32)
    st = (rng.standard_normal((Bt, Di, 3)) * 2.2).astype(np.float16)
    sc = {"s_cw": np.float32(6e-4), "s_xpre": np.float32(0.031), "inv_s_x": np.float32(1 / 0.011)}
    want, want_state = O.q_conv_step(xz[:, :Di], st, wq, b, sc)
    xq = empty((Bt, Di), torch.int8)
    dst = dev(st)
    Q.quamba_conv_step(dev(xz), ldx, dev(wq), dev(b), Bt, Di, sc["s_cw"], sc["s_xpre"], sc["inv_s_x"], xq, dst)
    assert_lsb(host(xq), want, "x_q")
    assert np.array_equal(host(dst).view(np.uint16), want_state.view(np.uint16))


# ------------------------------------------------------------------ scan
def _scan_inputs(rng, Bt, L, Di, N=16):
    sc = {"s_x": np.float32(0.004), "s_dt": np.float32(0.03), "s_z": np.float32(0.03), "s_B": np.float32(0.02),
          "s_C": np.float32(0.02), "s_A": np.float32(16 / 127), "s_D": np.float32(1 / 127)}
    x = rng.integers(-128, 128, (Bt, L, Di), dtype=np.int8)
    dt = rng.integers(-128, 128, (Bt, L, Di), dtype=np.int8)
    xz = rng.integers(-128, 128, (Bt, L, 2 * Di), dtype=np.int8)
    dbc = rng.integers(-128, 128, (Bt, L, 48 + 2 * N), dtype=np.int8)
    A = -rng.integers(1, 128, (Di, N)).astype(np.int8)
    D = rng.integers(-128, 128, Di, dtype=np.int8)
    u = rng.random(Di)
    step = np.exp(u * (np.log(1e-1) - np.log(1e-3)) + np.log(1e-3))
    bias = (step + np.log(-np.expm1(-step))).astype(np.float32)
    return sc, x, dt, xz, dbc, A, D, bias


@pytest.fixture(params=["chunked", "sweep"])
def scan_variant(request):
    """Both forms of the prefill scan: three chunked passes, and one sweep per sequence (taken wherever its
    layout rules hold: channel counts that are not multiples of 32 run the chunked form under either setting)."""
    Q.quamba_debug_set_scan_variant({"chunked": 1, "sweep": 2}[request.param])
    yield request.param
    Q.quamba_debug_set_scan_variant(0)


@pytest.mark.parametrize("Bt,L,Di,with_h0", [(1, 1, 64, False), (2, 45, 128, True), (1, 300, 320, False),
                                              (3, 67, 192, True), (1, 1000, 256, True), (1, 256, 1536, False),
                                              (2, 131, 1100, True), (1, 2048, 5120, True), (2, 129, 64, True),
                                              (1, 128, 96, False), (2, 8, 32, True),
                                              (9, 40, 1024, True),  # more than one workgroup per CU in the sweep
                                              # sequence ends on either side of the sweep's 64-token superblocks and 8-token groups
                                              (5, 65, 64, True), (1, 63, 32, False), (3, 127, 96, True), (2, 64, 64, False),
                                              (1, 71, 160, True)])
def test_scan_prefill(Bt, L, Di, with_h0, scan_variant):
    rng = np.random.default_rng(L * 31 + Di)
    sc, x, dt, xz, dbc, A, D, bias = _scan_inputs(rng, Bt, L, Di)
    R = 48
    h0 = (rng.standard_normal((Bt, Di, 16)) * 0.1).astype(np.float32) if with_h0 else None
    g_ref, g16_ref, h_ref = O.q_scan(x, dt, xz[..., Di:], dbc[..., R:R + 16], dbc[..., R + 16:], A, D, bias, sc, h0)
    full = dict(sc)
    for k in Q.SCALE_FIELDS:
        full.setdefault(k, 1.0)
    dxz, ddbc = dev(xz), dev(dbc)
    g16 = empty((Bt, L, Di), torch.float16)
    y32 = empty((Bt, L, Di), torch.float32)
    ssm = dev(h0) if with_h0 else torch.zeros((Bt, Di, 16), dtype=torch.float32, device="cuda:0")
    ws = workspace(Q.quamba_scan_workspace_bytes(Bt, L, Di))
    Q.quamba_scan_prefill(dev(x), dev(dt), dxz[..., Di:], 2 * Di, ddbc[..., R:], ddbc[..., R + 16:], dbc.shape[-1],
                          dev(A), dev(D), dev(bias), full, Bt, L, Di, g16, y32, ssm, ws)
    assert rel_err(host(y32), g_ref) <= 1e-3
    assert rel_err(host(g16).astype(np.float64), g_ref) <= 1e-3
    assert rel_err(host(ssm), h_ref) <= 1e-3
    # tighter: the fp32 path should sit near fp32 rounding of the fp64 recurrence
    assert rel_err(host(y32), g_ref) <= 2e-5


@pytest.mark.parametrize("Bt,L,Di,R,with_h0", [(1, 1, 64, 16, False), (2, 45, 128, 48, True), (1, 300, 320, 160, False),
                                                (3, 67, 192, 32, True), (1, 1000, 256, 256, True),
                                                (1, 256, 1536, 48, False), (1, 130, 100, 80, False),
                                                # the 2.8B layer at 2048 tokens and the Jamba-shaped one at 4096
                                                (1, 2048, 5120, 160, False), (1, 4096, 8192, 256, True),
                                                (9, 70, 1024, 64, True),  # more than one sweep workgroup per CU
                                                # whole workgroups of channels and dt_rank <= 160: the chunked pass stages its
                                                # dt_proj operands in LDS (one piece per row, an odd number of pieces, nine)
                                                (2, 200, 256, 16, True), (1, 333, 512, 80, False), (1, 97, 768, 144, True)])
def test_scan_prefill_with_fused_dt_proj(Bt, L, Di, R, with_h0, scan_variant):
    """dt_q computed inside the scan's first pass: bit-exact codes, same scan tolerances."""
    rng = np.random.default_rng(L * 17 + Di + R)
    sc, x, _, xz, _, A, D, bias = _scan_inputs(rng, Bt, L, Di)
    NX = R + 32
    dbc = rng.integers(-128, 128, (Bt, L, NX), dtype=np.int8)
    W_dt = rng.integers(-128, 128, (Di, R), dtype=np.int8)
    m_dt = np.float32(127.0 / (64.0 * 74.0 * np.sqrt(R) * 3.0))
    acc = O.int_matmul(dbc[..., :R].reshape(-1, R), W_dt)
    dt = O.requant_acc(acc, m_dt).reshape(Bt, L, Di)
    h0 = (rng.standard_normal((Bt, Di, 16)) * 0.1).astype(np.float32) if with_h0 else None
    g_ref, g16_ref, h_ref = O.q_scan(x, dt, xz[..., Di:], dbc[..., R:R + 16], dbc[..., R + 16:], A, D, bias, sc, h0)
    full = dict(sc)
    for k in Q.SCALE_FIELDS:
        full.setdefault(k, 1.0)
    dxz, ddbc = dev(xz), dev(dbc)
    g16 = empty((Bt, L, Di), torch.float16)
    y32 = empty((Bt, L, Di), torch.float32)
    dt_q = torch.full((Bt, L, Di), 99, dtype=torch.int8, device="cuda:0")
    ssm = dev(h0) if with_h0 else torch.zeros((Bt, Di, 16), dtype=torch.float32, device="cuda:0")
    ws = workspace(Q.quamba_scan_workspace_bytes(Bt, L, Di))
    Q.quamba_scan_prefill_dtproj(dev(x), ddbc, NX, dev(W_dt), R, m_dt, dt_q, dxz[..., Di:], 2 * Di, ddbc[..., R:],
                                 ddbc[..., R + 16:], NX, dev(A), dev(D), dev(bias), full, Bt, L, Di, g16, y32, ssm,
                                 ws)
    assert np.array_equal(host(dt_q), dt)
    assert rel_err(host(y32), g_ref) <= 2e-5
    assert rel_err(host(g16).astype(np.float64), g_ref) <= 1e-3
    assert rel_err(host(ssm), h_ref) <= 1e-3


def test_scan_prefill_with_fused_dt_proj_rejects_odd_rank():
    rng = np.random.default_rng(5)
    Bt, L, Di, R = 1, 8, 64, 24
    sc, x, _, xz, _, A, D, bias = _scan_inputs(rng, Bt, L, Di)
    full = dict(sc)
    for k in Q.SCALE_FIELDS:
        full.setdefault(k, 1.0)
    dbc = dev(rng.integers(-128, 128, (Bt, L, 64), dtype=np.int8))
    ws = workspace(Q.quamba_scan_workspace_bytes(Bt, L, Di))
    with pytest.raises(Q.QuambaError):
        Q.quamba_scan_prefill_dtproj(dev(x), dbc, 64, dev(rng.integers(-128, 128, (Di, R), dtype=np.int8)), R, 1e-3,
                                     empty((Bt, L, Di), torch.int8), dev(xz)[..., Di:], 2 * Di, dbc[..., 32:],
                                     dbc[..., 48:], 64, dev(A), dev(D), dev(bias), full, Bt, L, Di,
                                     empty((Bt, L, Di), torch.float16), None, None, ws)



@pytest.mark.parametrize("prefill", [False, True])
def test_scan_output_at_the_edge_of_half_precision(prefill, scan_variant):
    """The gated scan output is rounded to half precision once (Section 4.2: the quantized SSM "outputs half
    precision"): values up to the largest finite half (65504) come out finite and equal to the oracle's, values
    beyond it become infinities of the right sign on both sides (IEEE conversion, no saturation)."""
    Bt, L, Di, R = 2, (5 if prefill else 1), 64, 48
    rng = np.random.default_rng(7)
    sc, x, dt, xz, dbc, A, D, bias = _scan_inputs(rng, Bt, L, Di)
    # y = D x with D = 1 (B = C = 0 switch the state off), gate SiLU(40) = 40: g = 40 * 13 * x_q
    sc = dict(sc, s_x=np.float32(13.0), s_D=np.float32(1 / 127), s_z=np.float32(40 / 127))
    dbc[...] = 0
    D[:] = 127
    xz[..., Di:] = 127
    x[...] = rng.integers(-120, 121, x.shape)
    x[:, :, 0], x[:, :, 1], x[:, :, 2], x[:, :, 3] = 125, -125, 127, -127   # 65000, -65000, 66040, -66040
    x[:, :, 4], x[:, :, 5] = 126, -126                                        # 65520: the tie that rounds to infinity
    with np.errstate(over="ignore"):
        g_ref, g16_ref, h_ref = O.q_scan(x, dt, xz[..., Di:], dbc[..., R:R + 16], dbc[..., R + 16:], A, D, bias, sc, None)
    assert np.isinf(g16_ref[:, :, 2]).all() and np.isinf(g16_ref[:, :, 3]).all() and np.isfinite(g16_ref[:, :, :2]).all()
    full = dict(sc)
    for k in Q.SCALE_FIELDS:
        full.setdefault(k, 1.0)
    dxz, ddbc = dev(xz), dev(dbc)
    g16 = empty((Bt, L, Di), torch.float16)
    ssm = torch.zeros((Bt, Di, 16), dtype=torch.float32, device="cuda:0")
    if prefill:
        ws = workspace(Q.quamba_scan_workspace_bytes(Bt, L, Di))
        Q.quamba_scan_prefill(dev(x), dev(dt), dxz[..., Di:], 2 * Di, ddbc[..., R:], ddbc[..., R + 16:], dbc.shape[-1],
                              dev(A), dev(D), dev(bias), full, Bt, L, Di, g16, None, ssm, ws)
    else:
        Q.quamba_scan_step(dev(x[:, 0]), dev(dt[:, 0]), dxz[:, 0, Di:], 2 * Di, ddbc[:, 0, R:], ddbc[:, 0, R + 16:],
                           dbc.shape[-1], dev(A), dev(D), dev(bias), full, Bt, Di, g16, None, ssm)
    got = host(g16).reshape(Bt, L, Di)
    fin = np.isfinite(g16_ref)
    fin[:, :, 4:6] = False  # the exact tie may fall either way in fp32 against fp64: not compared
    assert np.isfinite(got[fin]).all()
    assert rel_err(got[fin].astype(np.float64), g_ref[fin]) <= 1e-3
    assert np.array_equal(got[:, :, 2:4], g16_ref[:, :, 2:4])  # +inf / -inf
    assert np.abs(got[:, :, :2].astype(np.float64)).min() >= 64960

@pytest.mark.parametrize("Bt,Di", [(1, 64), (7, 192), (64, 5120)])
def test_scan_step(Bt, Di):
    rng = np.random.default_rng(Bt * 13 + Di)
    sc, x, dt, xz, dbc, A, D, bias = _scan_inputs(rng, Bt, 1, Di)
    R = 48
    h0 = (rng.standard_normal((Bt, Di, 16)) * 0.1).astype(np.float32)
    g_ref, g16_ref, h_ref = O.q_scan(x, dt, xz[..., Di:], dbc[..., R:R + 16], dbc[..., R + 16:], A, D, bias, sc, h0)
    full = dict(sc)
    for k in Q.SCALE_FIELDS:
        full.setdefault(k, 1.0)
    dxz, ddbc = dev(xz[:, 0]), dev(dbc[:, 0])
    g16 = empty((Bt, Di), torch.float16)
    y32 = empty((Bt, Di), torch.float32)
    ssm = dev(h0)
    Q.quamba_scan_step(dev(x[:, 0]), dev(dt[:, 0]), dxz[:, Di:], 2 * Di, ddbc[:, R:], ddbc[:, R + 16:],
                       dbc.shape[-1], dev(A), dev(D), dev(bias), full, Bt, Di, g16, y32, ssm)
    assert rel_err(host(y32), g_ref[:, 0]) <= 2e-5
    assert rel_err(host(ssm), h_ref) <= 2e-6
    assert rel_err(host(g16).astype(np.float64), g_ref[:, 0]) <= 1e-3


# ------------------------------------------------------------------ Hadamard + quant
@pytest.mark.parametrize("M,n", [(3, 16), (5, 128), (4, 192), (4, 320), (33, 1536), (17, 5120), (9, 8192),
                                 (2, 2048), (2, 640), (1, 16384)])
def test_hadamard_quant(M, n):
    rng = np.random.default_rng(n + M)
    g = rng.standard_normal((M, n)).astype(np.float16)
    g[0, n // 3] = np.float16(300.0)  # an outlier channel
    gH = g.astype(np.float64) @ O.hadamard_matrix(n).astype(np.float64).T
    sc = {"inv_s_y": np.float32(127.0 / np.abs(gH).max())}
    gH_ref, q_ref = O.q_hadamard_quant(g, sc)
    q = empty((M, n), torch.int8)
    f = empty((M, n), torch.float32)
    Q.quamba_hadamard_quant(dev(g), M, n, sc["inv_s_y"], q, f)
    assert rel_err(host(f), gH_ref) <= 1e-5
    assert_lsb(host(q), q_ref, "gH_q")
    # unit vectors pick out columns of H (orientation of the non-symmetric factors)
    e = np.zeros((2, n), dtype=np.float16)
    e[0, 1] = 1
    e[1, n - 2] = 1
    q2, f2 = empty((2, n), torch.int8), empty((2, n), torch.float32)
    Q.quamba_hadamard_quant(dev(e), 2, n, 1.0, q2, f2)
    H = O.hadamard_matrix(n)
    assert np.array_equal(host(f2), np.stack([H[:, 1], H[:, n - 2]]).astype(np.float32))


def test_hadamard_rejects_unsupported_order():
    g = torch.zeros((1, 1792), dtype=torch.float16, device="cuda:0")
    q = torch.zeros((1, 1792), dtype=torch.int8, device="cuda:0")
    with pytest.raises(Q.QuambaError) as e:
        Q.quamba_hadamard_quant(g, 1, 1792, 1.0, q, None)  # 7 * 256
    assert e.value.code == -2


# ------------------------------------------------------------------ add + RMSNorm + quant
@pytest.mark.parametrize("M,Dm", [(1, 64), (37, 768), (256, 2560), (5, 4096)])
def test_add_rmsnorm_quant(M, Dm):
    rng = np.random.default_rng(M + Dm)
    a = rng.standard_normal((M, Dm)).astype(np.float16)
    r = (rng.standard_normal((M, Dm)) * 3).astype(np.float16)
    wt = (1 + 0.1 * rng.standard_normal(Dm)).astype(np.float16)
    inv = np.float32(127 / 5.0)
    q_ref, res_ref = O.add_rmsnorm_quant(a, r, wt, inv, eps=1e-5)
    dres = dev(r)
    q = empty((M, Dm), torch.int8)
    Q.quamba_add_rmsnorm_quant(dev(a), dres, dev(wt), 1e-5, inv, q, M, Dm)
    assert np.array_equal(host(dres).view(np.uint16), res_ref.view(np.uint16))
    assert_lsb(host(q), q_ref, "u_q")


# ------------------------------------------------------------------ clipping scalar search
@pytest.mark.parametrize("n,bits", [(1, 8), (255, 8), (70001, 8), (1 << 20, 8), (300007, 4)])
def test_clip_search_matches_oracle(n, bits):
    """Section 5.1 (enhanced variant): the fixed point of the clipping-scalar iteration, against
    the oracle on heavy-tailed data, at sizes below one workgroup, ragged, and beyond the grid."""
    rng = np.random.default_rng(n + bits)
    x = rng.standard_normal(n).astype(np.float32)
    if n > 100:
        x[rng.choice(n, max(n // 2000, 1), replace=False)] *= np.float32(11.0)
    want = O.optimal_clip(x, bits=bits)
    ws = workspace(Q.quamba_clip_search_workspace_bytes())
    got, iters = Q.quamba_clip_search(dev(x), n, bits, 32, ws)
    assert got == pytest.approx(want, rel=1e-12), (got, want)
    assert 0 <= iters <= 32
    again, _ = Q.quamba_clip_search(dev(x), n, bits, 32, ws)
    assert again == got  # fixed summation order


def test_clip_search_degenerate_and_errors():
    ws = workspace(Q.quamba_clip_search_workspace_bytes())
    z = torch.zeros(1000, dtype=torch.float32, device="cuda:0")
    assert Q.quamba_clip_search(z, 1000, 8, 32, ws) == (0.0, 0)
    c = torch.full((777,), -2.5, dtype=torch.float32, device="cuda:0")
    assert Q.quamba_clip_search(c, 777, 8, 32, ws) == (2.5, 0)
    x = dev(np.arange(1, 50001, dtype=np.float32))
    one, it1 = Q.quamba_clip_search(x, 50000, 8, 1, ws)
    assert it1 == 1 and one == pytest.approx(O.optimal_clip(host(x), max_iters=1), rel=1e-12)
    for bad in (dict(n=0), dict(bits=1), dict(bits=17), dict(iters=0)):
        with pytest.raises(Q.QuambaError):
            Q.quamba_clip_search(x, bad.get("n", 10), bad.get("bits", 8), bad.get("iters", 4), ws)
    with pytest.raises(Q.QuambaError):
        Q.quamba_clip_search(x, 10, 8, 4, workspace(256))


def test_empty_inputs_are_no_ops_and_an_empty_mixer_call_is_a_clear_error():
    """Zero rows or zero elements: the stage entry points return without touching their outputs;
    the mixer, whose shapes come from (batch, L), refuses batch or L below 1."""
    canary = torch.full((64,), 7, dtype=torch.int8, device="cuda:0")
    half = torch.zeros((64,), dtype=torch.float16, device="cuda:0")
    Q.quamba_quantize_f16(half, canary, 0, 1.0)
    Q.quamba_hadamard_quant(half, 0, 64, 1.0, canary, None)
    Q.quamba_add_rmsnorm_quant(half, half.clone(), half, 1e-5, 1.0, canary, 0, 64)
    w = torch.zeros((64, 64), dtype=torch.int8, device="cuda:0")
    Q.quamba_gemm_i8(w, 64, w, 64, 0, 64, 64, 64, 64, [1.0, 1.0, 1.0], canary, None, 64, None, None)
    Q.quamba_x_encode(Q.XFMT_LOG2, torch.zeros(4, device="cuda:0"), 0, 1.0, canary.view(torch.uint8))
    assert np.all(host(canary) == 7)
    cfg = W.tiny_config(name="te", d_model=64, d_inner=128, dt_rank=16, config_id=93)
    w_, qw, sc = oracle_setup(cfg)
    from gpu_util import qweights_to_dev
    qd = qweights_to_dev(qw)
    out = empty((1, 1, cfg.d_model), torch.float16)
    ws = workspace(Q.quamba_workspace_bytes(cfg, 1, 1))
    for Bt, L in ((0, 4), (1, 0)):
        with pytest.raises(Q.QuambaError):
            Q.quamba_mixer_prefill(cfg, qd, sc, half, Bt, L, out, None, None, None, ws)
    assert Q.quamba_workspace_bytes(cfg, 0, 4) == 0
