"""GPU parity of the individual HIP kernels against the CPU oracle, through the C ABI."""
import numpy as np
import pytest
import torch

import kvpr_inputs
from oracle import kvpr_oracle as ko
from kvpr_testlib import dev, rel_err, rel_err_rms

pytestmark = pytest.mark.gpu

TOL = 1e-2        # stated bar: max relative error in fp16 with fp32 accumulation
TIGHT = 2e-3      # what the arithmetic should actually achieve (fp16 rounding of the result is 4.9e-4)


@pytest.fixture(scope="module")
def k():
    import paper_2411_17089_amd as k
    return k


# ---- recompute GEMM (Eq. 7 + bias) ------------------------------------------
@pytest.mark.parametrize("variant", [0, 1, 2, 3])
@pytest.mark.parametrize("M,N,K", [(1, 1536, 768), (37, 1536, 768), (128, 1536, 768), (300, 520, 256),
                                   (1000, 8, 64), (257, 256, 128), (513, 776, 192)])
def test_recompute_gemm_matches_oracle(k, variant, M, N, K):
    print(f"gemm variant={variant} M={M} N={N} K={K}", flush=True)
    rng = np.random.default_rng(M * 7 + N)
    A = rng.standard_normal((M, K)).astype(np.float16)
    W = (rng.standard_normal((N, K)) * 0.05).astype(np.float16)
    bias = (rng.standard_normal(N) * 0.1).astype(np.float16)
    ldc = N + 8
    c = torch.full((M, ldc), float("nan"), dtype=torch.float16, device="cuda")
    k.lib.kvpr_debug_set_gemm_variant(variant)
    try:
        k.kvpr_recompute_gemm(dev(A), dev(W), dev(bias), c, M, N, K, ldc)
        torch.cuda.synchronize()
    finally:
        k.lib.kvpr_debug_set_gemm_variant(0)
    got = c.cpu().numpy()
    ref = ko.project(A, W.T, bias)
    assert np.isnan(got[:, N:]).all(), "columns beyond N must not be written"
    assert rel_err(got[:, :N], ref) <= TIGHT
    assert rel_err_rms(got[:, :N], ref) <= TOL
    # fp16-rounded oracle: at most 1 ulp apart almost everywhere
    assert np.mean(got[:, :N].astype(np.float64) != ko.round_fp16(ref)) < 0.05


@pytest.mark.parametrize("mapping", [0, 1])
@pytest.mark.parametrize("M,N,K", [(700, 2304, 256), (2100, 2048, 128), (5000, 4104, 64), (300, 3328, 192)])
def test_recompute_gemm_tile_mappings(k, mapping, M, N, K):
    """Both workgroup-to-tile mappings (XCDs split the tile rows / the tile columns) on shapes with 8-17 tile
    columns, uneven column bands and ragged tails in M and N: every element written once, none outside."""
    print(f"gemm mapping={mapping} M={M} N={N} K={K}", flush=True)
    rng = np.random.default_rng(M + N + mapping)
    A = rng.standard_normal((M, K)).astype(np.float16)
    W = (rng.standard_normal((N, K)) * 0.05).astype(np.float16)
    bias = (rng.standard_normal(N) * 0.1).astype(np.float16)
    ldc = N + 8
    c = torch.full((M + 3, ldc), float("nan"), dtype=torch.float16, device="cuda")
    k.lib.kvpr_debug_set_gemm_mapping(mapping)
    try:
        k.kvpr_recompute_gemm(dev(A), dev(W), dev(bias), c, M, N, K, ldc)
        torch.cuda.synchronize()
    finally:
        k.lib.kvpr_debug_set_gemm_mapping(-1)
    got = c.cpu().numpy()
    assert np.isnan(got[:M, N:]).all() and np.isnan(got[M:]).all()
    assert rel_err(got[:M, :N], ko.project(A, W.T, bias)) <= TIGHT


def test_recompute_gemm_no_bias_and_empty(k):
    rng = np.random.default_rng(1)
    A = rng.standard_normal((70, 128)).astype(np.float16)
    W = (rng.standard_normal((64, 128)) * 0.05).astype(np.float16)
    c = torch.zeros((70, 64), dtype=torch.float16, device="cuda")
    k.kvpr_recompute_gemm(dev(A), dev(W), None, c, 70, 64, 128, 64)
    torch.cuda.synchronize()
    assert rel_err(c.cpu().numpy(), ko.project(A, W.T)) <= TIGHT
    k.kvpr_recompute_gemm(None, None, None, None, 0, 64, 128, 64)      # M == 0: no-op, pointers unused
    with pytest.raises(k.KvprError):
        k.kvpr_recompute_gemm(dev(A), dev(W), None, c, 70, 64, 100, 64)  # K not a multiple of 64


# ---- decode attention (Eq. 2) ------------------------------------------------
@pytest.mark.parametrize("S,b,h,H", [(1, 1, 768, 12), (2, 3, 256, 2), (63, 2, 768, 12), (129, 1, 768, 12),
                                     (130, 3, 1024, 8), (1025, 2, 512, 4), (517, 1, 640, 10), (40, 5, 128, 1)])
@pytest.mark.parametrize("force_splits", [0, 1, 3])
def test_decode_attention_matches_oracle(k, S, b, h, H, force_splits):
    print(f"attention S={S} b={b} h={h} H={H} splits={force_splits}", flush=True)
    rng = np.random.default_rng(S * 13 + h)
    q = (rng.standard_normal((b, h)) * 1.5).astype(np.float32)
    kv = rng.standard_normal((S, b, 2 * h)).astype(np.float16)
    z = torch.full((b, h), float("nan"), dtype=torch.float16, device="cuda")
    ws = torch.empty(k.kvpr_attention_workspace_bytes(b, h, H, S), dtype=torch.uint8, device="cuda")
    k.lib.kvpr_debug_set_attention_splits(force_splits, 0)
    try:
        k.kvpr_decode_attention(dev(q, torch.float32), dev(kv), z, ws, S, b, h, H)
        torch.cuda.synchronize()
    finally:
        k.lib.kvpr_debug_set_attention_splits(0, 0)
    ref = ko.decode_attention(q, kv, H)
    got = z.cpu().numpy()
    assert rel_err(got, ref) <= TIGHT
    assert rel_err_rms(got, ref) <= TOL


def test_decode_attention_peaked_softmax(k):
    """Large scores: the running-max recurrence must not overflow."""
    S, b, h, H = 300, 2, 256, 2
    rng = np.random.default_rng(5)
    q = (rng.standard_normal((b, h)) * 30).astype(np.float32)
    kv = rng.standard_normal((S, b, 2 * h)).astype(np.float16)
    z = torch.empty((b, h), dtype=torch.float16, device="cuda")
    ws = torch.empty(k.kvpr_attention_workspace_bytes(b, h, H, S), dtype=torch.uint8, device="cuda")
    k.kvpr_decode_attention(dev(q, torch.float32), dev(kv), z, ws, S, b, h, H)
    torch.cuda.synchronize()
    assert rel_err(z.cpu().numpy(), ko.decode_attention(q, kv, H)) <= TIGHT


# ---- token GEMM (Eq. 1 / 3 / 5 for the decode token) ---------------------------
# cfg: -1 = the library's own choice of kernel; 0x100 + 64 / 128 = the wide kernel with that many features per workgroup
@pytest.mark.parametrize("cfg", [-1, 0x100 + 64, 0x100 + 128])
@pytest.mark.parametrize("M,N,K,f32", [(1, 2304, 768, 768), (32, 768, 768, 0), (3, 96, 128, 32), (16, 520, 256, 8),
                                       (33, 256, 384, 0), (64, 1056, 256, 256), (48, 1300, 1152, 0)])
def test_token_gemm_matches_oracle(k, M, N, K, f32, cfg):
    print(f"token gemm M={M} N={N} K={K} f32={f32} cfg={cfg:#x}", flush=True)
    rng = np.random.default_rng(M + N)
    x = rng.standard_normal((M, K)).astype(np.float16)
    W = (rng.standard_normal((N, K)) * 0.05).astype(np.float16)
    bias = (rng.standard_normal(N) * 0.1).astype(np.float16)
    ld16 = (N - f32) + 16
    y32 = torch.full((M, max(f32, 1)), float("nan"), dtype=torch.float32, device="cuda")
    y16 = torch.full((M, ld16), float("nan"), dtype=torch.float16, device="cuda")
    k.lib.kvpr_debug_set_token_gemm_cfg(cfg)
    try:
        k.kvpr_token_gemm(dev(x), dev(W), dev(bias), y32, y16, M, N, K, f32, ld16)
        torch.cuda.synchronize()
    finally:
        k.lib.kvpr_debug_set_token_gemm_cfg(-1)
    ref = ko.project(x, W.T, bias)
    if f32:
        assert rel_err(y32.cpu().numpy()[:, :f32], ref[:, :f32]) <= 1e-5
    got16 = y16.cpu().numpy()
    assert np.isnan(got16[:, N - f32:]).all()
    assert rel_err(got16[:, :N - f32], ref[:, f32:]) <= TIGHT


# The workspace form: K cut into slices over several workgroups, partial tiles added by the last one to arrive.
# cfg: -1 = automatic (narrow outputs split, wide ones do not); else 0x100 + features per workgroup + (slices << 12).
@pytest.mark.parametrize("cfg", [-1, 0x100 + 64 + (2 << 12), 0x100 + 64 + (3 << 12), 0x100 + 64 + (8 << 12), 0x100 + 128 + (4 << 12)])
@pytest.mark.parametrize("M,N,K,f32", [(1, 2304, 768, 768), (32, 768, 2048, 0), (3, 96, 128, 32), (16, 520, 1024, 8),
                                       (33, 256, 4096, 0), (64, 1056, 1280, 256), (48, 1300, 1152, 0)])
def test_token_gemm_with_workspace_matches_oracle(k, M, N, K, f32, cfg):
    print(f"token gemm ws M={M} N={N} K={K} f32={f32} cfg={cfg:#x}", flush=True)
    rng = np.random.default_rng(M + N + 1)
    x = rng.standard_normal((M, K)).astype(np.float16)
    W = (rng.standard_normal((N, K)) * 0.05).astype(np.float16)
    bias = (rng.standard_normal(N) * 0.1).astype(np.float16)
    ld16 = (N - f32) + 16
    ws_bytes = k.kvpr_token_gemm_workspace_bytes(M, N)
    assert ws_bytes > 4096
    ws = torch.full((ws_bytes,), 0xFF, dtype=torch.uint8, device="cuda")   # partial area poisoned (NaN pattern)
    ws[:4096] = 0
    ref = ko.project(x, W.T, bias)
    xd, Wd, bd = dev(x), dev(W), dev(bias)
    k.lib.kvpr_debug_set_token_gemm_cfg(cfg)
    try:
        for call in range(2):                                    # the second call finds the counters as the first left them
            y32 = torch.full((M, max(f32, 1)), float("nan"), dtype=torch.float32, device="cuda")
            y16 = torch.full((M, ld16), float("nan"), dtype=torch.float16, device="cuda")
            k.kvpr_token_gemm_ws(xd, Wd, bd, y32, y16, M, N, K, f32, ld16, ws, ws_bytes)
            torch.cuda.synchronize()
            assert int(ws[:4096].to(torch.int32).sum()) == 0
            if f32:
                assert rel_err(y32.cpu().numpy()[:, :f32], ref[:, :f32]) <= 1e-5
            got16 = y16.cpu().numpy()
            assert np.isnan(got16[:, N - f32:]).all()
            assert rel_err(got16[:, :N - f32], ref[:, f32:]) <= TIGHT
    finally:
        k.lib.kvpr_debug_set_token_gemm_cfg(-1)


def test_token_gemm_workspace_reused_by_different_products(k):
    """Launches that share a workspace one after the other, as the layer's output projection and second FFN matrix do:
    every launch must read the partial tiles of its own slices, not what an earlier launch left at the same addresses."""
    M = 32
    shapes = [(1024, 4096), (768, 8192), (1024, 4096), (1024, 2048), (520, 4096)]
    ws_bytes = k.kvpr_token_gemm_workspace_bytes(M, 1024)
    ws = torch.zeros(ws_bytes, dtype=torch.uint8, device="cuda")
    rng = np.random.default_rng(77)
    cases = []
    for N, K in shapes:
        x = rng.standard_normal((M, K)).astype(np.float16)
        W = (rng.standard_normal((N, K)) * 0.05).astype(np.float16)
        cases.append((N, K, x, W, dev(x), dev(W), torch.full((M, N), float("nan"), dtype=torch.float16, device="cuda")))
    for rounds in range(3):                                      # enqueued back to back, checked afterwards
        for N, K, x, W, xd, Wd, y in cases:
            y.fill_(float("nan"))
            k.kvpr_token_gemm_ws(xd, Wd, None, None, y, M, N, K, 0, N, ws, ws_bytes)
        torch.cuda.synchronize()
        for N, K, x, W, xd, Wd, y in cases:
            assert rel_err(y.cpu().numpy(), ko.project(x, W.T, np.zeros(N, np.float16))) <= TIGHT, (rounds, N, K)
    assert int(ws[:4096].to(torch.int32).sum()) == 0


def test_token_gemm_workspace_too_small_falls_back(k):
    M, N, K = 32, 512, 2048
    rng = np.random.default_rng(5)
    x = rng.standard_normal((M, K)).astype(np.float16)
    W = (rng.standard_normal((N, K)) * 0.05).astype(np.float16)
    ref = ko.project(x, W.T, np.zeros(N, np.float16))
    for ws_bytes in (0, 4096, 4096 + 2 * N * 32 * 4):            # none, counters only, room for two slices
        ws = torch.zeros(max(ws_bytes, 16), dtype=torch.uint8, device="cuda")
        y16 = torch.full((M, N), float("nan"), dtype=torch.float16, device="cuda")
        k.kvpr_token_gemm_ws(dev(x), dev(W), None, None, y16, M, N, K, 0, N, ws, ws_bytes)
        torch.cuda.synchronize()
        assert rel_err(y16.cpu().numpy(), ref) <= TIGHT
