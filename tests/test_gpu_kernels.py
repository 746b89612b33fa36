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
