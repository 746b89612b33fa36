"""CPU oracle for KVPR's split-point scheduler.  TEST INFRASTRUCTURE ONLY.

Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may import
this file.  It shares no code with the HIP library and never imports it.

The scheduler (Sec. 3.2, "Determining the optimal KV cache split point") has a
single integer unknown l, so the oracle is brute force: evaluate the cost for
every admissible l and keep the smallest.

  Eq. 6   M_X[0:l]   = b * l * h * p           bytes of activations sent first
          M_KV[l:s'] = 2 * b * (s' - l) * h * p bytes of cache sent afterwards
  Eq. 8   N_KV[0:l]  = 4 * b * l * h^2          flops of the recomputation
  Eq. 9   t_recomp   = N_KV / v_gpu
  Eq. 10  t = M_X / v_com + max(t_recomp, M_KV / v_com)
  Eq. 11  minimise t over 0 <= l <= s'

Three cost forms are provided:
  COST_EQ10  Eq. 10 as printed: the activations and the cache share one link,
             the activations go first (column-by-column schedule).
  COST_ROW   Eq. 10 with its first term dropped: the paper's row-by-row case
             (last sentence of the split-point paragraph).
  COST_NS    max(t_recomp + M_X/v_com, M_KV/v_com): the activation copy is
             charged only to the compute arm, as if it travelled on a second
             link.  Not in the paper; kept because the benchmark spec
             paraphrases the cost this way.
  COST_PIPE  max((M_X + M_KV)/v_com, t_recomp + t_other): steady state when the next
             layer's transfers overlap this layer's compute (double buffering across
             layers, Sec. 4 "Implementation"); t_other (default 0) is the rest of a
             layer's compute, which shares the GPU with the recomputation.  An
             extension: the paper does not model it.

Readings where the paper is silent: the integer problem is solved exactly by
enumeration, scanning l upward and keeping the first strict minimum (ties go to
the smallest l, i.e. the least GPU work); byte and flop counts are formed as
integers and converted to float64 once; every division is one IEEE-754 double
division.  Optional affine terms (a fixed latency per non-empty copy / GEMM)
extend the paper's purely linear model; they default to 0.
"""
from __future__ import annotations

COST_EQ10 = 0
COST_NS = 1
COST_ROW = 2
COST_PIPE = 3


def bytes_x(b: int, l: int, h: int, p: int) -> int:
    """Eq. 6, first line."""
    return b * l * h * p


def bytes_kv(b: int, l: int, s: int, h: int, p: int) -> int:
    """Eq. 6, second line."""
    return 2 * b * (s - l) * h * p


def flops_recompute(b: int, l: int, h: int) -> int:
    """Eq. 8."""
    return 4 * b * l * h * h


def cost(model: int, l: int, b: int, s: int, h: int, p: int,
         v_com: float, v_gpu: float, lat_com: float = 0.0, lat_gpu: float = 0.0, other: float = 0.0) -> float:
    """Predicted time of one layer's KV assembly at split l (seconds)."""
    t_act = float(bytes_x(b, l, h, p)) / v_com
    t_kv = float(bytes_kv(b, l, s, h, p)) / v_com
    t_rc = float(flops_recompute(b, l, h)) / v_gpu          # Eq. 9
    if l > 0:
        t_act = t_act + lat_com
        t_rc = t_rc + lat_gpu
    if l < s:
        t_kv = t_kv + lat_com
    if model == COST_EQ10:
        return t_act + max(t_rc, t_kv)                      # Eq. 10
    if model == COST_ROW:
        return max(t_rc, t_kv)
    if model == COST_NS:
        return max(t_rc + t_act, t_kv)
    if model == COST_PIPE:
        return max(t_act + t_kv, t_rc + other)
    raise ValueError(f"unknown cost model {model}")


def candidates(s: int, granularity: int = 1):
    """Admissible splits: multiples of `granularity` up to s, and s itself."""
    if granularity < 1:
        raise ValueError("granularity must be >= 1")
    ls = list(range(0, s + 1, granularity))
    if ls[-1] != s:
        ls.append(s)
    return ls


def plan_split(model: int, b: int, s: int, h: int, p: int, v_com: float, v_gpu: float,
               granularity: int = 1, lat_com: float = 0.0, lat_gpu: float = 0.0, other: float = 0.0):
    """Eq. 11 by enumeration.  Returns (l*, t(l*))."""
    best_l, best_t = -1, float("inf")
    for l in candidates(s, granularity):
        t = cost(model, l, b, s, h, p, v_com, v_gpu, lat_com, lat_gpu, other)
        if t < best_t:
            best_l, best_t = l, t
    return best_l, best_t


# --------------------------------------------------------------------------
# Extension (not in the paper): chunked activation copy.  X[0:l] travels as
# `chunks` equal parts; the GEMM of part j starts when part j has landed and
# part j-1 has been recomputed; the cache follows X on the same link.
# chunks = 1 is Eq. 10.
# --------------------------------------------------------------------------
def cost_chunked(chunks: int, l: int, b: int, s: int, h: int, p: int, v_com: float, v_gpu: float,
                 lat_com: float = 0.0, lat_gpu: float = 0.0) -> float:
    t_act = float(bytes_x(b, l, h, p)) / v_com
    t_kv = float(bytes_kv(b, l, s, h, p)) / v_com
    t_rc = float(flops_recompute(b, l, h)) / v_gpu
    if l < s:
        t_kv = t_kv + lat_com
    done = 0.0
    if l > 0:
        for j in range(1, chunks + 1):
            landed = t_act * float(j) / float(chunks) + lat_com
            start = landed if landed > done else done
            done = start + (t_rc / float(chunks) + lat_gpu)
    link = ((t_act + lat_com) if l > 0 else 0.0) + t_kv
    return done if done > link else link


def plan_split_chunked(chunks: int, b: int, s: int, h: int, p: int, v_com: float, v_gpu: float,
                       granularity: int = 1, lat_com: float = 0.0, lat_gpu: float = 0.0):
    best_l, best_t = -1, float("inf")
    for l in candidates(s, granularity):
        t = cost_chunked(chunks, l, b, s, h, p, v_com, v_gpu, lat_com, lat_gpu)
        if t < best_t:
            best_l, best_t = l, t
    return best_l, best_t


# --------------------------------------------------------------------------
# The same cost forms for any per-position sizes: Eq. 6 and Eq. 8 are linear in
# the number of positions, M_X = x_bpp * l, M_KV = kv_bpp * (s' - l),
# N_KV = flops_pp * l.  With x_bpp = b*h*p, kv_bpp = 2*b*h*p, flops_pp = 4*b*h^2
# this is the paper's model; a compressed store (Sec. 4.4) only changes the two
# byte rates.  chunks > 1 selects the chunked-copy extension above (Eq. 10 only).
# --------------------------------------------------------------------------
def cost_linear(model: int, chunks: int, l: int, s: int, x_bpp: int, kv_bpp: int, flops_pp: int,
                v_com: float, v_gpu: float, lat_com: float = 0.0, lat_gpu: float = 0.0, other: float = 0.0,
                round_flops: int = 0) -> float:
    """round_flops > 0 (an extension of Eq. 9): the GPU does the recomputation in indivisible rounds of that
    many flops (one tile per compute unit), so N_KV is charged rounded up to whole rounds."""
    m_x = x_bpp * l
    m_kv = kv_bpp * (s - l)
    n_kv = flops_pp * l
    if round_flops > 0:
        n_kv = -(-n_kv // round_flops) * round_flops
    send_x = float(m_x) / v_com
    send_kv = float(m_kv) / v_com
    gemm = float(n_kv) / v_gpu
    if chunks > 1:
        if model != COST_EQ10:
            raise ValueError("the chunked schedule is modelled for Eq. 10 only")
        if l < s:
            send_kv = send_kv + lat_com
        finished = 0.0
        if l > 0:
            for j in range(1, chunks + 1):
                arrived = send_x * float(j) / float(chunks) + lat_com
                begin = max(arrived, finished)
                finished = begin + (gemm / float(chunks) + lat_gpu)
        link = ((send_x + lat_com) if l > 0 else 0.0) + send_kv
        return max(finished, link)
    if l > 0:
        send_x = send_x + lat_com
        gemm = gemm + lat_gpu
    if l < s:
        send_kv = send_kv + lat_com
    if model == COST_EQ10:
        return send_x + max(gemm, send_kv)
    if model == COST_ROW:
        return max(gemm, send_kv)
    if model == COST_NS:
        return max(gemm + send_x, send_kv)
    if model == COST_PIPE:
        return max(send_x + send_kv, gemm + other)
    raise ValueError(f"unknown cost model {model}")


def plan_split_linear(model: int, chunks: int, s: int, x_bpp: int, kv_bpp: int, flops_pp: int,
                      v_com: float, v_gpu: float, granularity: int = 1,
                      lat_com: float = 0.0, lat_gpu: float = 0.0, other: float = 0.0, round_flops: int = 0):
    best_l, best_t = -1, float("inf")
    for l in candidates(s, granularity):
        t = cost_linear(model, chunks, l, s, x_bpp, kv_bpp, flops_pp, v_com, v_gpu, lat_com, lat_gpu, other, round_flops)
        if t < best_t:
            best_l, best_t = l, t
    return best_l, best_t


# --------------------------------------------------------------------------
# Extension (the paper profiles once, at start-up, and names run-time adaptation as
# future work in its Limitations section): exponential moving average of the two
# constants of Eq. 9 / Eq. 10 over what finished layers actually achieved.
#   v' = (1 - alpha) * v + alpha * (work / seconds)     for each constant whose sample is valid
# A sample is valid when it has work > 0 and seconds > 0.
# --------------------------------------------------------------------------
def adapt_update(v_com: float, v_gpu: float, alpha: float, link_bytes: int, link_s: float,
                 flops: int, gemm_s: float):
    if not 0.0 <= alpha <= 1.0:
        raise ValueError("alpha outside [0, 1]")
    if link_bytes > 0 and link_s > 0.0:
        v_com = (1.0 - alpha) * v_com + alpha * (float(link_bytes) / link_s)
    if flops > 0 and gemm_s > 0.0:
        v_gpu = (1.0 - alpha) * v_gpu + alpha * (float(flops) / gemm_s)
    return v_com, v_gpu
