"""The paper's performance model, written out step by step.  TEST INFRASTRUCTURE ONLY.

Follows Section "Multiplier for Convolution": the slice-size rule Eq. (slice1), the fit
constraints Eq. (slice2)/(slice3), the three guard-bit cases collected in "Maximizing
Processing Throughput", the operation count Eq. (tot_ops) and the exhaustive search of
Algorithm 1.  Shares no code with the HIP library's planner.

Readings taken where the paper is silent or inconsistent (each is listed in the design notes):

* Eq. (slice1)'s 1-bit special cases are used, although Algorithm 1 and the optimisation
  statement print S = p+q+G_b only: the paper's own 27x18 binary figure (N=9, K=4, 60 ops)
  is reachable only with them.
* Algorithm 1's printed loop bounds exclude the optimum it reports (8-bit on 32x32 needs
  N=2 but Max_N=2 with a strict `<`), so every n in [1, L_A] and k in [1, L_B] is tried;
  order and the strict `>` are the algorithm's: k outer ascending, n inner ascending.
* With a fixed number of kernel taps that does not fit one B word, the taps are cut into
  chunks of K (linearity of convolution); the objective is then multiply-accumulates per
  multiply, N*taps/ceil(taps/K), tried from the largest K and N downwards.

Pins: tests/test_plan_pins.py (values printed in the abstract, in "Maximizing Processing
Throughput" and in the 4-bit evaluation paragraph; brute-force count of Eq. (tot_ops)).
"""
from math import ceil

SINGLE, CONV1D, DNN = 0, 1, 2


def ceil_log2(x: int) -> int:
    """Smallest e with 2**e >= x (0 for x <= 1)."""
    return 0 if x <= 1 else (x - 1).bit_length()


def slice_bits(p: int, q: int, gb: int) -> int:
    """Eq. (slice1): a 1-bit operand does not widen the product."""
    if p == 1:
        return q + gb
    if q == 1:
        return p + gb
    return p + q + gb


def guard_bits(mode: int, n: int, k: int, m: int = 1, taps: int = 0) -> int:
    """Guard bits for the three uses of the multiplier.

    single multiplier: ceil(log2 min(K, N));  1-D convolution: ceil(log2 K);
    DNN convolution with M accumulated products: the paper prints ceil(log2(M*min(K,N))),
    which holds when segments are split before the overlap-add.  This build overlap-adds
    in the packed domain, where a segment can collect M*taps products, so that count is
    used for DNN mode.  `taps` (if non-zero) replaces K in the 1-D and DNN cases: all taps
    of a chunked kernel meet in one segment.
    """
    kk = taps if taps else k
    if mode == SINGLE:
        return ceil_log2(min(k, n))
    if mode == CONV1D:
        return ceil_log2(kk)
    if mode == DNN:
        return ceil_log2(m * kk)
    raise ValueError(mode)


def ops_per_multiply(n: int, k: int) -> int:
    """Eq. (tot_ops): N*K multiplications plus N*K-(N+K-1) additions."""
    return n * k + (n - 1) * (k - 1)


def fits(p, q, n, k, s, l_a, l_b) -> bool:
    """Eq. (slice2) and Eq. (slice3)."""
    return p + (n - 1) * s <= l_a and q + (k - 1) * s <= l_b


def paper_search(p, q, l_a, l_b, mode=SINGLE, m=1):
    """Algorithm 1 (free N and K): returns dict(N, K, S, G_b, ops) or None."""
    best = None
    for k in range(1, l_b + 1):
        for n in range(1, l_a + 1):
            gb = guard_bits(mode, n, k, m)
            s = slice_bits(p, q, gb)
            if not fits(p, q, n, k, s, l_a, l_b):
                continue
            cur = ops_per_multiply(n, k)
            if best is None or cur > best["ops"]:
                best = dict(N=n, K=k, S=s, G_b=gb, ops=cur)
    return best


def paper_search_taps(p, q, l_a, l_b, taps, mode=CONV1D, m=1):
    """Fixed kernel width `taps`, chunked if needed: maximise MACs per multiply."""
    best = None
    gb = guard_bits(mode, 1, 1, m, taps)
    s = slice_bits(p, q, gb)
    for k in range(taps, 0, -1):
        chunks = ceil(taps / k)
        for n in range(l_a, 0, -1):
            if not fits(p, q, n, k, s, l_a, l_b):
                continue
            score = (n * taps) / chunks
            if best is None or score > best["score"]:
                best = dict(N=n, K=k, S=s, G_b=gb, chunks=chunks, score=score,
                            ops=ops_per_multiply(n, k))
    return best
