"""The packed HiKonv algorithm in exact big-integer arithmetic.  TEST INFRASTRUCTURE ONLY.

This is the second CPU artefact (besides the direct definitions in hikonv_oracle.c): it
takes the paper's steps -- pack (Eq. inpack / Eq. signpackslice), one wide multiply
(Theorem 1, Eq. multiply / Eq. prod), overlap-add of neighbouring blocks (Theorem 2,
Eq. 1dnx), split with carried-sign correction (Eq. output_split), the row mapping of a DNN
layer (Theorem 3, Eq. dnn_hikonv / Eq. off) and accumulation of products before the split
-- in Python integers of unbounded width, so the identities can be checked on the CPU
against the direct definitions.  It shares no code with the HIP library.

Readings: Eq. inpack's slice order (element 0 in the least significant slice); the field of
Eq. output_split is sign-extended before the bit below it is added; Algorithm 2 as printed
is not executable (its packing register is never cleared, its index steps by one, `prev`
is never updated), so the loop below is derived from Theorem 2 and from the register-based
1-D architecture of Section "1-D & DNN layer Convolution Architecture" instead (the stored
word is shifted by N slices and the new product is added to it); a row whose length
is not a multiple of N is zero-extended (Eq. pad_f0); kernels wider than one B word are cut
into chunks and the chunk products are accumulated on correspondingly delayed inputs.

Pins: tests/test_packed_model_pins.py (the worked F_{3,2} example with its printed
multiplicands and product, the multi-channel INT4 identity Eq. xilinx4bit, brute-force
direct convolution, guard-bit sufficiency and a constructed failure with one bit fewer).
"""


def pack(values, s: int) -> int:
    """Eq. (inpack): sum of v[i] * 2**(S*i) as an ordinary (possibly negative) integer."""
    return sum(int(v) << (s * i) for i, v in enumerate(values))


def pack_slices_signed(values, s: int) -> int:
    """Eq. (signpackslice): build the two's-complement bit pattern slice by slice.

    Slice 0 holds f[0]; slice n>0 holds f[n] minus the top bit of the pattern below it.
    Returns the pattern as a non-negative integer of len(values)*S bits.
    """
    pattern = 0
    for n, v in enumerate(values):
        field = int(v)
        if n > 0:
            field -= (pattern >> (s * n - 1)) & 1
        pattern |= (field & ((1 << s) - 1)) << (s * n)
    return pattern


def sext(v: int, bits: int) -> int:
    v &= (1 << bits) - 1
    return v - (1 << bits) if v >> (bits - 1) else v


def split_unsigned(prod: int, s: int, count: int):
    return [(prod >> (s * m)) & ((1 << s) - 1) for m in range(count)]


def split_signed(prod: int, s: int, count: int):
    """Eq. (output_split): y[0] = low field; y[m] = field m + the bit just below it."""
    out = []
    for m in range(count):
        field = sext(prod >> (s * m), s)
        carry = (prod >> (s * m - 1)) & 1 if m > 0 else 0
        out.append(field + carry)
    return out


def split_signed_bias(prod: int, s: int, count: int):
    """Same values via a bias: add 2**(S-1) to every field, read unsigned, subtract."""
    bias = sum(1 << (s * m + s - 1) for m in range(count))
    return [u - (1 << (s - 1)) for u in split_unsigned(prod + bias, s, count)]


def fnk(f, g, s: int, signed: bool):
    """Theorem 1: one multiply of the packed operands gives the N+K-1 partial convolutions."""
    prod = pack(f, s) * pack(g, s)
    count = len(f) + len(g) - 1
    return (split_signed if signed else split_unsigned)(prod, s, count), prod


def _hi(prod: int, shift: int, signed: bool) -> int:
    """Segments N.. of a block product, as an integer aligned to segment 0 of the next block."""
    if not signed:
        return prod >> shift
    return (prod >> shift) + ((prod >> (shift - 1)) & 1)      # floor shift + carried sign


def conv1d_packed(f, g, n: int, k: int, s: int, signed: bool):
    """Full 1-D convolution (len(f)+len(g)-1 outputs) by blocks of N inputs (Theorem 2).

    g is cut into chunks of k taps; chunk c multiplies the input delayed by c*k positions.
    """
    f = [int(v) for v in f]
    g = [int(v) for v in g]
    taps = len(g)
    out_len = len(f) + taps - 1
    chunks = [g[c:c + k] for c in range(0, taps, k)]
    b_words = [pack(ch, s) for ch in chunks]
    n_blocks = -(-out_len // n)
    split = split_signed if signed else split_unsigned

    def elem(i):
        return f[i] if 0 <= i < len(f) else 0

    y = []
    prev = 0
    for x in range(n_blocks):
        prod = 0
        for c, b in enumerate(b_words):
            a = pack([elem(x * n + j - c * k) for j in range(n)], s)
            prod += a * b
        comb = prod + _hi(prev, s * n, signed)
        y.extend(split(comb, s, n))
        prev = comb          # the stored word keeps every pending segment (also when K-1 > N)
    return y[:out_len]


def conv2d_packed(x, w, pad: int, n: int, k: int, s: int, m_acc: int, signed: bool):
    """Stride-1 DNN layer through row convolutions (Theorem 3) with accumulation of up to
    m_acc block products (over input channels and kernel rows) before each split.

    x: [C][H][W] nested lists / array, w: [Co][C][Kh][Kw]; returns [Co][Ho][Wo] lists.
    The kernel row is reversed (g = W[co][ci][kh][K-1:0]) and output w is read at
    position w+Kw-1 of the row convolution of the zero-padded row.
    """
    c_in, h_in, w_in = len(x), len(x[0]), len(x[0][0])
    c_out, kh_n, kw_n = len(w), len(w[0][0]), len(w[0][0][0])
    ho, wo = h_in + 2 * pad - kh_n + 1, w_in + 2 * pad - kw_n + 1
    w_pad = w_in + 2 * pad
    out_len = w_pad + kw_n - 1
    n_blocks = -(-out_len // n)
    split = split_signed if signed else split_unsigned

    def row(ci, r):
        if r < 0 or r >= h_in:
            return [0] * w_pad
        return [0] * pad + [int(v) for v in x[ci][r]] + [0] * pad

    out = [[[0] * wo for _ in range(ho)] for _ in range(c_out)]
    for co in range(c_out):
        for h in range(ho):
            terms = [(ci, kh) for ci in range(c_in) for kh in range(kh_n)]
            for t0 in range(0, len(terms), m_acc):
                group = terms[t0:t0 + m_acc]
                acc = [0] * n_blocks
                for ci, kh in group:
                    f = row(ci, h + kh - pad)
                    g = [int(v) for v in w[co][ci][kh]][::-1]
                    for c0 in range(0, kw_n, k):
                        b = pack(g[c0:c0 + k], s)
                        for xb in range(n_blocks):
                            a = pack([f[i] if 0 <= i < w_pad else 0
                                      for i in range(xb * n - c0, xb * n - c0 + n)], s)
                            acc[xb] += a * b
                y = []
                prev = 0
                for xb in range(n_blocks):
                    comb = acc[xb] + _hi(prev, s * n, signed)
                    y.extend(split(comb, s, n))
                    prev = comb
                for wcol in range(wo):
                    out[co][h][wcol] += y[wcol + kw_n - 1]
    return out
