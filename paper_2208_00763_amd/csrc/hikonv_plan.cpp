// Host-side planner: the paper's performance model (Section "Multiplier for
// Convolution", Eq. slice1-slice3, the guard-bit cases of "Maximizing Processing
// Throughput", Eq. tot_ops and Algorithm 1), plus the exactness checks the model leaves
// out for signed data and for accumulation in a register of finite width.
//
// Differences from the printed algorithm (all deliberate):
//  * Eq. slice1's 1-bit cases are honoured (Algorithm 1 prints p+q+G_b only);
//  * every n in [1,L_A], k in [1,L_B] is tried (the printed loop bounds cut off the optimum);
//    order is the algorithm's: k outer, n inner, strict improvement;
//  * a candidate is kept only if every segment sum, both packed operands and the
//    accumulated product provably fit (exact interval arithmetic); when the slice of
//    Eq. slice1 is one bit short for signed data, S+1 is tried;
//  * with a fixed tap count the kernel may be cut into chunks of K taps;
//  * outside single-multiplier mode K <= N+1 is required (one-neighbour overlap-add);
//  * on request ("tight") the slice is the smallest one the exact check accepts, not
//    p+q+G_b: e.g. 3 signed 4-bit products sum to at most 192 in magnitude, which fits 9 bits.
#include <initializer_list>

#include "hikonv_internal.h"

namespace {

typedef __int128 i128;

inline int ceil_log2(long long x)
{
    int e = 0;
    while ((1LL << e) < x) ++e;
    return e;
}

inline int slice_bits(int p, int q, int gb)
{
    if (p == 1) return q + gb;
    if (q == 1) return p + gb;
    return p + q + gb;
}

struct Range {
    i128 lo, hi;
};

inline Range value_range(int bits, bool is_signed)
{
    if (is_signed) return Range{-((i128)1 << (bits - 1)), ((i128)1 << (bits - 1)) - 1};
    return Range{0, ((i128)1 << bits) - 1};
}

inline Range mul_range(Range a, Range b)
{
    i128 c[4] = {a.lo * b.lo, a.lo * b.hi, a.hi * b.lo, a.hi * b.hi};
    Range r{c[0], c[0]};
    for (int i = 1; i < 4; ++i) {
        if (c[i] < r.lo) r.lo = c[i];
        if (c[i] > r.hi) r.hi = c[i];
    }
    return r;
}

inline bool fits_width(Range r, int width, bool is_signed)
{
    if (width >= 127) return true;
    if (is_signed) return r.lo >= -((i128)1 << (width - 1)) && r.hi <= ((i128)1 << (width - 1)) - 1;
    return r.lo >= 0 && r.hi <= ((i128)1 << width) - 1;
}

struct Req {
    int p, q;
    bool a_signed, w_signed, any_signed, bipolar;
    int L_A, L_B, L_acc, mode, M, taps;
    bool tight;
    int objective, out_bits, max_N;
    Range fa, gw, prod;
};

Req make_req(const hikonv_plan_t &in)
{
    Req r;
    r.p = in.bits_a;
    r.q = in.bits_w;
    r.a_signed = in.a_signed != 0;
    r.w_signed = in.w_signed != 0;
    r.bipolar = in.bipolar != 0;
    if (r.bipolar) {
        // {-1,+1} values (0 in the zero padding) travel as signed two-bit slices
        r.p = r.q = 2;
        r.a_signed = r.w_signed = true;
    }
    r.any_signed = r.a_signed || r.w_signed;
    r.L_A = in.L_A;
    r.L_B = in.L_B;
    r.L_acc = in.L_acc > 0 ? in.L_acc : in.L_A + in.L_B;
    r.mode = in.mode;
    r.M = in.mode == HIKONV_MODE_DNN ? (in.M > 0 ? in.M : 1) : 1;
    r.taps = in.taps;
    r.objective = in.objective;
    // the cost objective of a layer plan searches the exact-interval slices as well: a narrower slice
    // lets more products accumulate before a split, which is what a layer pays for on this chip
    r.tight = in.tight != 0 ||
              (in.objective == HIKONV_OBJ_MEASURED_COST && in.mode == HIKONV_MODE_DNN && in.taps > 0);
    r.out_bits = in.out_bits;
    r.max_N = in.max_N;
    r.fa = r.bipolar ? Range{-1, 1} : value_range(r.p, r.a_signed);
    r.gw = r.bipolar ? Range{-1, 1} : value_range(r.q, r.w_signed);
    r.prod = mul_range(r.fa, r.gw);
    return r;
}

// Largest number of low-bit products that can meet in one output segment.
inline long long terms_per_segment(const Req &r, int n, int k)
{
    int kk = r.taps ? r.taps : k;
    switch (r.mode) {
    case HIKONV_MODE_SINGLE: return n < k ? n : k;
    case HIKONV_MODE_CONV1D: return kk;
    default: return (long long)r.M * kk;
    }
}

inline int guard_bits(const Req &r, int n, int k) { return ceil_log2(terms_per_segment(r, n, k)); }

// Eq. slice2 / slice3 as printed (bit counting only).
inline bool paper_fits(const Req &r, int n, int k, int s)
{
    return r.p + (long long)(n - 1) * s <= r.L_A && r.q + (long long)(k - 1) * s <= r.L_B;
}

// Exact check of (n, k, s): segment fields, operand words, accumulator.
bool exact_ok(const Req &r, int n, int k, int s)
{
    if (s < 1 || s > 62) return false;
    // operands are at most 64 bits wide: longer packings cannot fit (and would overflow the checks below)
    if ((long long)s * (n - 1) >= 64 || (long long)s * (k - 1) >= 64) return false;
    // the kernels overlap-add a block with its immediate neighbour only: the K-1 high
    // segments of a product must land inside the next block's N low segments
    if (r.mode != HIKONV_MODE_SINGLE && k - 1 > n) return false;
    const long long t = terms_per_segment(r, n, k);
    const Range seg{r.prod.lo * t, r.prod.hi * t};
    if (r.any_signed) {
        // symmetric bound: the carried-sign split needs value-1 to fit as well
        const i128 lim = ((i128)1 << (s - 1)) - 1;
        if (seg.lo < -lim || seg.hi > lim) return false;
    } else {
        if (seg.hi > ((i128)1 << s) - 1) return false;
    }
    i128 rn = 0, rk = 0;
    for (int i = 0; i < n; ++i) rn += (i128)1 << (s * i);
    for (int i = 0; i < k; ++i) rk += (i128)1 << (s * i);
    if (!fits_width(Range{r.fa.lo * rn, r.fa.hi * rn}, r.L_A, r.any_signed)) return false;
    if (!fits_width(Range{r.gw.lo * rk, r.gw.hi * rk}, r.L_B, r.any_signed)) return false;
    // a register of 127+ bits always holds one product of two <= 64-bit operands
    if (r.L_acc >= 127) return r.M == 1 && r.mode == HIKONV_MODE_SINGLE;
    if ((long long)s * (n + k - 1) > 120) return false;
    // accumulated word: per multiply, segment m holds c_m = #{(i,j): i+j=m} products; every
    // multiply that lands in the word before a split adds to it
    const int chunks = r.taps ? (r.taps + k - 1) / k : 1;
    const long long mults = (long long)r.M * chunks;
    Range acc{0, 0};
    for (int m = 0; m < n + k - 1; ++m) {
        int lo_i = m - (k - 1) > 0 ? m - (k - 1) : 0;
        int hi_i = m < n - 1 ? m : n - 1;
        long long c = (long long)(hi_i - lo_i + 1) * mults;
        // after the overlap-add the N low fields hold complete outputs
        if (r.mode != HIKONV_MODE_SINGLE && m < n && c < t) c = t;
        acc.lo += r.prod.lo * c * ((i128)1 << (s * m));
        acc.hi += r.prod.hi * c * ((i128)1 << (s * m));
    }
    if (r.any_signed && r.mode != HIKONV_MODE_SINGLE) {
        // the kernels add 2^(S-1) to each of the N low fields before reading them
        for (int m = 0; m < n; ++m) acc.hi += (i128)1 << (s * m + s - 1);
    }
    return fits_width(acc, r.L_acc, r.any_signed);
}

struct Cand {
    int n = 0, k = 0, s = 0, gb = 0, chunks = 1;
    int stride = 1;    // elements between the values of neighbouring slices (1: Eq. inpack)
    double cost = 0.0; // modelled VALU issue slots per output (measured-cost objective)
    bool found = false;
};

// ---- issue-cost model of the 1-D kernels (HIKONV_OBJ_MEASURED_COST) -----------------------
//
// Algorithm 1 prices every candidate by the low-bit operations one multiply replaces, as if
// the multiply were all a convolution costs.  On a gfx950 lane the multiply is one issue slot
// among many: building A from bit-dense containers, exchanging the high part with the
// neighbour lane, cutting the word into fields and storing them cost a slot per instruction
// too.  The model below counts VALU issue slots per output element for each kernel form.  The
// coefficients are fitted to SQ_INSTS_VALU (wave instructions x 64 / outputs) of the kernels
// on MI355X at 4096 rows x 65536, 3, 5 and 7 taps (every integer instruction the kernels use
// issues at 87-99 % of the full rate, so an instruction is priced as one slot).
//
//   window kernel, int32 outputs (taps <= 7, K = min(taps, N), N in {2,3,4,5,6,8,11}); a lane
//   makes G = 8 outputs from one window with containers of up to 4 bits, G = 4 with 8-bit ones;
//   per output: base + tap*taps + block*ceil((taps+G-1)/N)  [+ signed], kWin8* / kWin4*
//       (most of it index arithmetic, bounds tests and stores per group, not packed arithmetic)
//   lane-per-block kernel, int32 outputs (the other stride_elems = 1 plans), per block of N outputs:
//       kI32Block + kI32Elem*N  [+ N + 1 signed]  + per extra B word: kShareChunk when the
//       delayed words come from the preceding lanes (K = N), else a second packing
//   streaming kernel, requantised bit-dense outputs:
//       kRqBlock + kRqElem*N  [+ N + 1 signed] + the same per extra B word
//   one value and one tap per multiply (N = K = 1), requantised outputs: the one-product kernel,
//       13.7 .. 21 per output at 3 taps by output container, 1.9 per further tap
//   container-aligned slices (K = 1, S = SW, J = SW/c residues), per output dword of 32/c values:
//       2 per packed word of the window (shift, mask), J + taps - 1 of them
//       taps per residue word (multiply-add; AND + add for one-bit taps), J residue words
//       kAlignedRequant (2 unsigned, 4 signed, 3 nibble) per residue word for ReLU/shift/clamp
//       1.5 per residue word to place it in the output dword, kAlignedDword per dword for
//       window assembly, addresses and the store
//
// A kernel cannot run faster than its bytes move: the price of a plan is bounded below by the
// slots that pass during the HBM time of its algorithmic bytes per output at the published
// peaks (8 TB/s, 256 CUs x 64 lanes x 2.4 GHz: 4.9 slots per byte).  Plans under that floor tie
// and Algorithm 1's own order decides among them.
constexpr double kI32Block = 15.0, kI32Elem = 11.7;
constexpr double kRqBlock = 21.0, kRqElem = 13.9;
constexpr double kShareChunk = 4.2;
constexpr double kWin8Base = 6.1, kWin8Tap = 0.39, kWin8Block = 0.46, kWin8Signed = 1.3;
constexpr double kWin4Base = 4.7, kWin4Tap = 0.56, kWin4Block = 1.36, kWin4Signed = 1.4;

// plans the window kernel (int32 outputs) takes (the launcher's rule, without the geometry)
inline bool window_form(int taps, int n, int k)
{
    if (taps < 1 || taps > 7 || k != (taps < n ? taps : n)) return false;
    return n == 2 || n == 3 || n == 4 || n == 5 || n == 6 || n == 8 || n == 11;
}
constexpr double kAlignedDword = 25.0;
constexpr double kSlotsPerByte = 256.0 * 64.0 * 2.4e9 / 8.0e12;

inline int container_of(int bits) { return hikonv::container_bits(bits); }

double hbm_floor_slots(const Req &r)
{
    const double in_bytes = container_of(r.p) / 8.0;
    const double out_bytes = r.out_bits > 0 ? container_of(r.out_bits) / 8.0 : 4.0;
    return (in_bytes + out_bytes) * kSlotsPerByte;
}

// slots per output of the kernel that runs (n, k, s, stride) in CONV1D mode; < 0: no kernel
double conv1d_slots(const Req &r, int n, int k, int chunks, int s, int stride)
{
    // One value and one tap per multiply (the degenerate F_{1,1}) with requantised output: the entry
    // point runs the one-product-per-multiply kernel for it.  Measured slots per output at 3 taps by
    // output container (1, 2, 4, 8 bits: 19.4, 14.8, 13.7, 21), about 1.9 more per further tap.
    if (stride <= 1 && r.out_bits > 0 && n == 1 && k == 1) {
        const int co = container_of(r.out_bits);
        const double base = co == 1 ? 19.4 : co == 2 ? 14.8 : co == 4 ? 13.7 : 21.0;
        const double slots = base + 1.9 * (r.taps - 3);
        return slots < 8.0 ? 8.0 : slots;
    }
    if (stride > 1) {
        const int c = container_of(r.p);
        const int j = stride, per = 32 / c;
        const bool nibble = s == 4;
        const double words = j + r.taps - 1;
        const double requant = nibble ? 3.0 : (r.any_signed ? 4.0 : 2.0);
        const double mac = nibble ? 2.0 : 1.0;
        return (2.0 * words + j * (mac * r.taps + requant + 1.5) + kAlignedDword) / per;
    }
    if (r.out_bits == 0 && window_form(r.taps, n, k) && n * container_of(r.p) <= 32) {
        if (container_of(r.p) <= 4)
            return kWin8Base + kWin8Tap * r.taps + kWin8Block * ((r.taps + 7 + n - 1) / n) + (r.any_signed ? kWin8Signed : 0.0);
        return kWin4Base + kWin4Tap * r.taps + kWin4Block * ((r.taps + 3 + n - 1) / n) + (r.any_signed ? kWin4Signed : 0.0);
    }
    const bool share = chunks >= 2 && chunks <= 4 && k == n && n >= 2 && n <= 5;
    double block = r.out_bits > 0 ? kRqBlock + kRqElem * n : kI32Block + kI32Elem * n;
    if (r.any_signed) block += n + 1;
    if (chunks > 1) block += (chunks - 1) * (share ? kShareChunk : 2.0 * n + 3.0);
    // with 8-bit containers the streaming requantising kernel measures about 1.5 times these figures
    // (41 slots per output for N = 2, two B words at 3 taps; the fit above is to containers of up to 4 bits)
    if (r.out_bits > 0 && container_of(r.p) == 8) block *= 1.5;
    return block / n;
}

// Container-aligned slices of SW bits (16, or 4 for one-bit unsigned operands): K = 1, N = 32/SW,
// the values of a word SW/c elements apart, every tap's product accumulated in the same word
// (chunks = taps).  Exact when the sum of taps products fits the slice (the symmetric signed
// bound of the carried-sign split, as in exact_ok) and the packed word fits the 24-bit
// multiplier input that the kernel uses; the kernel also needs equal input and output
// containers, at most 7 taps and a window of one output dword within 64 bits.
bool aligned_ok(const Req &r, int sw, Cand *out)
{
    if (r.mode != HIKONV_MODE_CONV1D || r.taps < 1 || r.taps > 7 || r.bipolar) return false;
    const int c = container_of(r.p);
    if (r.out_bits < 1 || r.out_bits > 8 || container_of(r.out_bits) != c) return false;
    if (sw % c != 0 || (32 / c + r.taps - 1) * c > 64) return false;
    if (r.L_A < 24 || r.L_B < 8 || r.L_acc < 32) return false;
    if (sw == 4 && (r.p != 1 || r.q != 1 || r.any_signed)) return false;
    if (sw == 16 && r.any_signed && r.p > 7) return false; // two values 16 bits apart must fit 24 bits signed
    const Range seg{r.prod.lo * r.taps, r.prod.hi * r.taps};
    if (sw == 4) {
        if (seg.hi > 7) return false; // the threshold compare keeps bit 3 of every slice free
    } else if (r.any_signed) {
        const i128 lim = ((i128)1 << (sw - 1)) - 1;
        if (seg.lo < -lim || seg.hi > lim) return false;
    } else if (seg.hi > ((i128)1 << sw) - 1) {
        return false;
    }
    out->n = 32 / sw;
    out->k = 1;
    out->s = sw;
    out->chunks = r.taps;
    out->stride = sw / c;
    const int prod_bits = r.p == 1 ? r.q : (r.q == 1 ? r.p : r.p + r.q);
    out->gb = sw - prod_bits;
    return true;
}

inline double priced(const Req &r, double slots)
{
    const double floor = hbm_floor_slots(r);
    return slots < floor ? floor : slots;
}

// Issue-slot model of the layer kernels (DNN mode).  Measured on gfx950: v_mad_u64_u32 and
// v_mad_u32_u24 both issue at (nearly) the full VALU rate, the layer kernel spends about 1.4 issue
// slots per multiply-accumulate (address and LDS traffic included), and a split costs an
// exchange (64-bit shift, DPP moves, 64-bit add) plus three instructions per field; the narrow
// path needs half the exchange.  Used to choose M when the caller leaves it open and, under the
// measured-cost objective, to choose among the candidates of a layer plan.
double modelled_macs_per_slot(const Req &r, const Cand &c)
{
    const bool wide = r.L_acc > 32;
    const double c_mul = 1.4;
    const double c_split = (wide ? 8.0 : 5.0) + 3.0 * c.n;
    const double macs = (double)r.M * c.n * r.taps;
    return macs / (r.M * c.chunks * c_mul + c_split);
}

inline bool by_cost_dnn(const Req &r) { return r.objective == HIKONV_OBJ_MEASURED_COST && r.mode == HIKONV_MODE_DNN && r.taps > 0; }

// score comparison: free mode -> Eq. tot_ops; fixed taps -> MACs per multiply n*taps/chunks
inline bool by_cost(const Req &r) { return r.objective == HIKONV_OBJ_MEASURED_COST && r.mode == HIKONV_MODE_CONV1D && r.taps > 0; }

inline bool better(const Req &r, const Cand &c, const Cand &best)
{
    if (!best.found) return true;
    if (by_cost(r)) {
        const double pc = priced(r, c.cost), pb = priced(r, best.cost);
        if (pc != pb) return pc < pb;
        // both under the memory floor: the kernel waits for HBM either way, and Algorithm 1's own
        // order (most multiply-accumulates per multiply) decides; then fewer slots
        if ((long long)c.n * best.chunks != (long long)best.n * c.chunks)
            return (long long)c.n * best.chunks > (long long)best.n * c.chunks;
        return c.cost < best.cost;
    }
    if (by_cost_dnn(r)) {
        // layers: most multiply-accumulates per modelled issue slot (splits and extra B words priced in)
        const double sc = modelled_macs_per_slot(r, c), sb = modelled_macs_per_slot(r, best);
        if (sc != sb) return sc > sb;
    }
    if (r.taps == 0)
        return (long long)c.n * c.k + (long long)(c.n - 1) * (c.k - 1) >
               (long long)best.n * best.k + (long long)(best.n - 1) * (best.k - 1);
    return (long long)c.n * best.chunks > (long long)best.n * c.chunks;
}

// paper_only: Eq. slice1-slice3 as printed and Algorithm 1's own objective, whatever the request's
Cand search(const Req &r_in, bool paper_only)
{
    Req r = r_in;
    if (paper_only) r.objective = HIKONV_OBJ_PAPER_OPS;
    Cand best;
    auto try_one = [&](int n, int k) {
        if (!paper_only && r.max_N > 0 && n > r.max_N) return; // Algorithm 1 itself has no such bound
        Cand c;
        c.n = n;
        c.k = k;
        c.gb = guard_bits(r, n, k);
        c.chunks = r.taps ? (r.taps + k - 1) / k : 1;
        const int s0 = slice_bits(r.p, r.q, c.gb);
        if (paper_only) {
            c.s = s0;
            if (!paper_fits(r, n, k, s0)) return;
        } else {
            // tight: the smallest slice that is provably exact for the declared value ranges
            // (the paper's p+q+G_b is an upper bound on what the segment sums need)
            c.s = 0;
            // ({-1,+1} data always: products are -1, 0 or 1, far below what two-bit operands could give)
            for (int s = r.tight || r.bipolar ? 1 : s0; s <= s0 + 1; ++s)
                if (exact_ok(r, n, k, s)) {
                    c.s = s;
                    break;
                }
            if (!c.s) return;
            if (c.s < s0) c.gb -= s0 - c.s;
        }
        if (r.mode == HIKONV_MODE_CONV1D && r.taps > 0) c.cost = conv1d_slots(r, c.n, c.k, c.chunks, c.s, 1);
        if (r.mode == HIKONV_MODE_DNN && r.taps > 0) c.cost = 1.0 / modelled_macs_per_slot(r, c); // slots per multiply-accumulate
        c.found = true;
        if (better(r, c, best)) best = c;
    };
    // container-aligned slices (outside Eq. slice1's S = p + q + G_b): only under the cost objective
    if (!paper_only && by_cost(r) && r.out_bits > 0) {
        for (int sw : {16, 4}) {
            Cand c;
            if (!aligned_ok(r, sw, &c)) continue;
            if (r.max_N > 0 && c.n > r.max_N) continue;
            c.cost = conv1d_slots(r, c.n, c.k, c.chunks, c.s, c.stride);
            c.found = true;
            if (better(r, c, best)) best = c;
        }
    }
    if (r.taps == 0) {
        for (int k = 1; k <= r.L_B; ++k)
            for (int n = 1; n <= r.L_A; ++n) try_one(n, k);
    } else {
        for (int k = r.taps; k >= 1; --k)
            for (int n = r.L_A; n >= 1; --n) try_one(n, k);
    }
    return best;
}

bool valid_request(const hikonv_plan_t &in)
{
    if (in.bits_a < 1 || in.bits_a > 8 || in.bits_w < 1 || in.bits_w > 8) return false;
    if (in.L_A < 1 || in.L_A > 64 || in.L_B < 1 || in.L_B > 64) return false;
    if (in.L_acc < 0 || in.L_acc > 128) return false;
    if (in.mode < HIKONV_MODE_SINGLE || in.mode > HIKONV_MODE_DNN) return false;
    if (in.M < 0 || in.M > (1 << 20) || in.taps < 0 || in.taps > 64) return false;
    if (in.bipolar && (in.bits_a != 1 || in.bits_w != 1)) return false;
    if (in.tight != 0 && in.tight != 1) return false;
    if (in.objective != HIKONV_OBJ_PAPER_OPS && in.objective != HIKONV_OBJ_MEASURED_COST) return false;
    if (in.out_bits < 0 || in.out_bits > 8 || in.max_N < 0 || in.max_N > 64) return false;
    if (in.kernel < HIKONV_KERNEL_AUTO || in.kernel > HIKONV_KERNEL_WINDOW) return false;
    if (in.flags & ~HIKONV_F_STORES64) return false;
    return true;
}

void fill_result(hikonv_plan_t *out, const Req &r, const Cand &c, bool paper_exact)
{
    out->L_acc = r.L_acc;
    out->M = r.M;
    out->N = c.n;
    out->K = c.k;
    out->S = c.s;
    out->G_b = c.gb;
    out->chunks = c.chunks;
    out->ops_per_mul = c.n * c.k + (c.n - 1) * (c.k - 1);
    out->paper_exact = paper_exact ? 1 : 0;
    out->stride_elems = c.stride;
    out->cost_milli = (int32_t)(c.cost * 1000.0 + 0.5);
}

} // namespace

extern "C" int hikonv_plan_ex(const hikonv_plan_t *request, hikonv_plan_t *out)
{
    if (!request || !out) return HIKONV_EINVAL;
    hikonv_plan_t in = *request;
    if (!valid_request(in)) return HIKONV_EINVAL;
    if (in.mode == HIKONV_MODE_DNN && in.M == 0) {
        // choose M by the issue-slot model; needs a fixed tap count
        if (in.taps == 0) return HIKONV_EINVAL;
        double best_score = -1.0;
        hikonv_plan_t best_plan = in;
        bool any = false;
        for (int m = 1; m <= 512; ++m) {
            hikonv_plan_t trial = in;
            trial.M = m;
            Req r = make_req(trial);
            Cand c = search(r, false);
            if (!c.found) continue;
            double sc = modelled_macs_per_slot(r, c);
            if (sc > best_score * 1.0000001) {
                best_score = sc;
                Cand pc = search(r, true);
                fill_result(&trial, r, c, pc.found && pc.n == c.n && pc.k == c.k && pc.s == c.s && c.stride == 1);
                best_plan = trial;
                any = true;
            }
        }
        if (!any) return HIKONV_ENOPLAN;
        *out = best_plan;
        return HIKONV_OK;
    }
    Req r = make_req(in);
    Cand c = search(r, false);
    if (!c.found) return HIKONV_ENOPLAN;
    Cand pc = search(r, true);
    *out = in;
    fill_result(out, r, c, pc.found && pc.n == c.n && pc.k == c.k && pc.s == c.s && c.stride == 1);
    return HIKONV_OK;
}

extern "C" int hikonv_plan(int bits_a, int bits_w, int signedness, int mult_width, hikonv_plan_t *out)
{
    if (!out || signedness < 0 || signedness > 7) return HIKONV_EINVAL;
    hikonv_plan_t in = {};
    in.bits_a = bits_a;
    in.bits_w = bits_w;
    in.a_signed = (signedness & HIKONV_A_SIGNED) ? 1 : 0;
    in.w_signed = (signedness & HIKONV_W_SIGNED) ? 1 : 0;
    in.bipolar = (signedness & HIKONV_BIPOLAR) ? 1 : 0;
    in.L_A = in.L_B = mult_width;
    in.L_acc = 2 * mult_width;
    in.mode = HIKONV_MODE_SINGLE;
    return hikonv_plan_ex(&in, out);
}

extern "C" int hikonv_plan_check(const hikonv_plan_t *plan)
{
    if (!plan || !valid_request(*plan)) return HIKONV_EINVAL;
    if (plan->N < 1 || plan->K < 1 || plan->S < 1 || plan->N > 64 || plan->K > 64) return HIKONV_EINVAL;
    if (plan->taps && plan->chunks != (plan->taps + plan->K - 1) / plan->K) return HIKONV_EINVAL;
    if (plan->stride_elems < 0 || plan->stride_elems > 32) return HIKONV_EINVAL;
    if (plan->max_N > 0 && plan->N > plan->max_N) return HIKONV_EINVAL;
    Req r = make_req(*plan);
    if (plan->stride_elems > 1) {
        // container-aligned slices: the one form per slice width that aligned_ok describes
        if (r.out_bits == 0) r.out_bits = r.p; // the check needs a container: the input's own
        Cand c;
        if (!aligned_ok(r, plan->S, &c)) return plan->S == 16 || plan->S == 4 ? HIKONV_EOVERFLOW : HIKONV_EINVAL;
        if (c.n != plan->N || c.k != plan->K || c.stride != plan->stride_elems || c.chunks != plan->chunks)
            return HIKONV_EINVAL;
        return HIKONV_OK;
    }
    return exact_ok(r, plan->N, plan->K, plan->S) ? HIKONV_OK : HIKONV_EOVERFLOW;
}

extern "C" int hikonv_plan_cost(const hikonv_plan_t *plan)
{
    int rc = hikonv_plan_check(plan);
    if (rc != HIKONV_OK) return rc;
    if (plan->taps < 1 || plan->mode == HIKONV_MODE_SINGLE) return HIKONV_EUNSUPPORTED;
    Req r = make_req(*plan);
    if (plan->mode == HIKONV_MODE_DNN) {
        Cand c;
        c.n = plan->N;
        c.k = plan->K;
        c.chunks = plan->chunks;
        return (int)(1000.0 / modelled_macs_per_slot(r, c) + 0.5);
    }
    const double slots = conv1d_slots(r, plan->N, plan->K, plan->chunks, plan->S, plan->stride_elems > 1 ? plan->stride_elems : 1);
    return (int)(slots * 1000.0 + 0.5);
}

extern "C" int64_t hikonv_bitdense_row_bytes(int64_t len, int bits)
{
    int c = hikonv::container_bits(bits);
    if (c == 0 || len < 0) return -1;
    return ((len * c + 31) / 32) * 4;
}

extern "C" const char *hikonv_strerror(int code)
{
    switch (code) {
    case HIKONV_OK: return "ok";
    case HIKONV_EINVAL: return "invalid argument";
    case HIKONV_EOVERFLOW: return "result may not fit (int32 output or packed field)";
    case HIKONV_ENOPLAN: return "no packing plan satisfies the constraints";
    case HIKONV_EHIP: return "HIP runtime error";
    case HIKONV_EWORKSPACE: return "workspace missing, misaligned or too small";
    case HIKONV_EUNSUPPORTED: return "request not supported by this build";
    case HIKONV_ESCRATCH: return "layer needs more than the library's fixed scratch array (hikonv_conv2d_noalloc)";
    default: return "unknown error";
    }
}
