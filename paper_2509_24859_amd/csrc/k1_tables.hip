// Segment-cost table build for gfx950: running sums over the operator sequence.
//
// The planner of the paper's section 5.2.3 looks up the cost of a candidate stage (a contiguous
// operator range on a submesh) many times; section 5.1 stores those costs once.  Here the stored
// form is one running sum per quantity, so that a segment's compute time, all-reduce time and
// memory are each one subtraction: PF per GPU type, PP, PS, and PR per (group, degree).
//
// The work is a batch of independent row scans over L operators.  It is HBM-streaming work:
// reduce-then-scan in three launches (chunk sums, scan of chunk sums per row, scan of each chunk
// with its offset), every global access a coalesced 32-byte-per-lane run.  At L <= 1024 a row is a
// single chunk and only the last launch runs.  The same launch validates the inputs it reads.
#include "harp_internal.h"

namespace harp {

namespace {

__device__ __forceinline__ int64_t ceil_div_u(int64_t a, int64_t b) {
    return (int64_t)(((unsigned long long)a + (unsigned long long)b - 1ull) / (unsigned long long)b);
}

// ceil(a / b) for a row-invariant divisor b with inv = 1.0 / b precomputed.  For a, b < 2^52 the
// double product a * inv is within 1 of the true quotient, so one exact correction step on the
// integer remainder gives floor(a / b); larger operands take the plain 64-bit division.  Exact
// for all inputs; the point is that a table row costs a multiply per element instead of a
// software division, which would otherwise out-weigh the HBM traffic of the row.
constexpr int64_t kFastDivLimit = int64_t(1) << 52;

__device__ __forceinline__ int64_t ceil_div_inv(int64_t a, int64_t b, double inv) {
    if (a >= kFastDivLimit || b >= kFastDivLimit) return ceil_div_u(a, b);
    int64_t q = (int64_t)((double)a * inv);
    int64_t r = a - q * b;
    if (r < 0) { q -= 1; r += b; }
    else if (r >= b) { q += 1; r -= b; }
    return q + (r != 0 ? 1 : 0);
}

// Sum of two non-negative 64-bit values, with the sticky overflow note of the table build: `over`
// collects the upper halves of every sum formed, so its top bit says that some running sum reached
// 2^63.  The first sum to do so has operands below 2^63 and cannot wrap, and since all terms are
// non-negative a partial sum reaches 2^63 exactly when its row's total does: the verdict is the exact
// one, whatever the order in which the scan adds.
__device__ __forceinline__ int64_t add_checked(int64_t a, int64_t b, unsigned int &over) {
    const unsigned long long s = (unsigned long long)a + (unsigned long long)b;
    over |= (unsigned int)(s >> 32);
    return (int64_t)s;
}

// Value of element l of table row r, with the checks that belong to the inputs it touches.
struct RowSource {
    const int64_t *a;     // first addend
    const int64_t *b;     // second addend or nullptr
    int64_t num_mul;      // all-reduce rows: ar_count * 2 * (tp - 1); 0 for plain rows
    int64_t den;          // all-reduce rows: tp * bw[g][g]
    double inv_den;       // 1.0 / den
    bool is_ar;
    bool track_act;       // this row also reports max(act_bytes)
};

__device__ __forceinline__ RowSource row_source(const TablesDev &tb, int r) {
    RowSource s;
    s.b = nullptr; s.num_mul = 0; s.den = 1; s.inv_den = 1.0; s.is_ar = false; s.track_act = false;
    if (r < tb.T) {
        s.a = tb.fwd_us + int64_t(r) * tb.L;
        s.b = tb.bwd_us + int64_t(r) * tb.L;
    } else if (r == tb.T) {
        s.a = tb.param_bytes;
    } else if (r == tb.T + 1) {
        s.a = tb.stash_bytes;
    } else {
        int q = r - (tb.T + 2);
        int g = q / tb.n_tp, k = q - g * tb.n_tp;
        int64_t tp = tb.tp[k];
        s.a = tb.act_bytes;
        s.is_ar = true;
        s.track_act = (q == 0);
        s.num_mul = int64_t(tb.ar_count) * 2 * (tp - 1);
        int64_t link = tb.bw[int64_t(g) * tb.G + g];
        // a bad link value is reported by the finalize kernel; keep the division defined here
        s.den = (link >= 1 && link <= INT64_MAX / tp) ? tp * link : 1;
        s.inv_den = 1.0 / (double)s.den;
    }
    return s;
}

__device__ __forceinline__ int64_t row_value(const RowSource &s, int64_t l, const BuildLimits &lim,
                                             unsigned int &bad, unsigned int &ovf,
                                             unsigned long long &act_seen) {
    int64_t x = s.a[l];
    if (x < 0) { bad = 1; x = 0; }
    if (s.is_ar) {
        if ((unsigned long long)x > act_seen) act_seen = (unsigned long long)x;
        if (x > lim.act_max) { ovf |= 0x80000000u; x = 0; }     // the numerator ar_count 2 (tp - 1) act would leave int64
        if (s.num_mul == 0) return 0;
        return ceil_div_inv(s.num_mul * x, s.den, s.inv_den);
    }
    if (s.b) {
        int64_t y = s.b[l];
        if (y < 0) { bad = 1; y = 0; }
        x = add_checked(x, y, ovf);
    }
    return x;
}

__device__ __forceinline__ int64_t wave_inclusive_scan(int64_t v, int lane, unsigned int &over) {
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        int64_t up = __shfl_up(v, d, 64);
        if (lane >= d) v = add_checked(v, up, over);
    }
    return v;
}

__device__ __forceinline__ void report(BuildHeader *h, unsigned int bad, unsigned int ovf,
                                       unsigned long long act_seen, bool track_act) {
    if (__any(bad) && (threadIdx.x & 63) == 0) atomicOr(&h->bad_arg, 1u);
    if (__any(ovf >> 31) && (threadIdx.x & 63) == 0) atomicOr(&h->overflow, 1u);
    if (track_act) atomicMax(&h->max_act, act_seen);
}

// Launch 1 (only when a row spans several chunks): sum of every chunk.
__global__ __launch_bounds__(kScanThreads) void k1_chunk_sums(TablesDev tb, BuildLimits lim, int n_chunks) {
    const int r = blockIdx.x, chunk = blockIdx.y;   // rows fastest: a chunk of act_bytes is reused across rows while in L2
    const RowSource src = row_source(tb, r);
    unsigned int bad = 0, ovf = 0;
    unsigned long long act_seen = 0;
    int64_t base = int64_t(chunk) * kScanChunk + int64_t(threadIdx.x) * kScanItems;
    int64_t sum = 0;
#pragma unroll
    for (int q = 0; q < kScanItems; ++q)
        if (base + q < tb.L) sum += row_value(src, base + q, lim, bad, ovf, act_seen);
    __shared__ int64_t part[kScanThreads / 64];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    int64_t inc = wave_inclusive_scan(sum, lane, ovf);
    if (lane == 63) part[wave] = inc;
    __syncthreads();
    if (threadIdx.x == 0) {
        int64_t t = 0;
        for (int w = 0; w < kScanThreads / 64; ++w) t += part[w];
        tb.chunk_sums[int64_t(r) * n_chunks + chunk] = t;
    }
    // values and sums inside a chunk are checked again by the last launch, sums across chunks by
    // the next one; nothing to report here
}

// Launch 2: exclusive scan of the chunk sums of each row, in place.  A thread takes a stretch of
// consecutive sums - in registers when there are at most kSumsInRegs of them, so that the row is
// read in one round trip and written in one - and the stretches' totals are scanned over the
// workgroup.
constexpr int kSumsInRegs = 16;

__global__ __launch_bounds__(kScanThreads) void k1_scan_chunk_sums(TablesDev tb, int n_chunks) {
    int64_t *row = tb.chunk_sums + int64_t(blockIdx.x) * n_chunks;
    __shared__ int64_t part[kScanThreads / 64];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int per = (n_chunks + kScanThreads - 1) / kScanThreads;
    const int begin = threadIdx.x * per;
    const int end = begin + per < n_chunks ? begin + per : n_chunks;    // below begin for the idle threads
    unsigned int over = 0;
    int64_t vals[kSumsInRegs];
    int64_t mine = 0;
    if (per <= kSumsInRegs) {
#pragma unroll
        for (int q = 0; q < kSumsInRegs; ++q) vals[q] = begin + q < end ? row[begin + q] : 0;
#pragma unroll
        for (int q = 0; q < kSumsInRegs; ++q) mine = add_checked(mine, vals[q], over);
    } else {
        for (int i = begin; i < end; ++i) mine = add_checked(mine, row[i], over);
    }
    const int64_t inc = wave_inclusive_scan(mine, lane, over);
    if (lane == 63) part[wave] = inc;
    __syncthreads();
    int64_t off = 0;
    for (int w = 0; w < wave; ++w) off = add_checked(off, part[w], over);
    add_checked(off, inc, over);                                        // the last thread's is the row's total
    int64_t before = off + (inc - mine);                                // sum of everything before this stretch
    if (per <= kSumsInRegs) {
#pragma unroll
        for (int q = 0; q < kSumsInRegs; ++q) {
            if (begin + q < end) row[begin + q] = before;
            before += vals[q];
        }
    } else {
        for (int i = begin; i < end; ++i) {
            const int64_t v = row[i];
            row[i] = before;
            before += v;
        }
    }
    report(tb.header, 0, over, 0, false);
}

// Launch 3: scan each chunk, add the chunk's offset, write the table row (entry i = l + 1).
__global__ __launch_bounds__(kScanThreads) void k1_scan_rows(TablesDev tb, BuildLimits lim, int n_chunks) {
    const int r = blockIdx.x, chunk = blockIdx.y;   // rows fastest: a chunk of act_bytes is reused across rows while in L2
    const RowSource src = row_source(tb, r);
    unsigned int bad = 0, ovf = 0;
    unsigned long long act_seen = 0;
    int64_t base = int64_t(chunk) * kScanChunk + int64_t(threadIdx.x) * kScanItems;
    int64_t v[kScanItems];
    int64_t sum = 0;
#pragma unroll
    for (int q = 0; q < kScanItems; ++q) {
        v[q] = (base + q < tb.L) ? row_value(src, base + q, lim, bad, ovf, act_seen) : 0;
        sum = add_checked(sum, v[q], ovf);
    }
    __shared__ int64_t part[kScanThreads / 64];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    int64_t inc = wave_inclusive_scan(sum, lane, ovf);
    if (lane == 63) part[wave] = inc;
    __syncthreads();
    int64_t run = (n_chunks > 1) ? tb.chunk_sums[int64_t(r) * n_chunks + chunk] : 0;
    for (int w = 0; w < wave; ++w) run = add_checked(run, part[w], ovf);
    run = add_checked(run, inc - sum, ovf);
    int64_t *out = tb.rows + int64_t(r) * tb.pitch;
    if (chunk == 0 && threadIdx.x == 0) out[0] = 0;
#pragma unroll
    for (int q = 0; q < kScanItems; ++q) {
        run = add_checked(run, v[q], ovf);
        if (base + q < tb.L) out[base + q + 1] = run;
    }
    unsigned long long wave_act = act_seen;
    if (src.track_act) {
#pragma unroll
        for (int d = 32; d >= 1; d >>= 1) {
            unsigned long long o = __shfl_xor(wave_act, d, 64);
            wave_act = o > wave_act ? o : wave_act;
        }
    }
    report(tb.header, bad, ovf, wave_act, src.track_act && lane == 0);
}

// ---------------------------------------------------------------------------------------------
// Long sequences (L >= kLongL): the same three launches, but chunk-major.  One wavefront owns a
// run of 256 operators and walks all table rows over it, so the act_bytes of the run are read,
// checked and converted once for the G * n_tp all-reduce rows instead of once per row, no LDS and
// no barrier is needed (chunk = wavefront), and the per-element all-reduce time is a handful of
// double operations: for act < 2^32, multiplier < 2^20 and divisor < 2^52 the product is exact in
// a double, floor(product * (1 / divisor)) is within 1 of the quotient, and one exact fused
// multiply-add gives the remainder that corrects it.  What is left is the 8-byte store per table
// entry, i.e. the HBM write stream.

typedef long long i64x2 __attribute__((ext_vector_type(2)));
constexpr int kWaveItems = 4;
constexpr int kWaveChunk = 64 * kWaveItems;

struct ActRun {                 // one thread's operators of the run
    int64_t x[kWaveItems];      // act_bytes, 0 beyond L or when rejected
    double xd[kWaveItems];      // the same as doubles when all are below 2^32
    bool narrow;                // every x below 2^32
};

__device__ __forceinline__ ActRun load_act_run(const TablesDev &tb, const BuildLimits &lim, int64_t base,
                                               unsigned int &bad, unsigned int &ovf,
                                               unsigned long long &act_seen) {
    ActRun a;
    a.narrow = true;
#pragma unroll
    for (int q = 0; q < kWaveItems; ++q) {
        int64_t x = (base + q < tb.L) ? tb.act_bytes[base + q] : 0;
        if (x < 0) { bad = 1; x = 0; }
        if ((unsigned long long)x > act_seen) act_seen = (unsigned long long)x;
        if (x > lim.act_max) { ovf |= 0x80000000u; x = 0; }
        a.x[q] = x;
        a.narrow = a.narrow && x < (int64_t(1) << 32);
        a.xd[q] = (double)(uint32_t)x;
    }
    return a;
}

struct ArRow {                  // constants of one all-reduce row
    int64_t mul, den;
    double mul_d, den_d, inv;
    bool fast;                  // multiplier < 2^20 and divisor < 2^52
};

__device__ __forceinline__ ArRow ar_row(const RowSource &s) {
    ArRow r;
    r.mul = s.num_mul; r.den = s.den; r.inv = s.inv_den;
    r.mul_d = (double)s.num_mul; r.den_d = (double)s.den;
    r.fast = s.num_mul < (int64_t(1) << 20) && s.den < kFastDivLimit;
    return r;
}

__device__ __forceinline__ int64_t ar_value(const ArRow &r, const ActRun &a, int q, const BuildLimits &lim,
                                            unsigned int &ovf) {
    if (r.mul == 0) return 0;
    int64_t v;
    if (r.fast && a.narrow) {
        const double prod = a.xd[q] * r.mul_d;            // exact: below 2^52
        double quo = floor(prod * r.inv);
        double rem = fma(-quo, r.den_d, prod);            // exact: |rem| < 2 den
        if (rem < 0.0) { quo -= 1.0; rem += r.den_d; }
        else if (rem >= r.den_d) { quo += 1.0; rem -= r.den_d; }
        v = (int64_t)(quo + (rem > 0.0 ? 1.0 : 0.0));
    } else {
        v = ceil_div_inv(r.mul * a.x[q], r.den, r.inv);
    }
    return v;
}

// The common case of an all-reduce row, all four values at once: narrow operands (see ar_row), a
// divisor not below the multiplier (so the quotient stays below 2^32).  ceil(p / d) = floor((p + d - 1) / d); the sum p + d - 1 is
// exact in a double, the product with 1 / d is within 1 of the quotient, and the exact remainder
// from one fused multiply-add corrects it.
__device__ __forceinline__ bool ar_tight(const ArRow &r, bool all_narrow, const BuildLimits &lim) {
    return r.fast && all_narrow && r.den >= r.mul;
}

__device__ __forceinline__ void ar_values_tight(const ArRow &r, const ActRun &a, uint32_t v[kWaveItems]) {
    const double bias = r.den_d - 1.0;
#pragma unroll
    for (int q = 0; q < kWaveItems; ++q) {
        const double num = fma(a.xd[q], r.mul_d, bias);   // exact: below 2^53
        double quo = floor(num * r.inv);
        const double rem = fma(-quo, r.den_d, num);       // exact
        quo += rem < 0.0 ? -1.0 : (rem >= r.den_d ? 1.0 : 0.0);
        v[q] = r.mul == 0 ? 0u : (uint32_t)quo;
    }
}

// Raw values of one thread's four operators of a row that reads memory (a fixed row: fwd + bwd of
// a type, parameter bytes, stash bytes), loaded ahead of their use; zero beyond L.
constexpr int kRowsInFlight = 2;
struct MemRow {
    int64_t a[kWaveItems], b[kWaveItems];
};

__device__ __forceinline__ MemRow load_mem_row(const RowSource &s, int64_t base, int64_t L) {
    MemRow w;
#pragma unroll
    for (int q = 0; q < kWaveItems; ++q) {
        const bool in = base + q < L;
        w.a[q] = in ? s.a[base + q] : 0;
        w.b[q] = (in && s.b) ? s.b[base + q] : 0;
    }
    return w;
}

// the checks and the sum of row_value for a fixed row, on values already loaded
__device__ __forceinline__ int64_t mem_row_value(const MemRow &w, int q, unsigned int &bad, unsigned int &ovf) {
    int64_t x = w.a[q], y = w.b[q];
    if (x < 0) { bad = 1; x = 0; }
    if (y < 0) { bad = 1; y = 0; }
    return add_checked(x, y, ovf);
}

// value q of row r for this thread: all-reduce rows from the staged run, the others from memory
__device__ __forceinline__ int64_t long_value(const TablesDev &tb, const RowSource &src, const ArRow &arr,
                                              const ActRun &a, int q, int64_t base, const BuildLimits &lim,
                                              unsigned int &bad, unsigned int &ovf) {
    if (base + q >= tb.L) return 0;
    if (src.is_ar) return ar_value(arr, a, q, lim, ovf);
    unsigned long long unused = 0;
    return row_value(src, base + q, lim, bad, ovf, unused);
}

// Order in which the long kernels walk the table rows: the fixed rows first, then the all-reduce
// rows degree-major, so that groups whose own link has the same speed (the usual case: subclusters
// of one GPU type) come one after the other with identical constants, and a row that equals the
// one before it is stored again without being recomputed.  The gridDim.y parts of a launch take
// consecutive stretches of this order.  (Dealing the fixed rows, the ones that read their values
// from memory, evenly over the parts was measured and is slower: 0.45 against 0.40 ms per build.)
struct LongPart {
    int x_begin, x_end;     // walk positions of this part
};

__device__ __forceinline__ LongPart long_part(const TablesDev &tb) {
    const int n_rows = tb.n_rows();
    LongPart lp;
    lp.x_begin = int(int64_t(n_rows) * blockIdx.y / gridDim.y);
    lp.x_end = int(int64_t(n_rows) * (blockIdx.y + 1) / gridDim.y);
    return lp;
}

__device__ __forceinline__ int long_row_order(const TablesDev &tb, const LongPart &, int x) {
    const int n_fixed = tb.T + 2;
    if (x < n_fixed) return x;
    const int e = x - n_fixed;
    const int k = e / tb.G, g = e - k * tb.G;
    return n_fixed + g * tb.n_tp + k;
}

// Row constants of the table rows a workgroup walks (its part of the order
// above), worked out once per workgroup (each needs a link bandwidth from memory and a reciprocal)
// and kept in LDS.  The array is dynamic LDS sized for the workgroup's share of this problem's rows:
// a fixed array for the largest case would leave room for two workgroups per CU only.
struct LongRow {
    RowSource src;
    ArRow arr;
};
constexpr int kLongRowsInLds = 512;     // rows per workgroup beyond which the constants are recomputed per use

// What the walk needs first of a row, 8 bytes: the table row it is, and whether it is an all-reduce
// row of the tight form with the same multiplier and divisor as the row walked just before it.  Most
// rows of a cluster are (groups of one GPU type share their link speed), and for those the walk
// reads nothing else.
struct LongRowKey {
    int32_t r;
    int32_t same_as_previous;
};

__device__ __forceinline__ bool ar_tight_row(const LongRow &lr) {
    return lr.src.is_ar && lr.arr.fast && lr.arr.den >= lr.arr.mul;
}

// Dynamic LDS of the long kernels: the workgroup's row constants, then their keys.
__device__ __forceinline__ LongRowKey *long_row_keys(LongRow *rows_lds, int x_begin, int x_end) {
    return reinterpret_cast<LongRowKey *>(rows_lds + (x_end - x_begin));
}

__device__ __forceinline__ void stage_long_rows(const TablesDev &tb, LongRow *rows_lds, const LongPart &lp) {
    const int x_begin = lp.x_begin, x_end = lp.x_end;
    if (x_end - x_begin <= kLongRowsInLds) {
        LongRowKey *keys = long_row_keys(rows_lds, x_begin, x_end);
        for (int x = x_begin + threadIdx.x; x < x_end; x += blockDim.x) {
            const int r = long_row_order(tb, lp, x);
            rows_lds[x - x_begin].src = row_source(tb, r);
            rows_lds[x - x_begin].arr = ar_row(rows_lds[x - x_begin].src);
            keys[x - x_begin].r = r;
        }
        __syncthreads();
        for (int x = x_begin + threadIdx.x; x < x_end; x += blockDim.x) {
            bool same = false;
            if (x > x_begin) {
                const LongRow &a = rows_lds[x - x_begin], &b = rows_lds[x - 1 - x_begin];
                same = ar_tight_row(a) && ar_tight_row(b) && a.arr.mul == b.arr.mul && a.arr.den == b.arr.den;
            }
            keys[x - x_begin].same_as_previous = same ? 1 : 0;
        }
    }
    __syncthreads();
}

__device__ __forceinline__ LongRow long_row(const TablesDev &tb, const LongRow *rows_lds, const LongPart &lp, int x) {
    if (lp.x_end - lp.x_begin <= kLongRowsInLds) return rows_lds[x - lp.x_begin];
    LongRow lr;
    lr.src = row_source(tb, long_row_order(tb, lp, x));
    lr.arr = ar_row(lr.src);
    return lr;
}

// Launch 1 for long sequences: sum of every (row, run of 256 operators).
__global__ __launch_bounds__(kScanThreads) void k1_long_sums(TablesDev tb, BuildLimits lim, int n_runs) {
    extern __shared__ __align__(16) unsigned char long_lds[];
    LongRow *rows_lds = reinterpret_cast<LongRow *>(long_lds);
    // the rows are split over gridDim.y workgroups so that enough wavefronts are in flight
    const LongPart lp = long_part(tb);
    const int x_begin = lp.x_begin, x_end = lp.x_end;
    stage_long_rows(tb, rows_lds, lp);
    const bool keyed = x_end - x_begin <= kLongRowsInLds;
    const LongRowKey *keys = long_row_keys(rows_lds, x_begin, x_end);
    const int lane = threadIdx.x & 63;
    // a wavefront takes every (gridDim.x * wavefronts per workgroup)-th run, so that the row constants
    // staged above serve several runs
    for (int run = blockIdx.x * (kScanThreads / 64) + (threadIdx.x >> 6); run < n_runs;
         run += gridDim.x * (kScanThreads / 64)) {
    const int64_t base = int64_t(run) * kWaveChunk + int64_t(lane) * kWaveItems;
    unsigned int bad = 0, ovf = 0;
    unsigned long long act_seen = 0;
    const ActRun a = load_act_run(tb, lim, base, bad, ovf, act_seen);
    const bool all_narrow = __all(a.narrow);
    int64_t same_mul = -1, same_den = -1, same_sum = 0;     // the all-reduce row computed last
    // the rows that read their values from memory come first in the order: their loads are issued
    // kRowsInFlight rows at a time, so that a run waits for memory once per batch, not once per row
    const int n_fixed = tb.T + 2;
    const int m_end = x_end < n_fixed ? x_end : n_fixed;
    int x_from = x_begin;
    for (int x0 = x_begin; x0 < m_end; x0 += kRowsInFlight) {
        MemRow w[kRowsInFlight];
#pragma unroll
        for (int u = 0; u < kRowsInFlight; ++u)
            if (x0 + u < m_end) w[u] = load_mem_row(long_row(tb, rows_lds, lp, x0 + u).src, base, tb.L);
#pragma unroll
        for (int u = 0; u < kRowsInFlight; ++u) {
            if (x0 + u >= m_end) break;
            int64_t sum = 0;
#pragma unroll
            for (int q = 0; q < kWaveItems; ++q) sum += mem_row_value(w[u], q, bad, ovf);
#pragma unroll
            for (int d = 32; d >= 1; d >>= 1) sum += __shfl_xor(sum, d, 64);
            if (lane == 0) tb.chunk_sums[int64_t(x0 + u) * n_runs + run] = sum;
        }
        x_from = m_end;
    }
    for (int x = x_from; x < x_end; ++x) {
        if (keyed) {
            const LongRowKey key = keys[x - x_begin];
            if (key.same_as_previous && all_narrow) {       // the row before it took the tight form: same sum
                if (lane == 0) tb.chunk_sums[int64_t(key.r) * n_runs + run] = same_sum;
                continue;
            }
        }
        const int r = long_row_order(tb, lp, x);
        const LongRow lr = long_row(tb, rows_lds, lp, x);
        const RowSource &src = lr.src;
        const ArRow &arr = lr.arr;
        int64_t sum = 0;
        if (src.is_ar && ar_tight(arr, all_narrow, lim)) {
            if (arr.mul == same_mul && arr.den == same_den) {
                sum = same_sum;                             // same link speed and degree: the same row
            } else {
                uint32_t v[kWaveItems];
                ar_values_tight(arr, a, v);
#pragma unroll
                for (int q = 0; q < kWaveItems; ++q) sum += v[q];
#pragma unroll
                for (int d = 32; d >= 1; d >>= 1) sum += __shfl_xor(sum, d, 64);
                same_mul = arr.mul; same_den = arr.den; same_sum = sum;
            }
        } else {
#pragma unroll
            for (int q = 0; q < kWaveItems; ++q) sum += long_value(tb, src, arr, a, q, base, lim, bad, ovf);
#pragma unroll
            for (int d = 32; d >= 1; d >>= 1) sum += __shfl_xor(sum, d, 64);
        }
        if (lane == 0) tb.chunk_sums[int64_t(r) * n_runs + run] = sum;
    }
    }
    // values are checked again by the scan launch; nothing to report here
}

// Launch 3 for long sequences: scan every (row, run), add the run's offset, write the table rows.
__global__ __launch_bounds__(kScanThreads) void k1_long_scan(TablesDev tb, BuildLimits lim, int n_runs) {
    extern __shared__ __align__(16) unsigned char long_lds[];
    LongRow *rows_lds = reinterpret_cast<LongRow *>(long_lds);
    // the rows are split over gridDim.y workgroups so that enough wavefronts are in flight
    const LongPart lp = long_part(tb);
    const int x_begin = lp.x_begin, x_end = lp.x_end;
    stage_long_rows(tb, rows_lds, lp);
    __shared__ __align__(16) int64_t tiles[kScanThreads / 64][kWaveChunk + 2];
    const bool keyed = x_end - x_begin <= kLongRowsInLds;
    const LongRowKey *keys = long_row_keys(rows_lds, x_begin, x_end);
    const int lane = threadIdx.x & 63;
    int64_t *tile = tiles[threadIdx.x >> 6];
    unsigned int bad = 0, ovf = 0;
    unsigned long long act_seen = 0;
    for (int run = blockIdx.x * (kScanThreads / 64) + (threadIdx.x >> 6); run < n_runs;
         run += gridDim.x * (kScanThreads / 64)) {
    const int64_t base = int64_t(run) * kWaveChunk + int64_t(lane) * kWaveItems;
    const ActRun a = load_act_run(tb, lim, base, bad, ovf, act_seen);
    const bool all_narrow = __all(a.narrow);
    int64_t same_mul = -1, same_den = -1, same_start = -1;  // what the LDS tile currently holds
    for (int x = x_begin; x < x_end; ++x) {
        LongRowKey key;
        if (keyed) key = keys[x - x_begin];
        else { key.r = long_row_order(tb, lp, x); key.same_as_previous = 0; }
        const int r = key.r;
        int64_t *out = tb.rows + int64_t(r) * tb.pitch;
        const int64_t start = tb.chunk_sums[int64_t(r) * n_runs + run];   // sum of the row before this run
        // rows of groups with the same link speed and degree are identical: when the row walked just
        // before this one took the tight form with the same constants and started from the same sum,
        // the tile already holds this row (the key says so without a look at the row's constants)
        bool reuse = key.same_as_previous && all_narrow && same_mul >= 0 && start == same_start;
        if (!reuse) {
            const LongRow lr = long_row(tb, rows_lds, lp, x);
            const RowSource &src = lr.src;
            const ArRow &arr = lr.arr;
            const bool tight = src.is_ar && ar_tight(arr, all_narrow, lim);
            reuse = tight && arr.mul == same_mul && arr.den == same_den && start == same_start;
            if (!reuse) {
                int64_t v[kWaveItems];
                int64_t sum = 0;
                if (tight) {
                    uint32_t v32[kWaveItems];
                    ar_values_tight(arr, a, v32);
#pragma unroll
                    for (int q = 0; q < kWaveItems; ++q) { v[q] = v32[q]; sum += v32[q]; }
                    same_mul = arr.mul; same_den = arr.den; same_start = start;
                } else {
#pragma unroll
                    for (int q = 0; q < kWaveItems; ++q) {
                        v[q] = long_value(tb, src, arr, a, q, base, lim, bad, ovf);
                        sum = add_checked(sum, v[q], ovf);
                    }
                    same_mul = -1;
                }
                const int64_t inc = wave_inclusive_scan(sum, lane, ovf);
                int64_t acc = add_checked(start, inc - sum, ovf);
                // a lane holds four consecutive entries; passing them through the wavefront's LDS tile
                // turns four 8-byte stores at a 32-byte stride into four fully contiguous 512-byte stores
#pragma unroll
                for (int q = 0; q < kWaveItems; ++q) {
                    acc = add_checked(acc, v[q], ovf);
                    tile[lane * kWaveItems + q + 1] = acc;
                }
                if (lane == 0) tile[0] = start;
            }
        }
        // the wavefront stores entries first .. first + 255 of the row (entry first is the sum before
        // the run, so a row's leading zero comes from run 0), 16 bytes per lane: rows start on 128-byte
        // lines and so does every run, and a store instruction covers eight whole lines
        const int64_t first = int64_t(run) * kWaveChunk;
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const int e = h * 128 + 2 * lane;
            const i64x2 val = *reinterpret_cast<const i64x2 *>(&tile[e]);
            if (first + e + 1 <= tb.L) __builtin_nontemporal_store(val, reinterpret_cast<i64x2 *>(&out[first + e]));
            else if (first + e <= tb.L) out[first + e] = val.x;
        }
        // a sequence that ends with a full run: its last entry lies one past the last window
        if (first + kWaveChunk == tb.L && lane == 0) out[tb.L] = tile[kWaveChunk];
    }
    }
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) {
        const unsigned long long o = __shfl_xor(act_seen, d, 64);
        act_seen = o > act_seen ? o : act_seen;
    }
    report(tb.header, bad, ovf, act_seen, lane == 0 && blockIdx.y == 0);
}

// Launch 4 (one workgroup): checks of the small arrays, device numbering of the groups, the
// magnitude verdict, and whether the 32-bit fast path may be used.  The kernel is a chain of
// dependent memory round trips and little else, so everything whose address depends on nothing -
// each thread's first element of every array, the all-reduce totals, what thread 0 needs at the end -
// is loaded before the first wait; only the work totals (their row is the group's type) come second.
__global__ __launch_bounds__(256) void k1_finalize(TablesDev tb, BuildLimits lim) {
    __shared__ unsigned int bad_s, ovf_s;
    __shared__ unsigned long long min_bw_s;
    __shared__ long long worst_s, worst32_s;
    __shared__ long long wave_total[4];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int L = tb.L;
    const int64_t n_links = int64_t(tb.G) * tb.G;
    const int n_pairs = tb.G * tb.n_tp;
    const int per = (tb.G + 255) / 256;                 // consecutive groups per thread for the numbering
    const int g_begin = tid * per, g_end = (g_begin + per) < tb.G ? (g_begin + per) : tb.G;

    const int64_t bw0 = tid < n_links ? tb.bw[tid] : 1;
    const int64_t mem0 = tid < tb.T ? tb.type_mem[tid] : 0;
    int type0 = 0, ndev0 = 1;
    if (tid < tb.G) { type0 = tb.group_type[tid]; ndev0 = tb.group_ndev[tid]; }
    const int first_ndev = g_begin < g_end ? tb.group_ndev[g_begin] : 0;
    int pair_type = 0;
    unsigned long long pair_ar = 0;
    if (tid < n_pairs) {
        const int g = tid / tb.n_tp, k = tid - g * tb.n_tp;
        pair_type = tb.group_type[g];
        pair_ar = (unsigned long long)tb.PR(g, k)[L];
    }
    unsigned int h_bad = 0, h_ovf = 0;
    unsigned long long h_act = 0;
    long long pp = 0, ps = 0;
    if (tid == 0) {
        const BuildHeader *h = tb.header;
        h_bad = h->bad_arg; h_ovf = h->overflow; h_act = h->max_act;
        pp = tb.PP()[L]; ps = tb.PS()[L];
        bad_s = 0; ovf_s = 0; min_bw_s = ~0ull; worst_s = 0; worst32_s = 0;
    }
    __syncthreads();

    unsigned int bad = 0, ovf = 0;
    unsigned long long min_bw = ~0ull;
    for (int64_t e = tid; e < n_links; e += blockDim.x) {
        const int64_t b = e == tid ? bw0 : tb.bw[e];
        if (b < 1) bad = 1;
        else {
            // tp * bandwidth is formed for a group's own link only (the all-reduce time), degrees above 1
            const bool own = e / tb.G == e % tb.G;
            if (own && tb.n_tp > 1 && b > lim.bw_max) ovf = 1;
            if ((unsigned long long)b < min_bw) min_bw = (unsigned long long)b;
        }
    }
    for (int t = tid; t < tb.T; t += blockDim.x) {
        const int64_t m = t == tid ? mem0 : tb.type_mem[t];
        if (m < 0) bad = 1;
        else if (m > lim.mem_max) ovf = 1;
    }
    for (int g = tid; g < tb.G; g += blockDim.x) {
        const int t = g == tid ? type0 : tb.group_type[g];
        const int n = g == tid ? ndev0 : tb.group_ndev[g];
        if (t < 0 || t >= tb.T || n < 1) bad = 1;
    }
    if (bad) atomicOr(&bad_s, 1u);
    if (ovf) atomicOr(&ovf_s, 1u);
    if (min_bw != ~0ull) atomicMin(&min_bw_s, min_bw);

    // first device of every group: exclusive running sum of the group sizes.  Each thread takes a run
    // of consecutive groups; the runs' totals are scanned per wavefront and over the four wavefronts.
    long long mine = 0;
    for (int g = g_begin; g < g_end; ++g) {
        const int n = g == g_begin ? first_ndev : tb.group_ndev[g];
        mine += n > 0 ? n : 0;
    }
    long long upto = mine;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const long long up = __shfl_up(upto, d, 64);
        if (lane >= d) upto += up;
    }
    if (lane == 63) wave_total[wave] = upto;
    __syncthreads();
    const bool groups_ok = (bad_s == 0);
    long long all_devices = 0;
    for (int w = 0; w < 4; ++w) {
        if (w < wave) upto += wave_total[w];
        all_devices += wave_total[w];
    }
    {
        long long base = upto - mine;                               // devices before this thread's run
        for (int g = g_begin; g < g_end; ++g) {
            tb.group_base[g] = (int32_t)(base > INT32_MAX ? 0 : base);
            const int n = g == g_begin ? first_ndev : tb.group_ndev[g];
            base += n > 0 ? n : 0;
        }
        if (tid == 255) {
            // more devices than an int32 numbers: the problem is refused, the bases are not used
            if (all_devices > INT32_MAX) atomicOr(&ovf_s, 1u);
            tb.header->total_devices = all_devices > INT32_MAX ? 0 : all_devices;
        }
    }
    if (groups_ok) {
        long long worst = 0, worst32 = 0;
        for (int q = tid; q < n_pairs; q += blockDim.x) {
            const int g = q / tb.n_tp, k = q - g * tb.n_tp;
            // both totals are below 2^63 unless the build has already noted an overflow
            const unsigned long long work = (unsigned long long)tb.PF(q == tid ? pair_type : tb.group_type[g])[L];
            const unsigned long long ar = q == tid ? pair_ar : (unsigned long long)tb.PR(g, k)[L];
            const unsigned long long whole = work + ar;
            const long long w = whole >= (unsigned long long)kTimeLimit ? kTimeLimit : (long long)whole;
            worst = w > worst ? w : worst;
            const unsigned long long tp = (unsigned long long)tb.tp[k];
            const unsigned long long fused = (ar < (1ull << 40)) ? work + tp * ar + tp - 1 : ~0ull;
            const long long f = fused >= (unsigned long long)kTimeLimit ? kTimeLimit : (long long)fused;
            worst32 = f > worst32 ? f : worst32;
        }
        if (tid < n_pairs) { atomicMax(&worst_s, worst); atomicMax(&worst32_s, worst32); }
    }
    __syncthreads();
    if (tid == 0) {
        BuildHeader *h = tb.header;
        unsigned int bad_all = bad_s | h_bad, ovf_all = ovf_s | h_ovf;
        long long worst = worst_s, cut_worst = 0;
        if (!bad_all) {
            cut_worst = (long long)((h_act + min_bw_s - 1ull) / min_bw_s);
            if (cut_worst > worst) worst = cut_worst;
            if (worst >= kTimeLimit) ovf_all = 1;
            else if (worst > INT64_MAX / (3ll * L + tb.M)) ovf_all = 1;
            // memory need of any segment with any in-flight count
            long long n_max = tb.M < L ? tb.M : L;
            if (ps > (INT64_MAX - pp) / n_max) ovf_all = 1;
        }
        bool pow2 = true;
        for (int k = 0; k < tb.n_tp; ++k) pow2 = pow2 && tb.tp_shift[k] >= 0;
        const long long lim32 = 1ll << 31;
        h->bad_arg = bad_all;
        h->overflow = ovf_all;
        h->worst_time = worst;
        h->fast32 = (!bad_all && !ovf_all && lim.want_fast && pow2 && worst32_s < lim32 && cut_worst < lim32) ? 1u : 0u;
    }
}

// Launch 5: 32-bit rows of the fast path.  Row q < G*n_tp: PF[type g][i] + tp * PR[g][k][i]
// (so that time(j, i) = (row[i] + tp - 1 - row[j]) >> log2 tp); then G*G rows of per-link cut times.
__global__ __launch_bounds__(256) void k1_fast_rows(TablesDev tb) {
    if (tb.header->fast32 == 0) return;
    const int q = blockIdx.y;
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i > tb.L) return;
    const int n_time_rows = tb.G * tb.n_tp;
    if (q < n_time_rows) {
        int g = q / tb.n_tp, k = q - g * tb.n_tp;
        int64_t v = tb.PF(tb.group_type[g])[i] + int64_t(tb.tp[k]) * tb.PR(g, k)[i];
        tb.P32[int64_t(q) * tb.pitch32 + i] = (uint32_t)v;
    } else {
        int e = q - n_time_rows;
        const int64_t link = tb.bw[e];
        int64_t v = (i == 0) ? 0 : ceil_div_inv(tb.act_bytes[i - 1], link, 1.0 / (double)link);
        tb.CM[int64_t(e) * tb.pitch32 + i] = (uint32_t)v;
    }
}

__global__ void k1_clear_header(BuildHeader *h) {
    if (threadIdx.x == 0) {
        h->bad_arg = 0; h->overflow = 0; h->fast32 = 0; h->pad = 0;
        h->max_act = 0; h->worst_time = 0; h->total_devices = 0;
        for (int q = 0; q < 3; ++q) h->reserved[q] = 0;
    }
}

}  // namespace

void launch_build(const TablesDev &tb, const BuildLimits &lim, hipStream_t st) {
    const int n_chunks = (tb.L + kScanChunk - 1) / kScanChunk;
    const int n_rows = tb.n_rows();
    hipLaunchKernelGGL(k1_clear_header, dim3(1), dim3(64), 0, st, tb.header);
    if (tb.L >= kLongL) {
        const int n_runs = (tb.L + kWaveChunk - 1) / kWaveChunk;
        // workgroups walk several runs each (their row constants are staged once), never more of them
        // than half of what covers the sequence with one run per wavefront
        int groups = (n_runs + kScanThreads / 64 - 1) / (kScanThreads / 64);
        if (groups > 512) groups = (groups + 1) / 2;
        const int row_parts = n_rows >= 32 ? 4 : 1;
        const int rows_per_part = (n_rows + row_parts - 1) / row_parts + 1;
        const size_t row_lds = rows_per_part <= kLongRowsInLds ? size_t(rows_per_part) * (sizeof(LongRow) + sizeof(LongRowKey)) : 16;
        hipLaunchKernelGGL(k1_long_sums, dim3(groups, row_parts), dim3(kScanThreads), row_lds, st, tb, lim, n_runs);
        hipLaunchKernelGGL(k1_scan_chunk_sums, dim3(n_rows), dim3(kScanThreads), 0, st, tb, n_runs);
        hipLaunchKernelGGL(k1_long_scan, dim3(groups, row_parts), dim3(kScanThreads), row_lds, st, tb, lim, n_runs);
        hipLaunchKernelGGL(k1_finalize, dim3(1), dim3(256), 0, st, tb, lim);
        return;                   // sequences this long are beyond the 32-bit planner path
    }
    if (n_chunks > 1) {
        hipLaunchKernelGGL(k1_chunk_sums, dim3(n_rows, n_chunks), dim3(kScanThreads), 0, st, tb, lim, n_chunks);
        hipLaunchKernelGGL(k1_scan_chunk_sums, dim3(n_rows), dim3(kScanThreads), 0, st, tb, n_chunks);
    }
    hipLaunchKernelGGL(k1_scan_rows, dim3(n_rows, n_chunks), dim3(kScanThreads), 0, st, tb, lim, n_chunks);
    hipLaunchKernelGGL(k1_finalize, dim3(1), dim3(256), 0, st, tb, lim);
    if (lim.want_fast) {
        const int q = tb.G * tb.n_tp + tb.G * tb.G;
        hipLaunchKernelGGL(k1_fast_rows, dim3((tb.L + 256) / 256, q), dim3(256), 0, st, tb);
    }
}

}  // namespace harp
