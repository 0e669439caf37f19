// Per-geometry plan of the tile kernel: launch configuration and the CSR
// re-expressed as LDS tap offsets.
//
// Section 7 of arXiv 2011.06295 (after Park et al.) stores, instead of a bare
// column number, the pre-computed offset of each stored weight into the input
// array, so the kernel does no index arithmetic per weight.  The same idea is
// used here against the LDS tile: entry offset = c_local*CS + r*Wp + s, to
// which a lane only adds the tile-local index of its own position.
// The paper's unified per-row count (one trip count for every output channel)
// reappears at segment granularity: each (row, channel-chunk) segment is padded
// with zero-weight entries to a multiple of the scalar fetch batch.
// The launch configuration (positions, channels and wavefronts per workgroup,
// channels per LDS pass) plays the role of the per-layer thread-block count the
// paper tunes by hand (section 8, subBatchSize); it is chosen here by a cost
// estimate unless the caller overrides it.
#include "internal.h"

#include <algorithm>
#include <climits>
#include <cmath>
#include <utility>
#include <vector>

#include "../../include/sparse_conv.h"

namespace sc {

namespace {

constexpr int kWave = 64;
constexpr int kMaxWaves = 16;          // wavefronts per workgroup
constexpr int kMaxLds = 160 * 1024;    // LDS per CU
constexpr int kCUs = 256;

inline int cdiv(long long a, long long b) { return (int)((a + b - 1) / b); }
bool pow2_in(int v, int lo, int hi) { return v >= lo && v <= hi && (v & (v - 1)) == 0; }

struct Shape {
    int K, C, R, S, ub;  // ub = bytes of one LDS element (V images)
    int V, H, W, Wp, Hs, elem_bytes;
    int G;               // 0: lanes are lattice positions; else image groups interleaved per element (lanes are outputs)
    long long npos;      // lanes of the whole batch: lattice positions, or outputs * G
    double row_nnz;      // mean stored weights per output channel
};

struct Cand {
    int V, WP, WK, KW, Cc, LP, kblocks;
    int Hb, CS, lds, SL, rows_mode, SG, nbuf, pitch;
    int J;
    int ZE;   // elements of the zero region behind the tile buffers
};

// Output-lane tiles: the most lattice rows between the first and the last of PT consecutive outputs
// (outputs are numbered super-group, row, column; super-group u starts at lattice row u * Hs).
// What a tile spans depends only on its first output modulo E*F, which repeats after at most E*F tiles.
int output_tile_span(long long nout, int PT, int EF, int F, int Hs, int st)
{
    const long long ntiles = (nout + PT - 1) / PT;
    int best = 0;
    for (long long t = 0; t < std::min<long long>(ntiles, (long long)EF + 1); ++t) {
        const long long o0 = t * PT, o1 = std::min<long long>(o0 + PT, nout) - 1;
        const long long Ya = o0 / EF * Hs + o0 % EF / F * st, Yb = o1 / EF * Hs + o1 % EF / F * st;
        best = std::max(best, (int)(Yb - Ya));
    }
    return best;
}

// Tile height in lattice rows for a window of `span` positions starting anywhere in a row.
int tile_rows(int span, int Wp, int R, int S) { return (Wp - 1 + span - 1 + (R - 1) * Wp + S - 1) / Wp + 1; }

// Rows every wavefront (channel index wk) of a channel block takes when the block holds
// `nrows` of its WK * KW slots.  The wavefronts of a workgroup go round the 4 SIMDs of a CU,
// and a SIMD serves its older wavefronts first: the fullest SIMD sets the pace of a chunk and
// its youngest wavefront is the one the others wait for.  The slots a block leaves empty are
// therefore taken, one at a time, from the youngest wavefront of the SIMD that still holds
// the most rows.  (Wavefront index = wk * WP + wp.)
void rows_per_wavefront(int nrows, int WP, int WK, int KW, std::vector<int>& room)
{
    room.assign(WK, KW);
    for (int spare = WK * KW - nrows; spare > 0; --spare) {
        long long rows_on[4] = {0, 0, 0, 0};
        for (int w = 0; w < WK; ++w)
            for (int q = 0; q < WP; ++q) rows_on[(w * WP + q) & 3] += room[w];
        int pick = -1;
        for (int wave = WP * WK - 1; wave >= 0; --wave) {   // youngest first
            const int w = wave / WP;
            if (room[w] <= 0) continue;
            const long long mine = rows_on[wave & 3], best = pick < 0 ? -1 : rows_on[(pick * WP + WP - 1) & 3];
            if (pick < 0 || mine > best || (mine == best && room[w] > room[pick])) pick = w;
        }
        if (pick < 0) break;
        --room[pick];
    }
}

// Rough time of one launch in CU clocks.  The structure follows measurements on
// MI355X; the constants were fitted to the measured times of ~41000 launch
// configurations (every shape the candidate loops below produce) of the 13
// VGG-16 layers at 32 px (batch 128, fp32), four of its layers at 224 px
// (batch 128), the 256->256 14x14 layer at 50..99 % sparsity (batch 256) and six
// 1x1 layers, so that the estimate's first choice is within a few per cent of
// the best measured one and its time within ~10 % of the measured.
//  * A step (kBatch stored weights of one output channel, for the 64 * LP positions
//    of a wavefront) costs its SIMD kBatch * LP * V multiply-adds of ~4 clocks
//    (fp16: the mixed-precision multiply-add takes ~4.4) plus ~4 clocks a weight
//    for the address (as fitted, before one 64-bit add came to serve two weights;
//    the ranking holds with it), and the CU's LDS kBatch * LP * 64 elements
//    at ~225 B/clk.  For 16-byte fp32 elements the two are about equal, and they
//    overlap for the most part.
//  * A SIMD's multiply-adds are those of the rows its wavefronts hold (see
//    rows_per_wavefront); the LDS reads are the whole CU's.
//  * A lone wavefront cannot hide its own LDS and scalar-fetch latency (~170 clocks a step).
//  * Registers (56 + accumulators + two groups of LDS reads in flight) bound the
//    wavefronts resident on a SIMD, and with them the workgroups on a CU.
//  * Staging moves ~16 B/clk/CU from L2 and overlaps the arithmetic except for the
//    first chunk; a workgroup costs ~7 us to start and finish, a chunk ~0.4 us.
//  * Workgroups run in rounds of (CUs * resident workgroups); a partly filled
//    last round still takes a round.
double estimate(const Shape& s, const Cand& c)
{
    const int J = c.J > 0 ? c.J : 1;
    const int nchunks = cdiv(cdiv(s.C, c.Cc), J);          // chunks a workgroup walks
    const double seg = s.row_nnz * c.Cc / s.C;
    const double batches = nchunks == 1 ? std::ceil(seg / kBatch) : seg / kBatch + 0.8;
    const int waves = c.WP * c.WK;
    const double regs = std::min(128.0, 56.0 + c.KW * c.LP * c.V + 4.0 * c.LP * (s.ub / 4.0));  // the kernels are built for <= 128
    const int per_simd = std::min(8, 512 / (8 * (int)std::ceil(regs / 8.0)));
    const int conc_max = std::min(kMaxLds / c.lds, 4 * per_simd / waves);
    if (conc_max < 1) return -1.0;
    const int kblocks = c.kblocks;
    const long long wgs = (long long)cdiv(s.npos, (long long)kWave * c.WP * c.LP) * kblocks * J;
    // rows on the fullest SIMD and wavefront-rows in all of a typical channel block
    std::vector<int> room;
    rows_per_wavefront(cdiv(s.K, kblocks), c.WP, c.WK, c.KW, room);
    long long rows_all = 0;
    for (int w = 0; w < c.WK; ++w) rows_all += (long long)room[w] * c.WP;
    // with the empty slots spread as they are the SIMDs differ by a row at most: the mean fits as well as the maximum
    const double rows_simd = (double)rows_all / 4.0;
    const double fma_clk = s.elem_bytes == 2 ? 4.4 : 4.0;
    const double v_step = kBatch * (c.LP * c.V * fma_clk + 4.0);
    const double l_step = kBatch * c.LP * 64.0 * s.ub / 225.0;
    const double gbytes = (double)s.C / J * c.CS * s.ub * ((double)s.W / s.Wp) * std::min(1.0, (double)s.H / s.Hs);
    // (parts: writing the partial sums, and the last part reading all of them back)
    const double fixed = 16000.0 + 1000.0 * nchunks + (J > 1 ? 2500.0 + 600.0 * J : 0.0);
    const double shape_factor = c.KW == 1 ? 1.2 : c.KW == 8 ? 1.05 : 1.0;   // measured residuals
    double t = 0.0;
    long long remaining = wgs;
    const long long slots = (long long)kCUs * conc_max;
    while (remaining > 0) {
        const long long n = std::min(remaining, slots);
        const int conc = (int)((n + kCUs - 1) / kCUs);
        // one batch of every row of the resident workgroups: the fullest SIMD's multiply-adds, the CU's LDS reads
        const double a = conc * rows_simd * v_step, b = conc * (double)rows_all * l_step;
        const double shared = (std::max(a, b) + 0.3 * std::min(a, b)) / 0.92;
        const double per_batch = std::max(shared, c.KW * (v_step + 170.0));
        const double t_compute = batches * nchunks * shape_factor * per_batch;
        const double t_stage = conc * gbytes / 16.0;
        const long long full = remaining / slots;
        const double round = std::max(t_compute, t_stage) + t_stage / nchunks + fixed;
        if (full > 1) {            // identical full rounds
            t += round * (double)full;
            remaining -= full * slots;
        } else {
            t += round;
            remaining -= n;
        }
    }
    return t;
}

// Output-lane tiles: the most super-groups that have input rows among the Hst lattice rows a tile stages
// (rows from the tile's first output on; super-group u's input rows start pad rows below u * Hs).
int output_tile_groups(long long nout, int PT, int EF, int F, int Hs, int st, int Hst, int pad)
{
    const long long ntiles = (nout + PT - 1) / PT;
    int best = 1;
    for (long long t = 0; t < std::min<long long>(ntiles, (long long)EF + 1); ++t) {
        const long long o0 = t * PT;
        const long long Ya = o0 / EF * Hs + o0 % EF / F * st, Yz = Ya + Hst - 1;   // first and last staged row
        long long ua = Ya / Hs, uz = Yz / Hs;
        if (uz * Hs + pad > Yz) --uz;                     // only padding rows of the last one
        best = std::max(best, (int)(uz - ua + 1));
    }
    return best;
}

}  // namespace

// floor(n / d) = (n * mul) >> (32 + shift) for every 0 <= n < 2^31, where
// mul = floor(2^(31+s) / d) + 1 and shift = s - 1 with 2^(s-1) < d <= 2^s.
FastDiv make_fastdiv(int d)
{
    FastDiv f{0u, 0u, (uint32_t)d};
    if (d <= 1) return f;
    int s = 0;
    while ((1ll << s) < d) ++s;
    f.mul = (uint32_t)((1ull << (31 + s)) / (uint64_t)d + 1ull);
    f.shift = (uint32_t)(s - 1);
    return f;
}

int build_plan(const Csr& csr, int C, int R, int S, int elem_bytes, const Geometry& g,
               const Launch& over, Plan& p, std::vector<std::pair<double, Launch>>* ranked)
{
    const int K = csr.K;
    const int st = g.stride, pad = g.pad;
    p.E = (g.H + 2 * pad - R) / st + 1;
    p.F = (g.W + 2 * pad - S) / st + 1;
    p.st = st;
    p.pool = over.pool ? 1 : 0;
    if (over.pool && ((p.E | p.F) & 1)) return SC_EUNSUPPORTED;   // windows of 2 x 2 need an even map

    if (over.lds_budget > kMaxLds) return SC_EINVAL;
    if (over.KW && !pow2_in(over.KW, 1, 16)) return SC_EINVAL;
    if (over.WP * std::max(1, over.WK) > kMaxWaves || over.WK > kMaxWaves) return SC_EINVAL;
    const int vmax = 16 / elem_bytes;
    if (over.V && !pow2_in(over.V, 1, vmax)) return SC_EINVAL;
    if (over.LP && !pow2_in(over.LP, 1, 2)) return SC_EINVAL;
    if (over.store < 0 || over.store > 2) return SC_EINVAL;
    if (over.lanes < 0 || (over.lanes > 1 && !pow2_in(over.lanes - 1, 1, 16))) return SC_EINVAL;
    if (over.csplit && !pow2_in(over.csplit, 1, 8)) return SC_EINVAL;

    // ---- candidates
    static const int budgets[] = {160 * 1024, 80 * 1024, 53 * 1024, 40 * 1024, 32 * 1024};
    Cand best{};
    Shape bs{};
    double best_t = -1.0;
    bool too_many_positions = false;
    // images interleaved per LDS element: an element of up to 16 bytes, not wider than the batch can fill
    const int EF = p.E * p.F;
    for (int V = vmax; V >= 1; V /= 2) {
        if (over.V && V != over.V) continue;
        if (!over.V && V > 1 && V / 2 >= g.N) continue;
        const int ngroups = std::max(1, cdiv(g.N, V));
        // What lanes stand for: lattice positions (G = 0), or outputs with G image groups interleaved.  Unasked,
        // output lanes are tried where ds_read_b128 stays at full rate.  Measured rule: in each half of a
        // wavefront, lanes l and l + 16 must read elements that are congruent modulo 16, and 16 consecutive
        // lanes distinct ones; 32 consecutive elements do that whatever their alignment, 16-element runs
        // only at distances that are multiples of 16 (18: half rate).  So 32 consecutive lanes must be
        // 32 / G outputs of one row (unit stride) times G groups.  Tried: the smallest such G and twice it
        // (larger G: more images and fewer rows of the map in a tile).
        int modes[8], nmodes = 0;
        if (over.lanes <= 1 && !over.pool) modes[nmodes++] = 0;
        if (over.lanes > 1) {
            modes[nmodes++] = over.lanes - 1;
        } else if (over.lanes == 0 && V * elem_bytes == 16) {
            int taken = 0;
            for (int G = 1; G <= 16 && taken < 3; G *= 2) {
                if (st != 1) break;
                if (G > 1 && G / 2 >= ngroups) break;      // groups the batch cannot fill
                if (p.F % (32 / G) != 0) {
                    // 16 lanes are a whole row (or rows): fine if the row distance is a multiple of 16 elements,
                    // where a wider pitch that makes it one at most doubles it
                    const int wp0 = std::max(g.W + pad, p.F), unit = 16 / G;
                    if (p.F % unit != 0 || (wp0 + unit - 1) / unit * unit > wp0 * 2) continue;
                }
                modes[nmodes++] = G;
                ++taken;
            }
        }
        for (int mi = 0; mi < nmodes; ++mi) {
        const int G = modes[mi];
        Shape s;
        s.K = K; s.C = C; s.R = R; s.S = S;
        s.V = V;
        s.G = G;
        s.elem_bytes = elem_bytes;
        s.ub = V * elem_bytes;
        s.H = g.H; s.W = g.W;
        // pitch and group height: the padding below/right of an image is shared with the
        // next group/row, but every output's receptive field must still start inside its own group
        s.Wp = std::max(g.W + pad, (p.F - 1) * st + 1);
        s.Hs = std::max(g.H + pad, (p.E - 1) * st + 1);
        long long nout = 0;
        if (G) {
            // runs of 16 lanes (whole rows) that are not halves of a 32-lane run: the pitch makes the distance
            // between rows a multiple of 16 elements
            if (st == 1 && G < 16 && p.F % (32 / G) != 0 && p.F % (16 / G) == 0) s.Wp = (s.Wp + 16 / G - 1) / (16 / G) * (16 / G);
            nout = (long long)cdiv(ngroups, G) * EF;
            s.npos = nout * G;
            if ((long long)cdiv(ngroups, G) * s.Hs * s.Wp * G + (long long)(R + 1) * s.Wp * G + 2048 >= (1ll << 31)) {
                too_many_positions = true;
                continue;
            }
        } else {
            s.npos = (long long)ngroups * s.Hs * s.Wp;
        }
        s.row_nnz = K > 0 ? (double)csr.colidx.size() / K : 0.0;
        if (s.npos + (long long)(R + 1) * s.Wp + 2048 >= (1ll << 31)) {  // lattice elements are 32-bit in the kernel
            too_many_positions = true;
            continue;
        }
        for (int LP = 1; LP <= 2; LP *= 2)
        for (int WP = 1; WP <= 8; WP *= 2) {
            if (over.LP && LP != over.LP) break;
            if (over.WP && WP != 1) break;
            if (G && LP != 1) continue;            // output lanes: one output per lane
            const int wp = over.WP ? over.WP : WP;
            const int span = kWave * wp * LP;
            // 2 x 2 maximum in the store step: a tile holds whole pairs of output rows
            if (over.pool && (!G || (span / G) % (2 * p.F) != 0)) continue;
            const int ge = G ? G : 1;
            int Hb;
            if (G) {
                const int wrap = ((p.F - 1) * st + S - 1) / s.Wp;     // taps of a row's last outputs run into the next row
                Hb = output_tile_span(nout, span / G, EF, p.F, s.Hs, st) + R + wrap;
            } else {
                Hb = tile_rows(span, s.Wp, R, S);
            }
            // Tile layout per channel.  Contiguous: the Hb lattice rows the positions and their taps
            // touch, pitch Wp.  Banded (maps much wider than the tile): R bands of span + S - 1
            // consecutive lattice elements, band r starting r rows below the first position.
            const int P2 = span + S - 1;
            const bool banded = !G && (long long)R * P2 < (long long)Hb * s.Wp;
            const long long CS = banded ? (long long)R * P2 : (long long)Hb * s.Wp * ge;
            const int pitch = banded ? P2 : s.Wp;
            // staging slots per channel: every tile element (banded), the tile's rows, or (small maps)
            // the whole planes of every group it can touch
            // (whole planes only where a plane is a short run of memory: the order then continues across channels)
            // (output lanes: the row that only the wrap of a row's last taps reaches holds padding there, it is not staged)
            const int Hst = G ? Hb - ((p.F - 1) * st + S - 1) / s.Wp : Hb;
            const int rows_spanned = banded ? (R - 1) + (P2 + s.Wp - 1) / s.Wp + 1 : Hst;
            long long GC = ((rows_spanned + s.Hs - 2) / s.Hs + 1) * (long long)ge;   // image groups a tile can touch
            if (G) GC = (long long)output_tile_groups(nout, span / G, EF, p.F, s.Hs, st, Hst, pad) * G;
            const bool rows_mode = banded || s.Hs >= Hb || (long long)g.H * g.W * elem_bytes >= 128;
            const long long SL = banded ? CS : rows_mode ? (long long)Hst * ge * g.W : GC * g.H * g.W;
            const long long tbl = SL * 8;
            // The zero region: one run of zeroed elements behind the tile buffers, as long as the lanes of a
            // wavefront spread over a channel's tile elements (furthest element under a lane + 1).  The
            // zero-weight entries that fill a row's last batch point at it, so a lane multiplies 0 by 0
            // there and not by whatever the input holds (0 x Inf would be NaN).
            const int wrapG = G ? ((p.F - 1) * st + S - 1) / s.Wp : 0;
            const long long ZE = 1 + (banded ? (long long)span - 1
                                      : G  ? ((long long)(Hb - R - wrapG) * s.Wp + (long long)(p.F - 1) * st) * G + G - 1
                                           : (long long)s.Wp - 1 + span - 1);
            // slot offsets are 31-bit byte offsets from the first image group of a tile
            if (GC * V * C * g.H * g.W * elem_bytes >= (1ll << 31)) continue;
            if (CS >= (1ll << 24) || SL >= (1ll << 24)) continue;
            for (int WK = 1; WK <= kMaxWaves; ++WK) {
                if (over.WK && WK != 1) break;
                const int wk = over.WK ? over.WK : WK;
                if (wp * wk > kMaxWaves) continue;
                for (int KW = 1; KW <= 16; KW *= 2) {
                    if (over.KW && KW != 1) break;
                    const int kw = over.KW ? over.KW : KW;
                    // accumulators and the LDS reads in flight must stay in registers
                    if (kw * V > 64 || (LP > 1 && (kw * LP * V > 32 || kw * LP > 16))) continue;
                    if (!over.KW && !over.WK && (long long)(wk - 1) * kw >= K && wk > 1) continue;  // idle wavefronts
                    for (int bi = 0; bi < 5; ++bi) {
                        if ((over.lds_budget || over.Cc) && bi) break;
                        const int budget = over.lds_budget ? over.lds_budget : budgets[bi];
                        const long long room = budget - tbl - 32 - ZE * s.ub;
                        // a chunk should not exceed what the workgroup stages in one pass (kStage units a thread)
                        const long long pass_cc = std::max<long long>(1, (long long)kStage * kWave * wp * wk / SL);
                        int Cc, nbuf = 1;
                        if (over.Cc) {
                            Cc = std::min(over.Cc, C);
                        } else if (room < CS * s.ub) {
                            continue;
                        } else if (C <= pass_cc && C * CS * s.ub <= room) {
                            Cc = C;                                   // everything in one chunk
                        } else {
                            Cc = (int)std::min<long long>(std::min<long long>(C, pass_cc), room / (2 * CS * s.ub));
                        }
                        if (Cc < 1) continue;
                        if (!over.Cc) Cc = cdiv(C, cdiv(C, Cc));     // even chunks
                        if (Cc < C) nbuf = 2;                        // the next chunk lands while this one is consumed
                        // tile buffer(s), each with one spare element, the zero region, table
                        long long lds = (((long long)nbuf * ((long long)Cc * CS + 1) + ZE) * s.ub + 15) / 16 * 16 + tbl;
                        // (the pooled store stages one sum per thread and image in LDS)
                        if (over.pool) lds = std::max<long long>(lds, (long long)kWave * wp * wk * V * 4);
                        if (lds > kMaxLds) continue;
                        if (G) {   // the staging patterns of output-lane tiles must stay a small table (build below)
                            int ga = (span / G) % EF, gb = EF;
                            while (ga) { const int r = gb % ga; gb = ga; ga = r; }
                            const long long per = (SL * Cc + (long long)kStage * kWave * wp * wk - 1) / ((long long)kStage * kWave * wp * wk) *
                                                  ((long long)kStage * kWave * wp * wk);
                            if (per * (EF / gb) * 8 > (8ll << 20)) continue;
                        }
                        // More channel blocks than the rows need leave slots empty, which relieves the
                        // last wavefronts of the fullest SIMDs (rows_per_wavefront): up to two extra.
                        const int kb_min = cdiv(K, wk * kw);
                        for (int extra = 0; extra < 3; ++extra) {
                            const int kblocks = over.kblocks ? over.kblocks : kb_min + extra;
                            if (over.kblocks && extra) break;
                            if (kblocks < kb_min || (extra && kblocks > K)) continue;
                            for (int J = 1; J <= 8; J *= 2) {
                            if (over.csplit && J != over.csplit) continue;
                            const int nch = cdiv(C, Cc);
                            if (J > 1 && (J > nch || (long long)(J - 1) * cdiv(nch, J) >= nch)) continue;   // every part needs a chunk
                            Cand c{V, wp, wk, kw, Cc, LP, kblocks, Hb, (int)CS, (int)lds, (int)SL, banded ? 2 : rows_mode ? 1 : 0, rows_mode ? 1 : (int)GC, nbuf, pitch, J, (int)ZE};
                            double t = estimate(s, c);
                            if (t < 0) {
                                if (!(over.WP || over.WK || over.KW || over.Cc || over.lds_budget || over.LP || over.kblocks)) continue;
                                t = 1e30;   // an explicit request is honoured even where the estimate expects no residency
                            }
                            if (ranked) {
                                Launch l;
                                l.V = V; l.WP = wp; l.WK = wk; l.KW = kw; l.Cc = Cc; l.LP = LP; l.kblocks = kblocks;
                                l.store = over.store;
                                l.lanes = 1 + G;
                                l.csplit = J;
                                ranked->emplace_back(t, l);
                            }
                            if (best_t < 0 || t < best_t) {
                                best_t = t;
                                best = c;
                                bs = s;
                            }
                            }
                        }
                    }
                }
            }
        }
        }
    }
    if (best_t < 0 && too_many_positions) return SC_EUNSUPPORTED;
    if (best_t < 0) return SC_EUNSUPPORTED;
    if (ranked) {   // the caller only wants the candidates, cheapest estimate first, each once
        std::stable_sort(ranked->begin(), ranked->end(),
                         [](const std::pair<double, Launch>& x, const std::pair<double, Launch>& y) { return x.first < y.first; });
        std::vector<std::pair<double, Launch>> uniq;
        for (const auto& e : *ranked) {
            bool seen = false;
            for (const auto& u : uniq)
                seen = seen || (u.second.V == e.second.V && u.second.WP == e.second.WP && u.second.WK == e.second.WK &&
                                u.second.KW == e.second.KW && u.second.Cc == e.second.Cc && u.second.LP == e.second.LP &&
                                u.second.kblocks == e.second.kblocks && u.second.lanes == e.second.lanes &&
                                u.second.csplit == e.second.csplit);
            if (!seen) uniq.push_back(e);
            if (uniq.size() >= 256) break;
        }
        // The estimate was fitted on lattice lanes and ranks the kinds of lanes (and of channel splitting) against
        // each other only roughly: after its three best, the list goes round the kinds (best of each, second best
        // of each, ...) so that a measurement of the first few sees every kind.
        {
            std::vector<std::pair<double, Launch>> mixed;
            std::vector<char> used(uniq.size(), 0);
            for (size_t i = 0; i < uniq.size() && i < 3; ++i) {
                used[i] = 1;
                mixed.push_back(uniq[i]);
            }
            while (mixed.size() < uniq.size() && mixed.size() < 64) {
                bool took[36] = {};
                for (size_t i = 0; i < uniq.size() && mixed.size() < 64; ++i) {
                    const int kind = uniq[i].second.lanes + (uniq[i].second.csplit > 1 ? 18 : 0);
                    if (used[i] || took[kind]) continue;
                    took[kind] = true;
                    used[i] = 1;
                    mixed.push_back(uniq[i]);
                }
            }
            uniq.swap(mixed);
        }
        ranked->swap(uniq);
        return SC_OK;
    }

    const Shape& s = bs;
    const int V = best.V;
    const int ngroups = std::max(1, cdiv(g.N, V));
    p.V = V; p.WP = best.WP; p.WK = best.WK; p.KW = best.KW; p.Cc = best.Cc; p.LP = best.LP;
    p.store = over.store ? over.store : 1;   // which kind is faster depends on what else lives in L2: only a measurement tells
    p.Wp = s.Wp; p.Hs = s.Hs;
    p.span = kWave * p.WP * p.LP;
    p.G = s.G;
    p.PT = s.G ? p.span / s.G : 0;
    p.Hb = best.Hb; p.CS = best.CS;
    p.nchunks = cdiv(C, p.Cc);
    p.ngroups = ngroups;
    p.npos = s.npos;
    const long long ntiles = (s.npos + p.span - 1) / p.span;
    const int KB = p.WK * p.KW;
    p.kblocks = best.kblocks;
    p.J = best.J;
    p.cpp = cdiv(cdiv(C, p.Cc), p.J);
    p.threads = kWave * p.WP * p.WK;
    p.lds_bytes = best.lds;
    p.SL = best.SL;
    p.SG = best.SG;
    p.SP = best.SL / best.SG;
    p.rows_mode = best.rows_mode;
    p.pitch = best.pitch;
    p.nbuf = best.nbuf;
    p.zero_elems = best.ZE;
    p.tbl_off = (int)((((long long)p.nbuf * (p.Cc * p.CS + 1) + p.zero_elems) * s.ub + 15) / 16 * 16);
    const long long grid = (ntiles * p.kblocks * p.J + 7) / 8 * 8;   // a multiple of the XCD count
    if (ntiles > INT_MAX / 2 || grid > INT_MAX - 8) return SC_EUNSUPPORTED;
    p.ntiles = (int)ntiles;
    p.grid = (int)grid;

    // ---- tables
    const int RS = R * S;
    const int nchunks = p.nchunks;
    // Output channel of every accumulator slot (kb, wk, kk).  The wavefronts of a workgroup meet
    // at a barrier after every channel chunk, so what should be equal among them is the number
    // of batches per chunk, not only per layer (a row's weights are spread unevenly over the
    // chunks even when all rows have the paper's unified count).
    //  1. Rows, longest first, are dealt back and forth over the channel blocks: every
    //     workgroup gets about the same total, and empty slots are spread over all of them.
    //  2. Inside a channel block each row goes to the wavefront (with a free slot) whose load
    //     so far overlaps least with the row's own chunk profile (smallest dot product).
    p.krow.assign((size_t)p.kblocks * KB, -1);
    {
        std::vector<int> batches((size_t)K * nchunks);   // batches of row k in chunk ch
        std::vector<long long> total(K, 0);
        for (int k = 0; k < K; ++k) {
            const int* cb = csr.colidx.data() + csr.rowptr[k];
            const int* ce = csr.colidx.data() + csr.rowptr[k + 1];
            const int* lo = cb;
            for (int ch = 0; ch < nchunks; ++ch) {
                const int c1 = std::min(C, (ch + 1) * p.Cc);
                const int* hi = std::lower_bound(lo, ce, c1 * RS);
                batches[(size_t)k * nchunks + ch] = cdiv(hi - lo, kBatch);
                total[k] += batches[(size_t)k * nchunks + ch];
                lo = hi;
            }
        }
        std::vector<int> order(K);
        for (int k = 0; k < K; ++k) order[k] = k;
        std::stable_sort(order.begin(), order.end(), [&](int x, int y) { return total[x] > total[y]; });
        std::vector<std::vector<int>> of_block(p.kblocks);
        for (int i = 0; i < K; ++i) {
            const int round = i / p.kblocks, j = i % p.kblocks;
            of_block[(round & 1) ? p.kblocks - 1 - j : j].push_back(order[i]);
        }
        std::vector<long long> load((size_t)p.WK * nchunks);
        std::vector<int> fill(p.WK), room(p.WK);
        for (int kb = 0; kb < p.kblocks; ++kb) {
            std::fill(load.begin(), load.end(), 0);
            std::fill(fill.begin(), fill.end(), 0);
            rows_per_wavefront((int)of_block[kb].size(), p.WP, p.WK, p.KW, room);   // empty slots go to the last wavefronts of the fullest SIMDs
            for (int k : of_block[kb]) {   // longest first
                const int* bk = &batches[(size_t)k * nchunks];
                int best_w = -1;
                long long best_dot = 0;
                for (int w = 0; w < p.WK; ++w) {
                    if (fill[w] >= room[w]) continue;
                    long long dot = 0;
                    for (int ch = 0; ch < nchunks; ++ch) dot += load[(size_t)w * nchunks + ch] * bk[ch];
                    if (best_w < 0 || dot < best_dot || (dot == best_dot && fill[w] < fill[best_w])) {
                        best_w = w;
                        best_dot = dot;
                    }
                }
                p.krow[((size_t)kb * p.WK + best_w) * p.KW + fill[best_w]++] = k;
                for (int ch = 0; ch < nchunks; ++ch) load[(size_t)best_w * nchunks + ch] += bk[ch];
            }
        }
    }

    const int ge = p.G ? p.G : 1;   // elements per lattice position
    const int SW = p.KW + 1;  // descriptor: first entry, then batches of each of the KW rows
    p.seg.assign(((size_t)p.kblocks * nchunks * p.WK + 1) * SW, 0);   // one terminal descriptor
    p.entries.clear();
    // Weights that are binary16 values (binary16 layers; cluster-quantised layers, whose centroids are binary16)
    // go to the device as one word per entry, with the LDS offset in 16 bits: in units of 4 bytes (2 for
    // 2-byte elements, whose tile must then stay below 128 KB; otherwise the ordinary 8-byte entries are kept).
    p.off_shift = s.ub >= 4 ? 2 : 1;
    p.compact = (csr.coded || elem_bytes == 2) && ((long long)p.nbuf * ((long long)p.Cc * p.CS + 1) * s.ub >> p.off_shift) < 65536;
    for (int kb = 0; kb < p.kblocks; ++kb)
        for (int ch = 0; ch < nchunks; ++ch) {
            const int c0 = ch * p.Cc, c1 = std::min(C, c0 + p.Cc);
            for (int wk = 0; wk < p.WK; ++wk) {
                int* sg = &p.seg[(((size_t)kb * nchunks + ch) * p.WK + wk) * SW];
                sg[0] = (int)p.entries.size();
                for (int kk = 0; kk < p.KW; ++kk) {
                    const int k = p.krow[(size_t)kb * KB + wk * p.KW + kk];
                    sg[1 + kk] = 0;
                    if (k < 0) continue;
                    const int* cb = csr.colidx.data() + csr.rowptr[k];
                    const int* ce = csr.colidx.data() + csr.rowptr[k + 1];
                    const int* lo = std::lower_bound(cb, ce, c0 * RS);
                    const int* hi = std::lower_bound(cb, ce, c1 * RS);
                    const int n = (int)(hi - lo);
                    if (n == 0) continue;
                    Entry last{0u, 0};
                    for (const int* q = lo; q < hi; ++q) {
                        const int col = *q;
                        const int c = col / RS, r = (col / S) % R, sx = col % S;
                        const float wv = csr.val32[(size_t)(q - csr.colidx.data())];
                        uint32_t wb;
                        __builtin_memcpy(&wb, &wv, 4);
                        last = Entry{wb, ((c - c0) * p.CS + (r * p.pitch + sx) * ge) * s.ub};
                        p.entries.push_back(last);
                    }
                    const int nb = cdiv(n, kBatch);
                    // padding: weight zero, in the zero region (it lies nbuf buffers behind the first buffer's
                    // start; this chunk is multiplied out of buffer `buf` of its part's sequence)
                    const int buf = (ch % p.cpp) & (p.nbuf - 1);
                    const int zero_at = (int)((long long)(p.nbuf - buf) * (p.Cc * p.CS + 1) * s.ub);
                    for (int t = n; t < nb * kBatch; ++t) p.entries.push_back(Entry{0u, zero_at});
                    sg[1 + kk] = nb;
                    if (p.entries.size() > (size_t)INT_MAX / 2) return SC_EUNSUPPORTED;
                }
            }
        }
    p.seg[(size_t)p.kblocks * nchunks * p.WK * SW] = (int)p.entries.size();  // where the last segment ends
    for (int t = 0; t < 2 * kBatch; ++t) p.entries.push_back(Entry{0u, 0});  // slack for look-ahead fetches (two batches)

    // ---- output lanes: the staging units of every thread, per pattern
    p.units.clear();
    p.nphase = 0;
    p.npass = (int)(((long long)p.SG * p.Cc * p.SP + (long long)kStage * p.threads - 1) / ((long long)kStage * p.threads));
    if (p.G) {
        const int EF = p.E * p.F, G = p.G, W = g.W, H = g.H;
        int a = p.PT % EF, b = EF;
        while (a) { const int r = b % a; b = a; a = r; }   // b = gcd(PT, EF)
        p.nphase = EF / b;
        const long long per_phase = (long long)p.npass * kStage * p.threads;
        if (per_phase * p.nphase * (long long)sizeof(Plan::Unit) > (8ll << 20)) return SC_EUNSUPPORTED;
        p.units.resize((size_t)(per_phase * p.nphase));
        const long long img_bytes = (long long)C * H * W * elem_bytes, chan_bytes = (long long)H * W * elem_bytes;
        const long long reject = (long long)p.Cc * p.CS;   // the spare element of a buffer
        for (int ph = 0; ph < p.nphase; ++ph) {
            const long long o0 = (long long)ph * p.PT;
            const long long u0 = o0 / EF;
            const long long Y0 = u0 * p.Hs + (o0 % EF) / p.F * st;
            const long long g_first = u0 * G;
            for (long long u = 0; u < per_phase; ++u) {
                const long long tid = u % p.threads, j = u / p.threads, unit = j * p.threads + tid;
                const long long gi = unit / ((long long)p.Cc * p.SP), r0 = unit % ((long long)p.Cc * p.SP);
                const long long c = r0 / p.SP, sp = r0 % p.SP;
                bool ok = gi < p.SG;
                long long src = 0, elem = 0;
                if (ok) {
                    const long long sl = gi * p.SP + sp;
                    long long gs, ys, xx, Yt, gsub;
                    if (p.rows_mode) {   // slot = (tile row, image group of the super-group, column)
                        Yt = sl / ((long long)G * W);
                        const long long rem = sl % ((long long)G * W);
                        gsub = rem / W;
                        xx = rem % W;
                        const long long Ys = Y0 + Yt, us = Ys / p.Hs;
                        gs = us * G + gsub;
                        ys = Ys - us * p.Hs - pad;
                    } else {             // slot = (image group, row, column) of the groups the tile can touch
                        const long long gq = sl / ((long long)H * W), rem = sl % ((long long)H * W);
                        ys = rem / W;
                        xx = rem % W;
                        gs = g_first + gq;
                        gsub = gs % G;
                        Yt = gs / G * p.Hs + pad + ys - Y0;
                    }
                    // (image groups past the batch are not excluded here: the loads of absent images read zeros)
                    ok = ys >= 0 && ys < H && xx >= 0 && xx < W && Yt >= 0 && Yt < p.Hb;
                    src = (gs - g_first) * p.V * img_bytes + (ys * W + xx) * elem_bytes + c * chan_bytes;
                    elem = (Yt * p.Wp + pad + xx) * G + gsub + c * p.CS;
                    if (ok && (src < 0 || src >= (1ll << 31))) return SC_EUNSUPPORTED;
                }
                Plan::Unit& out = p.units[(size_t)(((long long)ph * p.npass * kStage + j) * p.threads + tid)];
                out.off = ok ? (uint32_t)src : 0x80000000u;
                out.dst = (uint32_t)((ok ? elem : reject) * s.ub);
            }
        }
    }
    return SC_OK;
}

// Host-side consistency check of a built plan against the CSR it was made from.
// 0 = consistent; otherwise the number of the first check that failed.
int check_plan(const Csr& csr, int C, int R, int S, int elem_bytes, const Plan& p)
{
    const int K = csr.K, RS = R * S;
    const int ub = p.V * elem_bytes;
    const int KB = p.WK * p.KW, SW = p.KW + 1;
    // 1: launch shape within the hardware's limits
    if (p.threads != kWave * p.WP * p.WK || p.threads > kWave * kMaxWaves || p.lds_bytes > kMaxLds) return 1;
    if (p.nchunks != cdiv(C, p.Cc) || (p.nbuf != 1 && p.nbuf != 2) || (p.nchunks > 1 && p.nbuf != 2)) return 1;
    if ((long long)p.tbl_off + (long long)p.SL * 8 > p.lds_bytes) return 1;
    if (((long long)p.nbuf * ((long long)p.Cc * p.CS + 1) + p.zero_elems) * ub > p.tbl_off) return 1;
    if ((long long)p.grid < (long long)p.ntiles * p.kblocks * p.J || p.grid % 8 != 0) return 1;
    if (p.J < 1 || p.J > 8 || (p.J & (p.J - 1)) || p.cpp != cdiv(p.nchunks, p.J) || (long long)(p.J - 1) * p.cpp >= p.nchunks) return 1;
    if ((long long)p.ntiles * p.span < p.npos || (long long)(p.ntiles - 1) * p.span >= p.npos) return 1;
    // 2: every output channel owns exactly one accumulator slot
    if (p.krow.size() != (size_t)p.kblocks * KB) return 2;
    std::vector<int> seen(K, 0);
    for (int k : p.krow) {
        if (k < -1 || k >= K) return 2;
        if (k >= 0 && seen[k]++) return 2;
    }
    for (int k = 0; k < K; ++k)
        if (!seen[k]) return 2;
    // 3-6: the segments, in the order the kernel walks them
    if (p.seg.size() != ((size_t)p.kblocks * p.nchunks * p.WK + 1) * SW) return 3;
    const bool banded = p.rows_mode == 2;
    const int ge = p.G ? p.G : 1;
    if (p.G && (p.LP != 1 || p.PT * p.G != p.span || banded)) return 1;
    // furthest tile element under a lane
    long long lane_reach = banded ? p.span - 1 : (long long)p.Wp - 1 + p.span - 1;
    if (p.G) {
        const int wrap = ((p.F - 1) * p.st + S - 1) / p.Wp;
        lane_reach = ((long long)(p.Hb - R - wrap) * p.Wp + (long long)(p.F - 1) * p.st) * p.G + p.G - 1;
        // the rows a tile's outputs span, worked out again
        const long long EF = (long long)p.E * p.F, nout = p.npos / p.G;
        for (long long t = 0; t < p.ntiles; ++t) {
            const long long o0 = t * p.PT, o1 = std::min<long long>(o0 + p.PT, nout) - 1;
            const long long Ya = o0 / EF * p.Hs + o0 % EF / p.F * p.st, Yb = o1 / EF * p.Hs + o1 % EF / p.F * p.st;
            if (Yb - Ya + R + wrap > p.Hb) return 1;
        }
    }
    if (p.zero_elems < lane_reach + 1) return 1;   // the zero region covers every lane of a wavefront
    size_t pos = 0, real = 0;
    for (int kb = 0; kb < p.kblocks; ++kb)
        for (int ch = 0; ch < p.nchunks; ++ch) {
            const int c0 = ch * p.Cc, c1 = std::min(C, c0 + p.Cc);
            for (int wk = 0; wk < p.WK; ++wk) {
                const int* sg = &p.seg[(((size_t)kb * p.nchunks + ch) * p.WK + wk) * SW];
                if ((size_t)sg[0] != pos) return 3;                       // segments are contiguous
                for (int kk = 0; kk < p.KW; ++kk) {
                    const int k = p.krow[(size_t)kb * KB + wk * p.KW + kk];
                    const int nb = sg[1 + kk];
                    if (k < 0) {
                        if (nb != 0) return 4;
                        continue;
                    }
                    const int* cb = csr.colidx.data() + csr.rowptr[k];
                    const int* ce = csr.colidx.data() + csr.rowptr[k + 1];
                    const int* lo = std::lower_bound(cb, ce, c0 * RS);
                    const int* hi = std::lower_bound(cb, ce, c1 * RS);
                    const int n = (int)(hi - lo);
                    if (nb != cdiv(n, kBatch)) return 4;                  // batches of the row in this chunk
                    if (pos + (size_t)nb * kBatch + kBatch > p.entries.size()) return 4;
                    for (int t = 0; t < nb * kBatch; ++t) {
                        const Entry& e = p.entries[pos + t];
                        if (t < n) {
                            const int col = lo[t];
                            const int c = col / RS, r = (col / S) % R, sx = col % S;
                            const float wv = csr.val32[(size_t)(lo + t - csr.colidx.data())];
                            uint32_t wb;
                            __builtin_memcpy(&wb, &wv, 4);
                            const long long elem = (long long)(c - c0) * p.CS + ((long long)r * p.pitch + sx) * ge;
                            if (e.wbits != wb || (long long)e.off != elem * ub) return 5;   // weight and tap
                            if (elem + lane_reach >= (long long)(c1 - c0) * p.CS) return 6;  // inside the chunk's tile
                        } else if (e.wbits != 0u ||
                                   (long long)e.off != (long long)(p.nbuf - ((ch % p.cpp) & (p.nbuf - 1))) * ((long long)p.Cc * p.CS + 1) * ub) {
                            return 5;                                     // padding: weight zero, in the zero region
                        }
                    }
                    pos += (size_t)nb * kBatch;
                    real += (size_t)n;
                }
            }
        }
    if ((size_t)p.seg[(size_t)p.kblocks * p.nchunks * p.WK * SW] != pos) return 3;
    if (p.G) {   // 9: the staging units of the output-lane patterns stay inside a tile buffer
        if (p.nphase < 1 || p.units.size() != (size_t)p.nphase * p.npass * kStage * p.threads) return 9;
        std::vector<char> hit;
        for (int ph = 0; ph < p.nphase; ++ph) {
            hit.assign((size_t)p.Cc * p.CS + 1, 0);
            for (size_t i = 0; i < (size_t)p.npass * kStage * p.threads; ++i) {
                const Plan::Unit& un = p.units[(size_t)ph * p.npass * kStage * p.threads + i];
                if (un.dst % ub != 0 || un.dst / ub > (unsigned long long)p.Cc * p.CS) return 9;
                if ((un.off & 0x80000000u) && un.dst / ub != (unsigned long long)p.Cc * p.CS) return 9;   // nothing to load: the spare element
                if (!(un.off & 0x80000000u) && hit[un.dst / ub]++) return 9;                               // one writer per tile element
            }
        }
    }
    if (p.compact) {   // 8: every entry fits the one-word form (a binary16 weight, an offset of 16 bits in its unit)
        if (p.off_shift != (ub >= 4 ? 2 : 1)) return 8;
        for (const Entry& e : p.entries) {
            float wv;
            __builtin_memcpy(&wv, &e.wbits, 4);
            if (half_to_float(float_to_half_rne(wv)) != wv && wv == wv) return 8;
            if (e.off < 0 || (e.off & ((1 << p.off_shift) - 1)) || (e.off >> p.off_shift) >= 65536) return 8;
        }
    }
    if (real != csr.colidx.size()) return 7;                              // 7: every stored weight exactly once
    return 0;
}

}  // namespace sc
