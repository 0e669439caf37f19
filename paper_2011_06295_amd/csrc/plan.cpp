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

#include "../../include/sparse_conv.h"

namespace sc {

namespace {

constexpr int kWave = 64;
constexpr int kMaxWaves = 16;          // wavefronts per workgroup
constexpr int kMaxLds = 160 * 1024;    // LDS per CU
constexpr int kCUs = 256;
constexpr int kCUWaves = 32;           // resident wavefronts per CU at <= 64 VGPRs

inline int cdiv(long long a, long long b) { return (int)((a + b - 1) / b); }
bool pow2_in(int v, int lo, int hi) { return v >= lo && v <= hi && (v & (v - 1)) == 0; }

struct Shape {
    int K, C, R, S, ub;  // ub = bytes of one LDS element (V images)
    int V, W, Wp, Hs;
    long long npos;
    double row_nnz;      // mean stored weights per output channel
};

struct Cand {
    int WP, WK, KW, Cc;
    int Hb, CS, lds;
};

// Tile height in lattice rows for a window of `span` positions starting anywhere in a row.
int tile_rows(int span, int Wp, int R, int S) { return (Wp - 1 + span - 1 + (R - 1) * Wp + S - 1) / Wp + 1; }

// Rough time of one launch in CU clocks.  The constants come from
// micro-benchmarks on MI355X: a 16-byte LDS read of a wavefront occupies the
// LDS for about 4.6 clocks once >= 16 wavefronts are resident; a wavefront's
// VALU instruction takes ~2.4 clocks; global->LDS staging sustains ~48 B/clk/CU.
double estimate(const Shape& s, const Cand& c)
{
    const int nchunks = cdiv(s.C, c.Cc);
    const double seg = s.row_nnz * c.Cc / s.C;
    const double padded = nchunks == 1 ? std::ceil(seg / kBatch) * kBatch : seg + 0.5 * (kBatch - 1);
    const int waves = c.WP * c.WK;
    const long long wgs = (long long)cdiv(s.npos, (long long)kWave * c.WP) * cdiv(s.K, c.WK * c.KW);
    int conc = std::min(kMaxLds / c.lds, kCUWaves / waves);
    conc = (int)std::max<long long>(1, std::min<long long>(conc, (wgs + kCUs - 1) / kCUs));
    const double reads_wave = c.KW * padded * nchunks;
    const double resident = (double)conc * waves;
    const double lds_clk = resident < 16 ? 4.6 * 16.0 / resident : 4.6;   // latency-bound below 16 wavefronts
    const double t_lds = conc * waves * reads_wave * lds_clk;
    const double t_valu = (resident / 4.0) * reads_wave * (s.V + 1) * 2.4;
    const double fill_bytes = (double)s.C * c.Hb * s.W * s.ub;
    const double t_fill = conc * fill_bytes / 48.0;
    const double t_fixed = 3000.0 + nchunks * (700.0 + 60.0 * c.KW);
    const double per_round = std::max(t_lds, t_valu) + t_fill + t_fixed;
    const double rounds = std::ceil((double)wgs / ((double)kCUs * conc));
    return rounds * per_round;
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
               const Launch& over, Plan& p)
{
    const int K = csr.K;
    const int st = g.stride, pad = g.pad;
    p.E = (g.H + 2 * pad - R) / st + 1;
    p.F = (g.W + 2 * pad - S) / st + 1;

    // ---- images interleaved per LDS element: as wide an element as the batch can fill (16 bytes at most)
    int V = over.V;
    const int vmax = 16 / elem_bytes;
    if (V == 0) {
        V = vmax;
        while (V > 1 && V / 2 >= g.N) V /= 2;
    }
    if (!pow2_in(V, 1, vmax)) return SC_EINVAL;

    Shape s;
    s.K = K; s.C = C; s.R = R; s.S = S;
    s.V = V;
    s.ub = V * elem_bytes;
    s.W = g.W;
    // pitch and group height: the padding below/right of an image is shared with the
    // next group/row, but every output's receptive field must still start inside its own group
    s.Wp = std::max(g.W + pad, (p.F - 1) * st + 1);
    s.Hs = std::max(g.H + pad, (p.E - 1) * st + 1);
    const int ngroups = std::max(1, cdiv(g.N, V));
    s.npos = (long long)ngroups * s.Hs * s.Wp;
    s.row_nnz = K > 0 ? (double)csr.colidx.size() / K : 0.0;
    if (s.npos + 1024 >= (1ll << 31)) return SC_EUNSUPPORTED;  // positions are 32-bit in the kernel

    if (over.lds_budget > kMaxLds) return SC_EINVAL;
    if (over.KW && !pow2_in(over.KW, 1, 16)) return SC_EINVAL;
    if (over.WP * std::max(1, over.WK) > kMaxWaves || over.WK > kMaxWaves) return SC_EINVAL;

    // ---- candidates
    static const int budgets[] = {40 * 1024, 52 * 1024, 80 * 1024, 160 * 1024};
    Cand best{};
    double best_t = -1.0;
    for (int WP = 1; WP <= 8; WP *= 2) {
        if (over.WP && WP != 1) break;
        const int wp = over.WP ? over.WP : WP;
        const int Hb = tile_rows(kWave * wp, s.Wp, R, S);
        const long long CS = (long long)Hb * s.Wp;
        for (int WK = 1; WK <= kMaxWaves; WK *= 2) {
            if (over.WK && WK != 1) break;
            const int wk = over.WK ? over.WK : WK;
            if (wp * wk > kMaxWaves) continue;
            for (int KW = 1; KW <= 16; KW *= 2) {
                if (over.KW && KW != 1) break;
                const int kw = over.KW ? over.KW : KW;
                if (kw * V > 64) continue;                       // accumulators must stay in registers
                if (!over.KW && !over.WK && (long long)wk * kw >= 2ll * K && wk * kw > 1) continue;
                for (int bi = 0; bi < 4; ++bi) {
                    if ((over.lds_budget || over.Cc) && bi) break;
                    const int budget = over.lds_budget ? over.lds_budget : budgets[bi];
                    int Cc = over.Cc ? std::min(over.Cc, C) : (int)std::min<long long>(C, budget / (CS * s.ub));
                    if (Cc < 1) continue;
                    Cc = std::min(Cc, 2047);                     // the staging map keeps the channel in 11 bits
                    if (!over.Cc) Cc = cdiv(C, cdiv(C, Cc));     // even chunks
                    const long long lds = (long long)Cc * CS * s.ub;
                    if (lds > kMaxLds) continue;
                    Cand c{wp, wk, kw, Cc, Hb, (int)CS, (int)lds};
                    const double t = estimate(s, c);
                    if (best_t < 0 || t < best_t) {
                        best_t = t;
                        best = c;
                    }
                }
            }
        }
    }
    if (best_t < 0) return SC_EUNSUPPORTED;

    p.V = V; p.WP = best.WP; p.WK = best.WK; p.KW = best.KW; p.Cc = best.Cc;
    p.Wp = s.Wp; p.Hs = s.Hs;
    p.span = kWave * p.WP;
    p.Hb = best.Hb; p.CS = best.CS;
    p.nchunks = cdiv(C, p.Cc);
    p.ngroups = ngroups;
    p.npos = s.npos;
    const long long ntiles = (s.npos + p.span - 1) / p.span;
    const int KB = p.WK * p.KW;
    p.kblocks = cdiv(K, KB);
    p.threads = kWave * p.WP * p.WK;
    p.lds_bytes = best.lds;
    const long long grid = (ntiles + 7) / 8 * 8 * p.kblocks;
    if (ntiles > INT_MAX / 2 || grid > INT_MAX) return SC_EUNSUPPORTED;
    p.ntiles = (int)ntiles;
    p.grid = (int)grid;

    // ---- tables
    p.krow.assign((size_t)p.kblocks * KB, -1);
    for (int k = 0; k < K; ++k) p.krow[k] = k;  // slot (kb, wk, kk) <-> channel kb*KB + wk*KW + kk

    const int RS = R * S;
    const int nchunks = p.nchunks;
    const int SW = p.KW + 1;  // descriptor: first entry, then batches of each of the KW rows
    p.seg.assign((size_t)p.kblocks * nchunks * p.WK * SW, 0);
    p.entries.clear();
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
                        last = Entry{wb, ((c - c0) * p.CS + r * p.Wp + sx) * s.ub};
                        p.entries.push_back(last);
                    }
                    const int nb = cdiv(n, kBatch);
                    // padding repeats the last real tap with weight zero
                    for (int t = n; t < nb * kBatch; ++t) p.entries.push_back(Entry{0u, last.off});
                    sg[1 + kk] = nb;
                    if (p.entries.size() > (size_t)INT_MAX / 2) return SC_EUNSUPPORTED;
                }
            }
        }
    for (int t = 0; t < kBatch; ++t) p.entries.push_back(Entry{0u, 0});  // slack for look-ahead fetches
    return SC_OK;
}

}  // namespace sc
