// Per-geometry plan of the tile kernel: launch configuration and the CSR
// re-expressed as LDS tap offsets.
//
// Section 7 of arXiv 2011.06295 (after Park et al.) stores, instead of a bare
// column number, the pre-computed offset of each stored weight into the input
// array, so the kernel does no index arithmetic per weight.  The same idea is
// used here against the LDS tile: entry offset = c_local*G*PS + r*Wp + s, to
// which a lane only adds the base address of its own output position.
// The paper's unified per-row count (one trip count for every output channel)
// reappears at segment granularity: each (row, channel-chunk) segment is padded
// with zero-weight entries to a multiple of the scalar fetch batch.
#include "internal.h"

#include <algorithm>
#include <climits>

#include "../../include/sparse_conv.h"

namespace sc {

namespace {

constexpr int kWave = 64;
constexpr int kMaxThreads = 1024;
constexpr int kMaxLds = 160 * 1024;
constexpr int kDefaultLds = 64 * 1024;

inline int cdiv(int a, int b) { return (a + b - 1) / b; }

bool pow2_in(int v, int lo, int hi) { return v >= lo && v <= hi && (v & (v - 1)) == 0; }

}  // namespace

int build_plan(const Csr& csr, int C, int R, int S, int elem_bytes, const Geometry& g,
               const Launch& over, Plan& p)
{
    const int K = csr.K;
    const int st = g.stride, pad = g.pad;
    const int E = (g.H + 2 * pad - R) / st + 1;
    const int F = (g.W + 2 * pad - S) / st + 1;
    p.E = E;
    p.F = F;

    // ---- images interleaved per LDS element: as wide an element as the batch can fill (16 bytes at most)
    int V = over.V;
    const int vmax = 16 / elem_bytes;
    if (V == 0) {
        V = vmax;
        while (V > 1 && V / 2 >= g.N) V /= 2;
    }
    if (!pow2_in(V, 1, vmax)) return SC_EINVAL;
    const int ub = V * elem_bytes;
    const int ngroups = std::max(1, cdiv(g.N, V));

    const int budget = over.lds_budget > 0 ? over.lds_budget : kDefaultLds;
    if (budget > kMaxLds) return SC_EINVAL;
    const int max_elems = budget / ub;
    const int Wp = g.W + 2 * pad;

    // ---- output rows per tile and image groups per tile: aim at 256 positions
    int B = over.B, G = over.G;
    if (B <= 0) B = (E * F >= 256) ? std::max(1, std::min(E, 256 / F)) : E;
    B = std::min(B, E);
    if (G <= 0) G = (B == E && E * F < 256) ? std::max(1, 256 / (E * F)) : 1;
    G = std::min(G, ngroups);
    int Hb = (B - 1) * st + R;
    int PS = Hb * Wp;
    if (over.B <= 0 || over.G <= 0) {
        // shrink automatically chosen extents until one channel fits
        while ((long long)G * PS > max_elems && over.G <= 0 && G > 1) G = (G + 1) / 2;
        while ((long long)G * PS > max_elems && over.B <= 0 && B > 1) {
            B = (B + 1) / 2;
            Hb = (B - 1) * st + R;
            PS = Hb * Wp;
        }
    }
    if ((long long)G * PS > max_elems) return SC_EUNSUPPORTED;

    int Cc = over.Cc > 0 ? std::min(over.Cc, C) : std::min(C, max_elems / (G * PS));
    if (Cc < 1 || (long long)Cc * G * PS > max_elems) return SC_EUNSUPPORTED;
    int nchunks = cdiv(C, Cc);
    if (over.Cc <= 0) Cc = cdiv(C, nchunks);  // even chunks
    nchunks = cdiv(C, Cc);

    const int slots = G * B * F;
    int WP = over.WP > 0 ? over.WP : cdiv(slots, kWave);
    if (WP * kWave < slots || WP * kWave > kMaxThreads) return over.WP > 0 ? SC_EINVAL : SC_EUNSUPPORTED;
    int KW = over.KW > 0 ? over.KW : 8;
    if (!pow2_in(KW, 1, 16)) return SC_EINVAL;
    int WK = over.WK > 0 ? over.WK : std::max(1, std::min(16 / WP, 8));
    if (over.KW <= 0) while (KW > 1 && KW / 2 >= K) KW /= 2;
    if (over.WK <= 0) while (WK > 1 && (WK - 1) * KW >= K) --WK;
    if (WP * WK * kWave > kMaxThreads) return SC_EINVAL;

    p.V = V; p.G = G; p.B = B; p.Cc = Cc; p.WP = WP; p.WK = WK; p.KW = KW;
    p.Hb = Hb; p.Wp = Wp; p.PS = PS;
    p.nchunks = nchunks;
    p.nbands = cdiv(E, B);
    p.ngroups = ngroups;
    p.ntg = cdiv(ngroups, G);
    p.ntiles = p.ntg * p.nbands;
    const int KB = WK * KW;
    p.kblocks = cdiv(K, KB);
    p.slots = slots;
    p.threads = kWave * WP * WK;
    p.lds_bytes = Cc * G * PS * ub;
    const long long grid = (long long)cdiv(p.ntiles, 8) * 8 * p.kblocks;
    if (grid > INT_MAX) return SC_EUNSUPPORTED;
    p.grid = (int)grid;

    // ---- tables
    p.krow.assign((size_t)p.kblocks * KB, -1);
    for (int k = 0; k < K; ++k) p.krow[k] = k;  // slot (kb, wk, kk) <-> channel kb*KB + wk*KW + kk

    const int RS = R * S;
    p.seg.assign((size_t)p.kblocks * nchunks * KB * 2, 0);
    p.entries.clear();
    for (int kb = 0; kb < p.kblocks; ++kb)
        for (int ch = 0; ch < nchunks; ++ch) {
            const int c0 = ch * Cc, c1 = std::min(C, c0 + Cc);
            for (int w = 0; w < KB; ++w) {
                const int k = p.krow[(size_t)kb * KB + w];
                int* sg = &p.seg[(((size_t)kb * nchunks + ch) * KB + w) * 2];
                sg[0] = (int)p.entries.size();
                sg[1] = 0;
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
                    const int c = col / RS, r = (col / S) % R, s = col % S;
                    float wv = csr.val32[(size_t)(q - csr.colidx.data())];
                    uint32_t wb;
                    static_assert(sizeof(float) == 4, "");
                    __builtin_memcpy(&wb, &wv, 4);
                    last = Entry{wb, ((c - c0) * G) * PS + r * Wp + s};
                    p.entries.push_back(last);
                }
                const int nb = cdiv(n, kBatch);
                for (int t = n; t < nb * kBatch; ++t) p.entries.push_back(Entry{0u, last.off});
                sg[1] = nb;
                if (p.entries.size() > (size_t)INT_MAX / 2) return SC_EUNSUPPORTED;
            }
        }
    for (int t = 0; t < kBatch; ++t) p.entries.push_back(Entry{0u, 0});  // slack for look-ahead fetches
    return SC_OK;
}

}  // namespace sc
