// Internal declarations shared by the host side and the kernels of
// libsparseconv.  Nothing here is part of the public ABI.
#pragma once

#include <cstdint>
#include <map>
#include <memory>
#include <tuple>
#include <vector>

namespace sc {

// ---------------------------------------------------------------- host CSR (section 7)

struct Csr {
    int K = 0, L = 0;
    std::vector<int> rowptr;       // [K+1]
    std::vector<int> colidx;       // [nnz], ascending inside a row
    std::vector<float> val32;      // stored values (for SC_F16: the binary16 values widened exactly)
    std::vector<uint16_t> val16;   // binary16 patterns, SC_F16 only
};

uint16_t float_to_half_rne(float f);
float half_to_float(uint16_t h);

// Encodes w*mask row by row; with unify every row is extended with explicit
// zeros to the count of the fullest row.  Returns false if nnz would not fit int32.
bool encode_csr(const float* w, const unsigned char* mask, int K, int L, bool unify, bool half, Csr& out);

// ---------------------------------------------------------------- launch configuration

// Tunables of the tile kernel; 0 = choose automatically.
struct Launch {
    int V = 0;    // images interleaved per LDS element
    int G = 0;    // image groups per tile
    int B = 0;    // output rows per tile
    int Cc = 0;   // channels per LDS pass
    int WP = 0;   // wavefronts across positions
    int WK = 0;   // wavefronts across output channels
    int KW = 0;   // output channels per wavefront
    int lds_budget = 0;
};

struct Geometry {
    int N, H, W, stride, pad;
    bool operator<(const Geometry& o) const {
        return std::tie(N, H, W, stride, pad) < std::tie(o.N, o.H, o.W, o.stride, o.pad);
    }
};

constexpr int kBatch = 8;  // plan entries fetched per scalar load; segments are padded to a multiple

// One stored weight as the kernel consumes it: fp32 weight bits and the LDS
// element offset (c_local * G * PS + r * Wp + s) of its tap inside the tile.
struct Entry {
    uint32_t wbits;
    int32_t off;
};

// Everything a forward call needs for one geometry.
struct Plan {
    // resolved configuration
    int V, G, B, Cc, WP, WK, KW;
    int E, F;
    int Hb;        // input rows held by a tile: (B-1)*stride + R
    int Wp;        // tile row pitch in elements: W + 2*pad (at least (F-1)*stride + S)
    int PS;        // plane stride in elements (one channel of one group)
    int nchunks;   // ceil(C / Cc)
    int nbands;    // ceil(E / B)
    int ngroups;   // ceil(N / V)
    int ntg;       // ceil(ngroups / G)
    int ntiles;    // ntg * nbands
    int kblocks;   // ceil(K / (WK*KW))
    int slots;     // G * B * F output positions per tile
    int threads;   // 64 * WP * WK
    int lds_bytes;
    int grid;      // workgroups launched (tiles rounded up to the XCD count, times kblocks)
    // host tables
    std::vector<Entry> entries;   // segments padded to kBatch
    std::vector<int> seg;         // [kblocks][nchunks][WK][KW][2] = (first entry, batches)
    std::vector<int> krow;        // [kblocks][WK][KW] output channel or -1
    // device copies (owned)
    void* d_entries = nullptr;
    void* d_seg = nullptr;
    void* d_krow = nullptr;
    bool uploaded = false;
    ~Plan();
};

// Chooses the configuration (honouring overrides) and builds the host tables.
// Returns an SC_* status.
int build_plan(const Csr& csr, int C, int R, int S, int elem_bytes, const Geometry& g,
               const Launch& over, Plan& plan);

// ---------------------------------------------------------------- kernels

struct KernelArgs {
    const void* x;
    void* y;
    const Entry* entries;
    const int* seg;
    const int* krow;
    int N, C, H, W, K, E, F, stride, pad;
    int G, B, Cc, WP, WK, Hb, Wp, PS;
    int nchunks, nbands, ngroups, ntiles, kblocks, slots;
    int tile_elems;  // Cc * G * PS
};

// Enqueues the tile kernel.  Returns a hipError_t value (0 = success).
int launch_tile_kernel(int dtype, int V, int KW, const KernelArgs& a, int grid, int threads,
                       int lds_bytes, void* stream);

}  // namespace sc

struct sparse_conv_s {
    int K, C, R, S, L, dtype;
    unsigned flags;
    sc::Csr csr;
    sc::Launch over;
    std::map<sc::Geometry, std::unique_ptr<sc::Plan>> plans;
    int last_hip = 0;
};
