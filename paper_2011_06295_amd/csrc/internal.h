// Internal declarations shared by the host side and the kernels of
// libsparseconv.  Nothing here is part of the public ABI.
#pragma once

#include <cstdint>
#include <map>
#include <memory>
#include <tuple>
#include <utility>
#include <vector>

namespace sc {

// ---------------------------------------------------------------- host CSR (section 7)

struct Csr {
    int K = 0, L = 0;
    std::vector<int> rowptr;       // [K+1]
    std::vector<int> colidx;       // [nnz], ascending inside a row
    std::vector<float> val32;      // stored values (for SC_F16: the binary16 values widened exactly)
    std::vector<uint16_t> val16;   // binary16 patterns, SC_F16 only
    // cluster-quantised layers only: 4-bit centroid numbers of the stored entries, two to a
    // byte (entry 2i in the low nibble), and the 16 centroids as binary16
    bool coded = false;
    std::vector<uint8_t> code;
    uint16_t centroid[16] = {};
};

uint16_t float_to_half_rne(float f);
float half_to_float(uint16_t h);

// Encodes w*mask row by row; with unify every row is extended with explicit
// zeros to the count of the fullest row.  Returns false if nnz would not fit int32.
bool encode_csr(const float* w, const unsigned char* mask, int K, int L, bool unify, bool half, Csr& out);

// The same for cluster-quantised weights: index [K][L] holds centroid numbers 0..15,
// centroids[16] are rounded to binary16; the stored value of an entry is its centroid
// (an explicit zero of the unify step: the first centroid that is zero).
// Returns an SC_* status (SC_EINVAL: an index above 15, or a zero is needed and no centroid is zero).
int encode_csr_codebook(const unsigned char* index, const float* centroids, const unsigned char* mask,
                        int K, int L, bool unify, bool half, Csr& out);

// ---------------------------------------------------------------- launch configuration

// Tunables of the tile kernel; 0 = choose automatically.
struct Launch {
    int V = 0;    // images interleaved per LDS element
    int WP = 0;   // wavefronts across output positions (64 * LP positions each)
    int WK = 0;   // wavefronts across output channels
    int KW = 0;   // output channels per wavefront
    int Cc = 0;   // channels per LDS pass
    int lds_budget = 0;
    int LP = 0;   // positions per lane (1 or 2)
    int kblocks = 0;  // channel blocks (at least ceil(K / (WK * KW)); more leaves slots empty)
    int store = 0;    // output stores: 1 ordinary, 2 non-temporal (the output is not read again by this kernel)
    int lanes = 0;    // what a lane stands for: 1 a lattice position, 1 + G (G = 1, 2, 4, 8, 16) an output element, with
                      // G image groups interleaved element by element (see Plan)
    int csplit = 0;   // parts the input channels of a (tile, channel block) are dealt over (1, 2, 4, 8), each part a
                      // workgroup of its own; the last one to finish adds the partial sums up
    int pool = 0;     // not a launch parameter: set from the handle's epilogue.  1: the store step takes the maximum over
                      // 2 x 2 windows, so a tile has to hold whole pairs of output rows (output lanes only)
};

struct Geometry {
    int N, H, W, stride, pad;
    bool operator<(const Geometry& o) const {
        return std::tie(N, H, W, stride, pad) < std::tie(o.N, o.H, o.W, o.stride, o.pad);
    }
};

constexpr int kStage = 4;  // tile elements a thread stages per chunk (loads in flight: kStage * V)
constexpr int kBatch = 4;  // plan entries fetched per scalar load; segments are padded to a multiple

// One stored weight as the kernel consumes it: fp32 weight bits and the LDS
// byte offset ((c_local * CS + r * Wp + s) * element bytes) of its tap relative
// to a position.
struct Entry {
    uint32_t wbits;
    int32_t off;
};

// A batch of kBatch entries as the kernel fetches it (the device image of the entry table):
// the weights, then the offsets, two to a 64-bit word (the lower entry in the lower half).
struct Batch {
    uint32_t w[kBatch];
    unsigned long long off2[kBatch / 2];
};
static_assert(sizeof(Batch) == kBatch * sizeof(Entry), "same bytes as the entries it holds");

// Everything a forward call needs for one geometry.
//
// The batch is laid out (virtually) as one tall zero-padded image per channel:
// image group g (V images interleaved) occupies rows [g*Hs, (g+1)*Hs) with its
// `pad` top rows zero, Hs = H + pad; a row holds `pad` zero columns followed by
// the W real ones, Wp = W + pad.  Bottom and right padding are the next
// group's top rows and the next row's left columns (Hs and Wp grow by extra
// zero rows/columns when the padding exceeds the filter, so that every
// receptive field still starts inside its own group and row).  A position q = Y*Wp + X of
// that lattice stands for the output whose receptive field starts there; tap
// (r, s) of it is the element at q + r*Wp + s, so neighbouring lanes always
// read neighbouring LDS elements, whatever the tap.
//
// Lanes stand either for lattice positions (64 * LP consecutive ones a wavefront; positions on padding
// compute a value nobody stores), or for output elements only (G > 0): G consecutive image groups form a
// super-group whose lattice is interleaved element by element, element index ((Y*Wp + X)*G + g); the
// outputs of the batch are numbered (super-group, i, j), a tile owns span / G consecutive ones, and lane
// l of a wavefront is image group l % G of the wavefront's output l / G.  Sixteen consecutive lanes then
// still read sixteen consecutive 16-byte elements (16 / G outputs of one row x G groups), which is what
// keeps ds_read_b128 free of bank conflicts, and no lane is spent on padding.
struct Plan {
    int V, WP, WK, KW, Cc, LP;
    int G;         // 0: lanes are lattice positions; else image groups interleaved per element, lanes are outputs
    int PT;        // G > 0: outputs per tile (span / G)
    int store;     // 1 ordinary output stores, 2 non-temporal
    int E, F, st;  // output size (of the convolution), stride
    int pool;      // 1: 2 x 2 maximum in the store step (the stored map is E/2 x F/2)
    int Wp;        // row pitch of the padded lattice
    int Hs;        // rows per image group
    int span;      // positions per workgroup = 64 * WP
    int Hb;        // lattice rows held by a tile
    int CS;        // channel stride inside the tile, in elements (= Hb * Wp)
    int nchunks;   // ceil(C / Cc)
    int ngroups;   // ceil(N / V)
    long long npos;  // positions of the whole batch = ngroups * Hs * Wp
    int ntiles;    // ceil(npos / span)
    int kblocks;   // ceil(K / (WK*KW))
    int J;         // parts the channel chunks of a (tile, channel block) are dealt over (one workgroup each)
    int cpp;       // chunks per part = ceil(nchunks / J)
    int threads;   // 64 * WP * WK
    int nbuf;      // tile buffers in LDS: 2 when there are several chunks
    int SL;        // staging slots per channel = SG * SP
    int SG, SP;    // slot groups and slots per group
    int rows_mode; // staging slots: 0 whole planes group by group, 1 tile rows, 2 every element of a banded tile
    int pitch;     // row pitch inside the tile: Wp, or span + S - 1 for a banded tile
    int zero_elems;   // elements of the zero region behind the tile buffers (what zero-weight padding entries read)
    int tbl_off;   // LDS byte offset of the slot table
    int lds_bytes; // tile + slot table
    int grid;      // workgroups launched (ntiles * kblocks rounded up to the XCD count)
    // host tables
    bool compact = false;         // binary16 weights (binary16 layers, cluster-quantised layers): one word per device entry
    int off_shift = 0;            // compact: LDS byte offset = (entry >> 16) << off_shift
    std::vector<uint32_t> image4; // compact: the entry table as the device reads it, (offset >> off_shift) << 16 | binary16 weight
    std::vector<Entry> entries;   // segments padded to kBatch
    std::vector<int> seg;         // [kblocks][nchunks][WK][1 + KW] = first entry, batches of each row; then one
                                  // terminal descriptor whose first entry is the end of the last segment
    std::vector<int> krow;        // [kblocks][WK][KW] output channel or -1
    // Output-lane plans: what every thread stages per chunk, worked out here instead of in every workgroup.
    // Tiles whose first output has the same place within a super-group stage the same pattern; there are
    // nphase such places (tile t has pattern t % nphase).  units[(ph * npass * kStage + j) * threads + tid] is
    // the j-th unit of thread tid: .off = source byte offset relative to the tile's first image group at the
    // chunk's first channel (0x80000000: nothing to load), .dst = byte offset in the first tile buffer.
    struct Unit {
        uint32_t off, dst;
    };
    int nphase = 0, npass = 0;
    std::vector<Unit> units;
    std::vector<Batch> image;     // the entry table as the device reads it (built with the first upload)
    unsigned long long id = 0;    // unique per built plan (names what the static device scratch currently holds)
    // device copies (owned)
    void* d_entries = nullptr;
    void* d_seg = nullptr;
    void* d_krow = nullptr;
    void* d_units = nullptr;
    void* d_partial = nullptr;    // J > 1: partial sums [ntiles * kblocks * J][KW * LP * V][threads] fp32 and ...
    void* d_counters = nullptr;   // ... one arrival counter per (tile, channel block), zero between launches
    bool uploaded = false;
    ~Plan();
};

// Chooses the configuration (honouring overrides) and builds the host tables.
// With `ranked` it only lists the candidate configurations (estimated clocks,
// full override), cheapest first, and builds nothing.  Returns an SC_* status.
int build_plan(const Csr& csr, int C, int R, int S, int elem_bytes, const Geometry& g,
               const Launch& over, Plan& plan, std::vector<std::pair<double, Launch>>* ranked = nullptr);

// Checks a built plan against its CSR on the host (every stored weight exactly once, with its
// tap's LDS offset, inside the tile; every output channel in one slot; table sizes; launch
// limits).  Returns 0, or the number of the first failed check.
int check_plan(const Csr& csr, int C, int R, int S, int elem_bytes, const Plan& plan);

// ---------------------------------------------------------------- kernels

// Division by a run-time constant: q = n / d for 0 <= n < 2^31.
struct FastDiv {
    uint32_t mul, shift, d;
};
FastDiv make_fastdiv(int d);

struct KernelArgs {
    const void* x;
    void* y;
    const uint32_t* entries;   // device image: one Batch per kBatch entries (compact: one 32-bit word per entry)
    int compact;               // entries are (offset units << 16 | binary16 weight) words
    int off_shift;             // compact: bytes per offset unit, as a shift (1 or 2)
    const int* seg;
    const int* krow;
    const float* bias;   // [K] or null
    int relu;            // clamp the stored value at zero
    int pool;            // 1: store the maximum over 2 x 2 windows of the (biased, clamped) sums: [N][K][E/2][F/2]
    int pool_rows;       // pooled store: output channels per wavefront that go through LDS together (1..KW, as LDS allows)
    int nt_store;        // non-temporal output stores
    int N, C, H, W, K, E, F, stride, pad;
    int WP, WK, Cc, Wp, Hs, Hb, CS, span;
    int nchunks, ngroups, ntiles, kblocks;
    int tile_elems;  // elements from one tile buffer to the next: Cc * CS and a spare one
    // staging: a channel of the tile is SG groups of SP slots (SL = SG * SP); units are
    // ordered (group, channel, slot-in-group) and a thread's next unit is nthreads further on
    int SL;          // slots of one channel
    int SG, SP;      // rows mode: 1 group of Hb*W slots; groups mode: GC image groups of H*W slots
    int rows_mode;   // slots: 0 whole planes group by group, 1 tile rows, 2 every element of a banded tile
    int pitch;       // banded tile: elements per band (span + S - 1)
    int zero_elems;  // zeroed elements behind the tile buffers
    int tbl_off;     // byte offset of the slot table in LDS (after the tile buffers and the zero region)
    int st_dg, st_dc, st_dp; // nthreads = st_dg * (Cc * SP) + st_dc * SP + st_dp
    int nbuf;                // tile buffers in LDS: 2 when there are several chunks
    int npass;               // staging passes per chunk: ceil(SG * Cc * SP / (kStage * threads))
    int J, logJ, cpp;        // channel parts per (tile, channel block), its log2, chunks per part
    float* partial;          // J > 1: partial sums of every part, [item][accumulator][thread]
    unsigned* counters;      // J > 1: parts of a (tile, channel block) that have delivered theirs
    const void* units;       // output lanes: per-thread staging units (Plan::Unit), nphase patterns
    int nphase;              // output lanes: staging patterns; tile t uses pattern t % nphase
    int real;                // lanes are output elements (else lattice positions)
    int logG;                // log2 of the image groups interleaved per element (0 unless real)
    int PT;                  // real: outputs per tile
    int nout;                // real: outputs of the whole batch = super-groups * E * F
    FastDiv fd_Wp, fd_Hs, fd_W, fd_HW, fd_SP, fd_CP, fd_pitch;  // divisors Wp, Hs, W, H*W, SP, Cc*SP, pitch
    FastDiv fd_EF, fd_F, fd_GW, fd_nphase;                      // real: divisors E*F, F, G*W, nphase
#ifdef SC_PHASE_TIMING
    unsigned long long* phase;  // 8 counters per workgroup, or null
#endif
};

// Size of the static device array behind sparse_conv_forward_static, and its address on the current
// device (looked up once per device).  Returns a hipError_t value (0 = success).
constexpr size_t kStaticScratchBytes = 16u << 20;   // SC_STATIC_SCRATCH_BYTES of the public header
int static_scratch(void** ptr);

// Enqueues the tile kernel.  Returns a hipError_t value (0 = success).
int launch_tile_kernel(int dtype, int V, int KW, int LP, const KernelArgs& a, int grid, int threads,
                       int lds_bytes, void* stream);

// Roof probes (probes.hip).  Each enqueues one kernel and returns a hipError_t value.
int launch_lds_read_probe(void* sink, int workgroups, int iterations, void* stream, long long* bytes_read);
int launch_copy_probe(void* dst, const void* src, long long bytes, void* stream);

}  // namespace sc

struct sparse_conv_s {
    int K, C, R, S, L, dtype;
    unsigned flags;
    sc::Csr csr;
    sc::Launch over;
    float* d_bias = nullptr;   // device copy of the epilogue bias (owned)
    unsigned epilogue = 0;
    std::map<sc::Geometry, sc::Launch> tuned;   // per geometry: configuration found by sparse_conv_autotune
    std::map<sc::Geometry, std::unique_ptr<sc::Plan>> plans;
    int last_hip = 0;
    int device = -1;           // HIP device that holds the handle's device buffers; -1 until the first is made
};
