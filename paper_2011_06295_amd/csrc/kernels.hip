// Direct sparse convolution tile kernel for gfx950 (CDNA4).
//
// What it computes (arXiv 2011.06295, section 3 eq. 1 restricted to the stored
// weights of section 7; the kernel organisation replaces the one of section 8):
//   Out[n][k][i][j] = sum over stored entries t of row k of
//                     w[t] * Xpad[n][c_t][i*stride + r_t][j*stride + s_t]
//
// Organisation.  The batch is seen as one tall zero-padded lattice per channel
// (image groups of V element-wise interleaved images stacked vertically, each
// with `pad` zero rows above and `pad` zero columns to the left; see Plan in
// internal.h).  A workgroup owns `span` consecutive lattice positions and keeps
// what they touch, for Cc channels at a time, in LDS: the lattice rows they
// span, or, for maps much wider than a tile, R bands of span + S - 1 elements.
// A lane owns LP (1 or 2) positions, 64 apart: tap (r, s) of channel c is the LDS element
// at position + c*CS + r*pitch + s, so the 64 lanes of a wavefront always read 64
// consecutive, naturally aligned V-vectors (one ds_read_b128 for 4 fp32 or
// 8 fp16 images), free of bank conflicts whatever the tap.  Positions that fall
// on padding compute a value nobody stores.  A wavefront owns KW output
// channels whose accumulators stay in registers across the channel chunks.
// Stored weights arrive as (weight, LDS offset) pairs, wave-uniform, fetched in
// batches of kBatch through the scalar path, a batch ahead of their use; per
// pair a lane forms one LDS address, reads its LP positions at constant
// distances from it, and does LP * V fused multiply-adds in fp32: the address
// arithmetic, the scalar fetches and the loop control are shared by LP reads.
// Channel chunks alternate between two LDS buffers: the global loads of the
// next chunk are issued into registers during the arithmetic of the current
// one and written to the other buffer after it (one barrier per chunk).
//
// Second kind of tile (REAL = true): lanes are output elements, G image groups
// interleaved element by element, so small maps spend no lanes on padding; the
// staging units of a thread then come from a per-plan table.  Further down:
// the issue priority that falls with the rows done, the deep form of the
// multiply loop (a whole batch of reads in flight), channel parts (the input
// channels of a tile dealt over several workgroups, summed by the last to
// finish), and the store step (bias, ReLU, optionally the 2 x 2 maximum).
#include <hip/hip_runtime.h>

#include <atomic>
#include <mutex>

#include "internal.h"

namespace sc {

// Read-only plan tables are addressed through the constant address space: a
// wave-uniform load from it is always issued on the scalar path (s_load), which
// an ordinary global pointer loses once a barrier sits between store and load.
#define SC_CONSTANT __attribute__((address_space(4)))
#pragma clang diagnostic push
#pragma clang diagnostic ignored "-Wold-style-cast"
template <typename T>
__device__ __forceinline__ const SC_CONSTANT T* as_constant(const T* p)
{
    return (const SC_CONSTANT T*)(p);
}
// The kernel's argument block as it lies in the kernel-argument segment (the one by-value argument starts it).
__device__ __forceinline__ const SC_CONSTANT KernelArgs* argument_segment()
{
    return (const SC_CONSTANT KernelArgs*)(__builtin_amdgcn_kernarg_segment_ptr());
}
#pragma clang diagnostic pop

// LDS addressed by its 32-bit address: what a read takes is the sum the kernel formed, as it is
// (a read through an ordinary pointer into the LDS array adds the array's address once more).
#define SC_LDS __attribute__((address_space(3)))
#pragma clang diagnostic push
#pragma clang diagnostic ignored "-Wold-style-cast"
__device__ __forceinline__ unsigned lds_address(const unsigned char* in_lds)
{
    return (unsigned)(unsigned long long)(const SC_LDS unsigned char*)(in_lds);
}
template <typename Vt>
__device__ __forceinline__ Vt lds_read(unsigned address)
{
    return *(const SC_LDS Vt*)(address);
}
template <typename Vt>
__device__ __forceinline__ void lds_write(unsigned address, const Vt& value)
{
    *(SC_LDS Vt*)(address) = value;
}
#pragma clang diagnostic pop

// n / d for 0 <= n < 2^31 with the multiplier prepared on the host.
template <typename FD>   // a FastDiv in whatever address space
__device__ __forceinline__ int fdiv(int n, const FD& f)
{
    return f.d == 1 ? n : (int)(__umulhi((unsigned)n, f.mul) >> f.shift);
}

// One element through a buffer descriptor; out-of-range offsets read as zero.
template <typename T>
__device__ __forceinline__ T load_elem(__amdgpu_buffer_rsrc_t rs, unsigned off);
template <>
__device__ __forceinline__ float load_elem<float>(__amdgpu_buffer_rsrc_t rs, unsigned off)
{
    return __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(rs, (int)off, 0, 0));
}
template <>
__device__ __forceinline__ _Float16 load_elem<_Float16>(__amdgpu_buffer_rsrc_t rs, unsigned off)
{
    const unsigned short h = __builtin_amdgcn_raw_buffer_load_b16(rs, (int)off, 0, 0);
    _Float16 r;
    __builtin_memcpy(&r, &h, 2);
    return r;
}

// One output element stored with the non-temporal hint.  Written as an instruction of its
// own: a hinted and a plain store under a run-time switch would be merged into one plain store.
__device__ __forceinline__ void store_nontemporal(float* p, float v)
{
    asm volatile("global_store_dword %0, %1, off nt" ::"v"(p), "v"(v) : "memory");
}
__device__ __forceinline__ void store_nontemporal(_Float16* p, _Float16 v)
{
    unsigned short h;
    __builtin_memcpy(&h, &v, 2);
    const unsigned bits = h;
    asm volatile("global_store_short %0, %1, off nt" ::"v"(p), "v"(bits) : "memory");
}

template <typename T, int V>
struct Vec {
    typedef T type __attribute__((ext_vector_type(V)));
    static __device__ __forceinline__ T get(const type& v, int i) { return v[i]; }
    static __device__ __forceinline__ void set(type& v, int i, T x) { v[i] = x; }
    static __device__ __forceinline__ type zero() { return type(T(0)); }
};
template <typename T>
struct Vec<T, 1> {
    typedef T type;
    static __device__ __forceinline__ T get(const type& v, int) { return v; }
    static __device__ __forceinline__ void set(type& v, int, T x) { v = x; }
    static __device__ __forceinline__ type zero() { return T(0); }
};

// Developer instrumentation (builds with -DSC_PHASE_TIMING only): every
// wavefront accumulates the 100 MHz wall-clock ticks spent in [0] set-up and
// the first chunk's staging, [1] starting a chunk's loads, [2] the gather-FMA,
// [3] depositing the next chunk and waiting for the other wavefronts, [4] the
// store, and reports [5] its start and [6] its end tick (8 counters per
// wavefront, 16 wavefront slots per workgroup).
#ifdef SC_PHASE_TIMING
#define SC_PHASE(i)                                  \
    do {                                             \
        const unsigned long long n_ = wall_clock64(); \
        ph_acc[i] += n_ - ph_t;                      \
        ph_t = n_;                                   \
    } while (0)
#else
#define SC_PHASE(i) \
    do {            \
    } while (0)
#endif

template <typename T, int V, int KW, int LP, bool COMPACT, bool REAL>
__global__ __launch_bounds__(1024) void tile_kernel(const KernelArgs a)
{
#ifdef SC_PHASE_TIMING
    unsigned long long ph_t = wall_clock64();
    const unsigned long long ph_start = ph_t;
    unsigned long long ph_acc[5] = {0, 0, 0, 0, 0};
#endif
    using VT = Vec<T, V>;
    using vec = typename VT::type;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];

    const int tid = threadIdx.x;
    const int nthreads = blockDim.x;

    // Workgroup -> (tile, channel block).  Consecutive workgroup ids go round
    // the 8 XCDs.  The (tile, channel block) pairs, tile-major, are cut into 8
    // equal contiguous ranges, one per XCD: the XCDs get the same number of
    // workgroups, and a tile's rows, which its neighbours and its other channel
    // blocks stage again, are fetched into one L2 (two where a range ends).
    // With J > 1 the channel chunks of a (tile, channel block) are dealt over J workgroups (neighbours in the
    // numbering, hence on one XCD); each walks its own chunks, and the last to finish adds the partial sums up.
    const int bid = blockIdx.x;
    const int item = (bid & 7) * (int)(gridDim.x >> 3) + (bid >> 3);
    if (item >= a.ntiles * a.kblocks * a.J) return;
    const int pair = item >> a.logJ;                  // (tile, channel block)
    const int part = item & (a.J - 1);
    const int tile_id = pair / a.kblocks;
    const int kb = pair - tile_id * a.kblocks;
    const int ch_first = part * a.cpp;                // the host gives every part at least one chunk
    const int ch_end = ch_first + a.cpp < a.nchunks ? ch_first + a.cpp : a.nchunks;

    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lane = tid & 63;
    const int wp = wave % a.WP;
    const int wk = wave / a.WP;

    // Lattice lanes: the tile covers lattice positions [q0, q0 + span); its row 0 is lattice row Y0; wavefront wp
    // covers positions [wp*LP*64, (wp+1)*LP*64) of the tile, the lane's p-th position is 64*p after its first.
    // Output lanes: the tile covers outputs [o0, o0 + PT) of the numbering (super-group, i, j); its row 0 is the
    // lattice row of its first output; lane l of wavefront wp is image group l % G of output wp * (64 / G) + l / G.
    int Y0, g_first, lrel = 0, lpos, my_o = 0;
    long long q0 = 0;
    if constexpr (REAL) {
        const int G1 = (1 << a.logG) - 1;
        const int EF = a.E * a.F;
        const int o0 = tile_id * a.PT;                   // the host guarantees fewer than 2^31 lanes in all
        const int u0 = fdiv(o0, a.fd_EF);
        Y0 = u0 * a.Hs + fdiv(o0 - u0 * EF, a.fd_F) * a.stride;
        g_first = u0 << a.logG;
        my_o = o0 + wp * (64 >> a.logG) + (lane >> a.logG);
        // lanes past the last output work on the last output again (nothing of theirs is stored)
        const int o = my_o < a.nout ? my_o : a.nout - 1;
        const int u = fdiv(o, a.fd_EF);
        const int rem = o - u * EF;
        const int i = fdiv(rem, a.fd_F);
        const int j = rem - i * a.F;
        lpos = (((u * a.Hs + i * a.stride - Y0) * a.Wp + j * a.stride) << a.logG) + (lane & G1);
    } else {
        q0 = (long long)tile_id * a.span;
        Y0 = fdiv((int)q0, a.fd_Wp);      // the host guarantees fewer than 2^31 positions
        const int lq0 = (int)q0 - Y0 * a.Wp;
        lrel = lq0 + wp * (LP * 64) + lane;  // first position, relative to the start of lattice row Y0
        // tile element of that position: the tile starts at that row, or (banded tile) at the first position
        lpos = a.rows_mode == 2 ? wp * (LP * 64) + lane : lrel;
        g_first = fdiv(Y0, a.fd_Hs);
    }
    const int lposb = lpos * (int)sizeof(vec);

    float acc[KW][LP][V];
#pragma unroll
    for (int kk = 0; kk < KW; ++kk)
#pragma unroll
        for (int p = 0; p < LP; ++p)
#pragma unroll
            for (int v = 0; v < V; ++v) acc[kk][p][v] = 0.f;

    const T* __restrict__ x = static_cast<const T*>(a.x);
    const int chan_stride = a.H * a.W;
    const int img_stride = a.C * chan_stride;   // the host guarantees N*C*H*W < 2^31
    const unsigned chan_bytes = (unsigned)chan_stride * (unsigned)sizeof(T);
    const unsigned img_bytes = (unsigned)img_stride * (unsigned)sizeof(T);
    // Input is read through a buffer descriptor that starts at the first image
    // group of the tile (plus the chunk's first channel) and ends with the
    // input: offsets marked invalid (>= 2^31) and images past the end of the
    // batch are out of its range and read as zero, so no load needs a branch.
    const size_t tile_base = (size_t)g_first * V * img_bytes;
    const size_t total_bytes = (size_t)a.N * img_bytes;
    auto chunk_rsrc = [&](int c0) {
        const size_t chunk_base = tile_base + (size_t)c0 * chan_bytes;
        const size_t remain = total_bytes > chunk_base ? total_bytes - chunk_base : 0;
        return __builtin_amdgcn_make_buffer_rsrc(const_cast<char*>(reinterpret_cast<const char*>(x)) + chunk_base, 0,
                                                 remain > 0x80000000ull ? 0x80000000u : (unsigned)remain, 0x00020000);
    };

    // Per (channel block, chunk, wavefront) descriptor: first plan entry, then the
    // batch count of each of the KW rows; the KW segments are contiguous in the
    // entry table.  The descriptor of the next chunk and the first batch of this
    // chunk are requested a phase ahead, so their latency is hidden.
    const SC_CONSTANT int* sg = as_constant(a.seg) + (((size_t)kb * a.nchunks + ch_first) * a.WK + wk) * (KW + 1);
    const size_t sg_step = (size_t)a.WK * (KW + 1);
    int d_start = sg[0];
    int d_end = sg[KW + 1];  // the next descriptor's first entry: segments are laid out in descriptor order
    int d_nb[KW];
#pragma unroll
    for (int kk = 0; kk < KW; ++kk) d_nb[kk] = sg[1 + kk];
    // Compact entries (binary16 layers, and cluster-quantised layers, whose weights are binary16 centroids:
    // sections 6 and 9): an entry is one word, (LDS offset in units of 2 or 4 bytes) << 16 | binary16 weight,
    // half the bytes of the (fp32 weight, offset) pair.  A batch is decoded once, when it has arrived, on the
    // scalar unit: the offsets are shifted into the places an ordinary batch has them in; the weight stays
    // where it is and goes into the mixed-precision multiply-add as a binary16 operand (no conversion).
    // (A 4-bit centroid number in the entry and a table lookup per entry were measured, with the table in
    // a register (v_readlane) and in the scalar cache (dependent s_load): both a third slower.)
    constexpr bool compact = COMPACT;
    constexpr int epd = compact ? 1 : 2;       // 32-bit words per entry
    const SC_CONSTANT uint32_t* e = nullptr;   // epd * kBatch dwords per batch
    int nb[KW];
    Batch cur;
    Batch ahead;   // the batch after cur (deep pipeline only)
    constexpr bool kDeep = REAL && LP == 1 && sizeof(T) == 4;   // whole batches of reads in flight (see compute)
    auto fetch_batch = [&](Batch& b, const SC_CONSTANT uint32_t* p) __attribute__((always_inline)) {
#pragma unroll
        for (int u = 0; u < kBatch; ++u) b.w[u] = p[u];
        if constexpr (!compact) {
            const SC_CONSTANT unsigned long long* q = reinterpret_cast<const SC_CONSTANT unsigned long long*>(p + kBatch);
#pragma unroll
            for (int u = 0; u < kBatch / 2; ++u) b.off2[u] = q[u];
        }
    };
    auto decode = [&](Batch& b) __attribute__((always_inline)) {
        if constexpr (!compact) return;
#pragma unroll
        for (int u = 0; u < kBatch / 2; ++u)
            b.off2[u] = ((unsigned long long)((b.w[2 * u + 1] >> 16) << a.off_shift) << 32) |
                        (unsigned long long)((b.w[2 * u] >> 16) << a.off_shift);
    };
    // the weight of an entry as the multiply-add takes it
    auto weight = [](uint32_t word) __attribute__((always_inline)) -> float {
        if constexpr (compact) {
            const unsigned short h = (unsigned short)word;
            _Float16 f;
            __builtin_memcpy(&f, &h, 2);
            return (float)f;
        } else {
            return __uint_as_float(word);
        }
    };
    auto begin_chunk = [&](int ch) __attribute__((always_inline)) {
        e = as_constant(a.entries) + (size_t)epd * (size_t)d_start;
#pragma unroll
        for (int kk = 0; kk < KW; ++kk) nb[kk] = d_nb[kk];
        fetch_batch(cur, e);  // the table ends in 2 * kBatch slack entries
        if constexpr (kDeep) {
            e += epd * kBatch;
            fetch_batch(ahead, e);
        }
        if (ch + 1 < ch_end) {
            sg += sg_step;
            d_start = sg[0];
            d_end = sg[KW + 1];
#pragma unroll
            for (int kk = 0; kk < KW; ++kk) d_nb[kk] = sg[1 + kk];
        }
    };
    // The entries of a wavefront's segment are read once, batch by batch, through the scalar
    // cache; coming from HBM each batch would cost a full memory latency.  One vector load per
    // 64 bytes of the coming segment (d_start..d_end), issued a chunk ahead, brings the lines
    // into L2 first.  The loaded value is only kept until the next wait for staged data.
    auto touch = [&]() __attribute__((always_inline)) -> unsigned {
        const size_t first = (size_t)epd * (size_t)d_start + (size_t)lane * 16;  // 16 words = 64 bytes
        return first < (size_t)epd * (size_t)d_end ? a.entries[first] : 0u;
    };
    auto retire = [](unsigned t) __attribute__((always_inline)) { asm volatile("" ::"v"(t)); };

    // ---- LDS: nbuf tile buffers (two when the channels come in several chunks), each followed by
    // one spare element (where staging units without a real element are written), the slot table
    vec* tile = reinterpret_cast<vec*>(smem);
    const int reject = a.tile_elems - 1;   // the spare element, relative to a buffer
    const unsigned tile_at = lds_address(smem);

    // Staging table.  What a tile holds of one channel is the same for every
    // channel: a set of SL slots, each one real (non-padding) element of the
    // lattice rows the tile covers.  Slots are enumerated so that neighbouring
    // slots are neighbours in memory: row by row for maps taller than the tile,
    // image group by image group (whole H x W planes) for small maps.  Each
    // slot is decoded once into
    //   .x  byte offset of image 0 of its group, relative to the first group
    //       of the tile, at channel 0 (0x80000000: the slot is not in the tile)
    //   .y  tile element index at channel 0
    // and staging then only adds channel strides.
    // (Output lanes: tiles whose first output has the same place in a super-group stage the same pattern, and the
    // host has worked out every thread's units for each of the few patterns: no table is built here.)
    int2* tbl = reinterpret_cast<int2*>(smem + a.tbl_off);
    if constexpr (!REAL) {
    for (int sl = tid; sl < a.SL; sl += nthreads) {
        int gs, ys, xx, Yt;
        if (a.rows_mode == 2) {  // banded tile: element sl is lattice element q0 + band * Wp + offset
            const int band = fdiv(sl, a.fd_pitch);
            const int Ls = (int)q0 + band * a.Wp + (sl - band * a.pitch);
            const int Ys = fdiv(Ls, a.fd_Wp);
            gs = fdiv(Ys, a.fd_Hs);
            ys = Ys - gs * a.Hs - a.pad;
            xx = Ls - Ys * a.Wp - a.pad;
            Yt = 0;
        } else if (a.rows_mode) {   // slot = (tile row, column)
            Yt = fdiv(sl, a.fd_W);
            xx = sl - Yt * a.W;
            const int Ys = Y0 + Yt;
            gs = fdiv(Ys, a.fd_Hs);
            ys = Ys - gs * a.Hs - a.pad;
        } else {                    // slot = (image group, row, column) of the groups the tile can touch
            const int gi = fdiv(sl, a.fd_HW);
            const int rem = sl - gi * chan_stride;
            ys = fdiv(rem, a.fd_W);
            xx = rem - ys * a.W;
            gs = g_first + gi;
            Yt = gs * a.Hs + a.pad + ys - Y0;
        }
        const bool ok = gs < a.ngroups && ys >= 0 && ys < a.H && xx >= 0 && xx < a.W && Yt >= 0 && Yt < a.Hb;
        int2 t;
        // (gs - g_first) * V * img_bytes < 2^31 is guaranteed by the host
        t.x = ok ? (int)((unsigned)((gs - g_first) * V) * img_bytes + (unsigned)(ys * a.W + xx) * (unsigned)sizeof(T))
                 : (int)0x80000000;
        t.y = !ok ? 0 : a.rows_mode == 2 ? sl : Yt * a.Wp + a.pad + xx;
        tbl[sl] = t;
    }
    }
    // A chunk is SG * Cc * SP units, unit u = (slot group * Cc + channel) * SP + slot: in that
    // order consecutive units are consecutive in memory across the channels of an image.
    // Thread `tid` owns units tid, tid + nthreads, ..., kStage of them per pass (the host
    // sizes chunks for a single pass where it can).  Staging has two halves, so that the
    // loads of the next chunk can be in flight while the current one is consumed:
    // `fetch_unit` issues the loads of one unit into registers (the units of the next chunk
    // are spread over the rows of the current one, so that the wavefronts of a workgroup do
    // not all queue on the memory pipeline at once), `deposit` writes them into a tile buffer.
    // A thread's units of the first pass are the same in every chunk (only the descriptor's
    // base moves on), so their source offset and tile element are worked out once, after
    // the table is complete (`prepare_units`).  In a short last chunk the units of absent
    // channels load whatever follows in memory (or zero past the end) into tile channels
    // that no plan entry refers to.
    vec st_val[kStage];
    unsigned st_dst[kStage];       // where the unit in flight goes: LDS address in the first tile buffer
    unsigned u_off[kStage];        // first pass: source offset (0x80000000: none) ...
    unsigned u_dst[kStage];        // ... and LDS address in the first buffer (the spare element if none)
    int gi = 0, c = 0, sp = 0;     // later passes: the thread's next unit
    int f_cn = 0;                  // later passes: channels of the chunk being fetched
    __amdgpu_buffer_rsrc_t f_rs = chunk_rsrc(0);
    auto next_unit = [&]() __attribute__((always_inline)) {
        sp += a.st_dp;
        const bool k1 = sp >= a.SP;
        sp -= k1 ? a.SP : 0;
        c += a.st_dc + (k1 ? 1 : 0);
        const bool k2 = c >= a.Cc;
        c -= k2 ? a.Cc : 0;
        gi += a.st_dg + (k2 ? 1 : 0);
    };
    // output lanes: this thread's units of the tile's pattern, kStage per pass, as the host laid them out
    const uint2* my_units = nullptr;
    if constexpr (REAL) {
        const int phase = tile_id - fdiv(tile_id, a.fd_nphase) * a.nphase;
        my_units = static_cast<const uint2*>(a.units) + (size_t)phase * a.npass * kStage * nthreads + tid;
    }
    auto prepare_units = [&]() __attribute__((always_inline)) {
        if constexpr (REAL) {
#pragma unroll
            for (int t = 0; t < kStage; ++t) {
                const uint2 un = my_units[(size_t)t * nthreads];
                u_off[t] = un.x;
                u_dst[t] = tile_at + un.y;
            }
            return;
        }
        gi = fdiv(tid, a.fd_CP);
        const int r0 = tid - gi * a.Cc * a.SP;
        c = fdiv(r0, a.fd_SP);
        sp = r0 - c * a.SP;
#pragma unroll
        for (int t = 0; t < kStage; ++t) {
            const bool in = gi < a.SG;
            const int2 sd = tbl[in ? (int)__umul24(gi, a.SP) + sp : 0];
            const bool ok = in && sd.x >= 0;
            u_off[t] = ok ? (unsigned)sd.x + (unsigned)c * chan_bytes : 0x80000000u;
            u_dst[t] = tile_at + (unsigned)(ok ? sd.y + (int)__umul24(c, a.CS) : reject) * (unsigned)sizeof(vec);
            next_unit();
        }
    };
    auto fetch_begin = [&](int ch) __attribute__((always_inline)) {
        const int c0 = ch * a.Cc;
        f_cn = (a.C - c0) < a.Cc ? (a.C - c0) : a.Cc;
        f_rs = chunk_rsrc(c0);
    };
    auto fetch_unit = [&](int t) __attribute__((always_inline)) {  // first pass; t is a constant after unrolling
        st_dst[t] = u_dst[t];
        unsigned ib = img_bytes;
        // with many accumulators, keep the V offsets of all units from being worked out once and held in registers
        if constexpr (KW * LP * V > 16 || LP * V > 8) asm volatile("" : "+s"(ib));
#pragma unroll
        for (int v = 0; v < V; ++v) VT::set(st_val[t], v, load_elem<T>(f_rs, u_off[t] + (unsigned)v * ib));
    };
    auto fetch_more = [&](int p) __attribute__((always_inline)) {  // pass p >= 1: units decoded on the fly
        if constexpr (REAL) {
#pragma unroll
            for (int t = 0; t < kStage; ++t) {
                const uint2 un = my_units[(size_t)(p * kStage + t) * nthreads];
                st_dst[t] = tile_at + un.y;
#pragma unroll
                for (int v = 0; v < V; ++v) VT::set(st_val[t], v, load_elem<T>(f_rs, un.x + (unsigned)v * img_bytes));
            }
            return;
        }
        if (p == 1) {  // (gi, c, sp) of unit tid + kStage * nthreads
            gi = fdiv(tid, a.fd_CP);
            const int r0 = tid - gi * a.Cc * a.SP;
            c = fdiv(r0, a.fd_SP);
            sp = r0 - c * a.SP;
            for (int t = 0; t < kStage; ++t) next_unit();
        }
#pragma unroll
        for (int t = 0; t < kStage; ++t) {
            const bool in = gi < a.SG && c < f_cn;
            const int2 sd = tbl[in ? (int)__umul24(gi, a.SP) + sp : 0];
            const bool ok = in && sd.x >= 0;
            const unsigned off = ok ? (unsigned)sd.x + (unsigned)c * chan_bytes : 0x80000000u;
            st_dst[t] = tile_at + (unsigned)(ok ? sd.y + (int)__umul24(c, a.CS) : reject) * (unsigned)sizeof(vec);
#pragma unroll
            for (int v = 0; v < V; ++v) VT::set(st_val[t], v, load_elem<T>(f_rs, off + (unsigned)v * img_bytes));
            next_unit();
        }
    };
    auto deposit = [&](int buf) __attribute__((always_inline)) {
        const unsigned base = (unsigned)(buf * a.tile_elems) * (unsigned)sizeof(vec);
#pragma unroll
        for (int t = 0; t < kStage; ++t)  // unconditional (units without an element go to the buffer's spare one): one add a write
            lds_write<vec>(st_dst[t] + base, st_val[t]);
    };

    // Gather-FMA over this wavefront's KW rows of one chunk whose tile starts at
    // LDS byte `base` (already offset by the lane's position).  The stored
    // weights of the wavefront's rows form one stream of batches; a step
    // consumes the batch in A in two halves and requests the following batch
    // (possibly the next row's first) into B.  While the multiply-adds of one
    // half run, the LDS reads of the next half (and, in the first half, the
    // scalar fetch of B) are in flight; the wait at the end of a half therefore
    // finds them complete, and one wait serves LDS and scalar returns alike.
    // Entry offsets are in bytes and come two to a 64-bit scalar: one 64-bit add of the lane's
    // address (held twice, in both halves of a register pair) forms the addresses of two reads.
    constexpr int kGroup = 2;                          // entries whose reads are issued together
    constexpr int kGroups = kBatch / kGroup;           // even: the two read buffers alternate
    constexpr int kPosBytes = 64 * (int)sizeof(vec);   // LDS distance between a lane's successive positions
    // empty statements that use a group's registers: the compiler has to complete their loads before them
    auto arrived = [](const vec(&x)[kGroup][LP]) __attribute__((always_inline)) {
#pragma unroll
        for (int u = 0; u < kGroup; ++u)
#pragma unroll
            for (int p = 0; p < LP; ++p) asm volatile("" ::"v"(x[u][p]));
    };
    // A SIMD issues from the oldest of its ready wavefronts first, so the four wavefronts it holds of a
    // workgroup would finish a chunk one after the other, and the last of them would run alone, at the
    // rate at which one wavefront can hide its own read latencies.  The wavefront's issue priority therefore
    // falls as it gets through its rows: highest while more than half of them are left, then while more
    // than a quarter, more than an eighth, lowest after that.  Those behind are served first, and all
    // reach the end of the chunk within the last few rows of each other.
    auto level = [](int kk) constexpr { const int left = KW - kk; return left * 2 > KW ? 3 : left * 4 > KW ? 2 : left * 8 > KW ? 1 : 0; };
    auto yield_to_slower = [&](int kk) __attribute__((always_inline)) {
        if constexpr (KW >= 2) {
            if (kk > 0 && level(kk) == level(kk - 1)) return;
            switch (level(kk)) {
                case 3: __builtin_amdgcn_s_setprio(3); break;
                case 2: __builtin_amdgcn_s_setprio(2); break;
                case 1: __builtin_amdgcn_s_setprio(1); break;
                default: __builtin_amdgcn_s_setprio(0); break;
            }
        }
    };
    auto compute = [&](int base, bool prefetch) __attribute__((always_inline)) {
        vec xs[2][kGroup][LP];
        static_assert(kGroup == 2, "a group is the two entries whose offsets share a 64-bit scalar");
        // the lane's LDS address (of the tile element under its first position), in both halves
        const unsigned lane_at = lds_address(smem) + (unsigned)base;
        const unsigned long long base2 = ((unsigned long long)lane_at << 32) | lane_at;
        auto gather = [&](vec(&x)[kGroup][LP], const Batch& E, int g) __attribute__((always_inline)) {
            const unsigned long long at2 = base2 + E.off2[g];   // no carry between the halves: LDS addresses are small
#pragma unroll
            for (int u = 0; u < kGroup; ++u) {
                const unsigned at = (unsigned)(u ? at2 >> 32 : at2);
#pragma unroll
                for (int p = 0; p < LP; ++p) x[u][p] = lds_read<vec>(at + p * kPosBytes);
            }
        };
        auto fma = [&](const vec(&x)[kGroup][LP], const Batch& E, int g, float (&ac)[LP][V]) __attribute__((always_inline)) {
#pragma unroll
            for (int u = 0; u < kGroup; ++u) {
                const float w = weight(E.w[g * kGroup + u]);
#pragma unroll
                for (int p = 0; p < LP; ++p)
#pragma unroll
                    for (int v = 0; v < V; ++v) ac[p][v] = __builtin_fmaf(w, (float)VT::get(x[u][p], v), ac[p][v]);
            }
        };
        if constexpr (kDeep) {
            // One position per lane: a whole batch of reads is in flight while the multiply-adds of the
            // batch before it run (twice the distance between a read and its use that the grouped form
            // below has).  Three batches are live: `cur` (its reads issued), `ahead` (requested a step
            // ago) and the one a step requests.  The two read buffers p and q (eight separate registers-to-be,
            // not an array: an array of them is handled as one wide value and moved about as a whole where
            // control flow joins) take turns; a row with an odd number of batches ends in a step that reads the
            // next batch into the registers it has just used, one by one, so that every row begins in p.
            static_assert(kBatch == 4, "the read buffers below are written out for four entries");
            vec p0, p1, p2, p3, q0, q1, q2, q3;
            auto fma1 = [&](const vec& x, uint32_t word, float (&ac)[LP][V]) __attribute__((always_inline)) {
                const float w = weight(word);
#pragma unroll
                for (int v = 0; v < V; ++v) ac[0][v] = __builtin_fmaf(w, (float)VT::get(x, v), ac[0][v]);
            };
            auto arrived4 = [](const vec& x0, const vec& x1, const vec& x2, const vec& x3) __attribute__((always_inline)) {
                asm volatile("" ::"v"(x0));
                asm volatile("" ::"v"(x1));
                asm volatile("" ::"v"(x2));
                asm volatile("" ::"v"(x3));
            };
            {
                decode(cur);
                const unsigned long long lo = base2 + cur.off2[0], hi = base2 + cur.off2[1];
                p0 = lds_read<vec>((unsigned)lo);
                p1 = lds_read<vec>((unsigned)(lo >> 32));
                p2 = lds_read<vec>((unsigned)hi);
                p3 = lds_read<vec>((unsigned)(hi >> 32));
            }
            // a step: the reads of A (into x) and the fetch of B have been issued before; wait for both, issue
            // B's reads into y and the fetch of the batch after B into C, then run A's multiply-adds
            auto step = [&](const Batch& A, Batch& B, Batch& C, vec& x0, vec& x1, vec& x2, vec& x3, vec& y0, vec& y1, vec& y2,
                            vec& y3, float (&ac)[LP][V]) __attribute__((always_inline)) {
                __builtin_amdgcn_sched_barrier(0);
                arrived4(x0, x1, x2, x3);
                decode(B);
                const unsigned long long lo = base2 + B.off2[0], hi = base2 + B.off2[1];
                y0 = lds_read<vec>((unsigned)lo);
                y1 = lds_read<vec>((unsigned)(lo >> 32));
                y2 = lds_read<vec>((unsigned)hi);
                y3 = lds_read<vec>((unsigned)(hi >> 32));
                e += epd * kBatch;
                fetch_batch(C, e);
                __builtin_amdgcn_sched_barrier(0);
                fma1(x0, A.w[0], ac);
                fma1(x1, A.w[1], ac);
                fma1(x2, A.w[2], ac);
                fma1(x3, A.w[3], ac);
                __builtin_amdgcn_sched_barrier(0);
            };
#pragma unroll
            for (int kk = 0; kk < KW; ++kk) {
                yield_to_slower(kk);
                if (prefetch) {
#pragma unroll
                    for (int t = kk * kStage / KW; t < (kk + 1) * kStage / KW; ++t) fetch_unit(t);
                }
                int b = 0;
                for (; b + 2 <= nb[kk]; b += 2) {
                    Batch far, farther;
                    step(cur, ahead, far, p0, p1, p2, p3, q0, q1, q2, q3, acc[kk]);
                    step(ahead, far, farther, q0, q1, q2, q3, p0, p1, p2, p3, acc[kk]);
                    cur = far;
                    ahead = farther;
                }
                if (b < nb[kk]) {
                    Batch far;
                    __builtin_amdgcn_sched_barrier(0);
                    arrived4(p0, p1, p2, p3);
                    decode(ahead);
                    const unsigned long long lo = base2 + ahead.off2[0], hi = base2 + ahead.off2[1];
                    e += epd * kBatch;
                    fetch_batch(far, e);
                    __builtin_amdgcn_sched_barrier(0);
                    fma1(p0, cur.w[0], acc[kk]);
                    p0 = lds_read<vec>((unsigned)lo);
                    __builtin_amdgcn_sched_barrier(0);
                    fma1(p1, cur.w[1], acc[kk]);
                    p1 = lds_read<vec>((unsigned)(lo >> 32));
                    __builtin_amdgcn_sched_barrier(0);
                    fma1(p2, cur.w[2], acc[kk]);
                    p2 = lds_read<vec>((unsigned)hi);
                    __builtin_amdgcn_sched_barrier(0);
                    fma1(p3, cur.w[3], acc[kk]);
                    p3 = lds_read<vec>((unsigned)(hi >> 32));
                    __builtin_amdgcn_sched_barrier(0);
                    cur = ahead;
                    ahead = far;
                }
            }
            arrived4(p0, p1, p2, p3);   // the reads issued for the batch after the last one end here
            return;
        }
        decode(cur);
        gather(xs[0], cur, 0);
        arrived(xs[0]);
        // A step consumes batch A group by group: while the multiply-adds of group j run on one
        // read buffer, the reads of group j + 1 (after A's last group: B's first) fill the other,
        // and during the first group the scalar fetch of B is in flight as well.
        auto step = [&](const Batch& A, Batch& B, float (&ac)[LP][V]) __attribute__((always_inline)) {
#pragma unroll
            for (int j = 0; j < kGroups; ++j) {
                __builtin_amdgcn_sched_barrier(0);
                if (j == 0) {
                    gather(xs[1], A, 1);
                    e += epd * kBatch;
                    fetch_batch(B, e);
                } else if (j + 1 < kGroups) {
                    gather(xs[(j + 1) & 1], A, j + 1);
                } else {
                    decode(B);   // complete since the wait that ended the first group
                    gather(xs[0], B, 0);
                }
                __builtin_amdgcn_sched_barrier(0);
                fma(xs[j & 1], A, j, ac);
                __builtin_amdgcn_sched_barrier(0);
                arrived(xs[(j + 1) & 1]);
            }
        };
#pragma unroll
        for (int kk = 0; kk < KW; ++kk) {
            yield_to_slower(kk);
            if (prefetch) {  // this row's share of the next chunk's staging loads
#pragma unroll
                for (int t = kk * kStage / KW; t < (kk + 1) * kStage / KW; ++t) fetch_unit(t);
            }
            Batch nxt;
            int b = 0;
            for (; b + 2 <= nb[kk]; b += 2) {
                step(cur, nxt, acc[kk]);
                step(nxt, cur, acc[kk]);
            }
            if (b < nb[kk]) {
                step(cur, nxt, acc[kk]);
                cur = nxt;
            }
        }
    };

    if constexpr (!REAL) __syncthreads();  // slot table complete
    prepare_units();
    fetch_begin(ch_first);
#pragma unroll
    for (int t = 0; t < kStage; ++t) fetch_unit(t);
    // the input loads do not wait for the descriptor (requested at the top); what needs it comes after them
    unsigned warm = touch();  // the first chunk's entries
    begin_chunk(ch_first);
    // while the first loads are in flight: padding rows/columns and absent images are zeroed
    // once and stay zero for the whole kernel (staging writes real elements only)
    for (int u = tid; u < a.nbuf * a.tile_elems + a.zero_elems; u += nthreads) tile[u] = VT::zero();   // and the zero region behind them
    __syncthreads();  // zero fill complete
    deposit(0);
    for (int p = 1; p < a.npass; ++p) {
        fetch_more(p);
        deposit(0);
    }
    retire(warm);
    __syncthreads();  // chunk 0 is in LDS
    SC_PHASE(0);
    const int tile_bytes = a.tile_elems * (int)sizeof(vec);
    for (int ch = ch_first; ch < ch_end; ++ch) {
        const bool more = ch + 1 < ch_end;
        if (more) {
            warm = touch();           // chunk ch+1's entries (its descriptor was requested a chunk ago)
            fetch_begin(ch + 1);
        }
        SC_PHASE(1);
        compute(((ch - ch_first) & (a.nbuf - 1)) * tile_bytes + lposb, more);  // chunk ch+1's loads are issued along the way
        if constexpr (KW >= 2) __builtin_amdgcn_s_setprio(3);   // what follows is short and others wait for it
        SC_PHASE(2);
        if (more) {
            begin_chunk(ch + 1);
            deposit((ch + 1 - ch_first) & (a.nbuf - 1));
            retire(warm);
            for (int p = 1; p < a.npass; ++p) {
                fetch_more(p);
                deposit((ch + 1 - ch_first) & (a.nbuf - 1));
            }
            __syncthreads();  // chunk ch+1 is in LDS; everyone is done with chunk ch's buffer
            SC_PHASE(3);
        }
    }

    // What follows needs launch constants that nothing before it uses (output pointer, channel slots, bias, the
    // exchange buffers of split channels, the divisors of the store's position decode).  Held in scalar registers
    // from the kernel's start they would be spilled across the whole multiply loop; they are read here instead,
    // from the kernel-argument segment, through a pointer the compiler cannot trace back to it.
    const SC_CONSTANT KernelArgs* late = argument_segment();
    asm volatile("" : "+s"(late));
    const SC_CONSTANT KernelArgs& la = *late;

    // ---- channel parts: every part leaves its sums in global memory; the one that finds all others done
    // (a counter per (tile, channel block), back at zero when the launch ends) adds them up in the order of
    // the parts, whichever came last, and goes on to the store.  The sums travel as device-scope atomic
    // stores and loads (written through to, and read from, the level all XCDs share) and the arrival is a
    // device-scope atomic: no cache of the chip is flushed or invalidated as a whole, which a device-scope
    // fence would do (measured: it made a 27 us layer take 78).  A part's stores are complete (the wait at
    // the workgroup-scope fence) before its arrival is counted.
    if (la.J > 1) {
        constexpr int kAcc = KW * LP * V;
        float* mine = la.partial + (size_t)item * kAcc * nthreads + tid;
#pragma unroll
        for (int kk = 0; kk < KW; ++kk)
#pragma unroll
            for (int p = 0; p < LP; ++p)
#pragma unroll
                for (int v = 0; v < V; ++v)
                    __hip_atomic_store(mine + (size_t)((kk * LP + p) * V + v) * nthreads, acc[kk][p][v], __ATOMIC_RELAXED,
                                       __HIP_MEMORY_SCOPE_AGENT);
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");   // this wavefront's stores have completed
        __syncthreads();                                         // ... and every wavefront's; nobody reads the tile any more
        unsigned* ticket = reinterpret_cast<unsigned*>(smem);
        if (tid == 0) *ticket = __hip_atomic_fetch_add(la.counters + pair, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __syncthreads();
        if (*ticket != (unsigned)(la.J - 1)) return;
        if (tid == 0) __hip_atomic_store(la.counters + pair, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        const float* all = la.partial + (size_t)(pair << la.logJ) * kAcc * nthreads + tid;
#pragma unroll
        for (int kk = 0; kk < KW; ++kk)
#pragma unroll
            for (int p = 0; p < LP; ++p)
#pragma unroll
                for (int v = 0; v < V; ++v) acc[kk][p][v] = 0.f;
        for (int j = 0; j < la.J; ++j) {   // in the order of the parts; all loads of a part are in flight together
            float got[kAcc];
#pragma unroll
            for (int i = 0; i < kAcc; ++i)
                got[i] = __hip_atomic_load(all + ((size_t)j * kAcc + i) * nthreads, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
#pragma unroll
            for (int kk = 0; kk < KW; ++kk)
#pragma unroll
                for (int p = 0; p < LP; ++p)
#pragma unroll
                    for (int v = 0; v < V; ++v) acc[kk][p][v] += got[(kk * LP + p) * V + v];
        }
    }

    // ---- store: one writer per output element
    T* __restrict__ y = static_cast<T*>(la.y);
    const SC_CONSTANT int* kr = as_constant(la.krow) + ((size_t)kb * la.WK + wk) * KW;
    const size_t plane = (size_t)la.E * la.F;
    // ---- pooled store (the pooling step that follows the activation in section 3's layer sequence): the
    // workgroup's sums (after bias and ReLU) go through LDS, as many of a wavefront's channels at a time as
    // it holds, and the 2 x 2 windows staged there are dealt over all threads: each takes the maximum of a
    // window's four values and stores it into the E/2 x F/2 map.  A tile holds whole pairs of output rows
    // (the planner's condition, which makes F and the tile powers of two), so a window's other three values
    // lie G, F*G and F*G + G elements after its first.  Consecutive threads take consecutive windows of a row.
    if constexpr (REAL) {
        if (la.pool) {
            float* stage = reinterpret_cast<float*>(smem);
            const int elems = 64 * la.WP, G = 1 << la.logG, FG = la.F << la.logG;
            const int logF = __builtin_ctz((unsigned)la.F), logW = __builtin_ctz((unsigned)elems) - 2;   // windows per slot: elems / 4
            const int planes = la.WK * V;                           // slots (of `elems` sums) per staged channel row
            const size_t pooled = (size_t)(la.E >> 1) * (la.F >> 1);
            const int o0 = tile_id * la.PT;
            const int* krow = la.krow + (size_t)kb * la.WK * KW;
            const int rows = la.pool_rows, row_floats = (int)nthreads * V;
            float* mine = stage + (size_t)(wk * V) * elems + wp * 64 + lane;
            __syncthreads();   // nobody reads the tile any more
            int round_first = 0;
#pragma unroll
            for (int kk = 0; kk < KW; ++kk) {
                const int k = kr[kk];
                const float bias = (la.bias && k >= 0) ? as_constant(la.bias)[k] : 0.f;
#pragma unroll
                for (int v = 0; v < V; ++v) {
                    float r = acc[kk][0][v] + bias;
                    if (la.relu) r = r > 0.f ? r : 0.f;
                    mine[(kk - round_first) * row_floats + v * elems] = r;
                }
                if (kk + 1 - round_first < rows && kk + 1 < KW) continue;
                __syncthreads();
                const int windows = ((kk + 1 - round_first) * planes) << logW;
                for (int it = tid; it < windows; it += (int)nthreads) {
                    const int slot = it >> logW, pe = it & ((1 << logW) - 1);
                    const int qr = slot / planes, pl = slot - qr * planes;      // staged row, (wavefront row, image) of the slot
                    const int wkq = pl / V, v = pl - wkq * V;
                    const int kq = krow[wkq * KW + round_first + qr];
                    const int gsel = pe & (G - 1), po = pe >> la.logG;           // image group, window of the tile
                    const int jj = po & ((la.F >> 1) - 1), rp = po >> (logF - 1);
                    const int orel = (rp << (logF + 1)) + (jj << 1);             // the window's first output, in the tile
                    const int o = o0 + orel;
                    const int u = fdiv(o, la.fd_EF);
                    const int rem = o - u * (la.E * la.F);
                    const int oi = rem >> logF, oj = rem & (la.F - 1);
                    const int n = (((u << la.logG) + gsel) * V) + v;
                    if (kq < 0 || o >= la.nout || n >= la.N) continue;
                    const float* w4 = stage + (size_t)slot * elems + (orel << la.logG) + gsel;
                    const float a0 = w4[0], a1 = w4[G], a2 = w4[FG], a3 = w4[FG + G];
                    const float m0 = a1 > a0 ? a1 : a0, m1 = a3 > a2 ? a3 : a2;
                    const float r = m1 > m0 ? m1 : m0;
                    T* at = &y[((size_t)n * la.K + kq) * pooled + (size_t)(oi >> 1) * (la.F >> 1) + (oj >> 1)];
                    if (la.nt_store)
                        store_nontemporal(at, (T)r);
                    else
                        *at = (T)r;
                }
                __syncthreads();   // the staged sums have been read: the next round's may come
                round_first = kk + 1;
            }
            return;
        }
    }
#pragma unroll
    for (int p = 0; p < LP; ++p) {
        // lane -> output element (if any) and image group
        int g, oi, oj;
        bool valid;
        if constexpr (REAL) {
            const int u = fdiv(my_o, la.fd_EF);
            const int rem = my_o - u * (la.E * la.F);
            oi = fdiv(rem, la.fd_F);
            oj = rem - oi * la.F;
            g = (u << la.logG) + (lane & ((1 << la.logG) - 1));
            valid = my_o < la.nout && g < la.ngroups;
        } else {
            const int rel = lrel + p * 64;
            const int Yl = fdiv(rel, la.fd_Wp);
            const int X = rel - Yl * la.Wp;
            const int Y = Y0 + Yl;
            g = fdiv(Y, la.fd_Hs);
            const int yy = Y - g * la.Hs;
            oi = yy / la.stride;
            oj = X / la.stride;
            valid = g < la.ngroups && oi * la.stride == yy && oj * la.stride == X && oi < la.E && oj < la.F;
        }
        if (!valid) continue;
        const size_t pix = (size_t)oi * la.F + oj;
#pragma unroll
        for (int kk = 0; kk < KW; ++kk) {
            const int k = kr[kk];
            if (k < 0) continue;
            const float bias = la.bias ? as_constant(la.bias)[k] : 0.f;  // section 3: bias, then activation
#pragma unroll
            for (int v = 0; v < V; ++v) {
                const int n = g * V + v;
                float r = acc[kk][p][v] + bias;
                if (la.relu) r = r > 0.f ? r : 0.f;
                if (n >= la.N) continue;
                T* at = &y[((size_t)n * la.K + k) * plane + pix];
                if (la.nt_store)
                    store_nontemporal(at, (T)r);
                else
                    *at = (T)r;
            }
        }
    }
#ifdef SC_PHASE_TIMING
    SC_PHASE(4);
    if (lane == 0 && a.phase) {
        unsigned long long* o = a.phase + ((size_t)bid * 16 + wave) * 8;
        for (int i = 0; i < 5; ++i) o[i] = ph_acc[i];
        o[5] = ph_start;
        o[6] = ph_t;
        o[7] = 1;
    }
#endif
}

namespace {

template <typename T, int V, int KW, int LP, bool COMPACT, bool REAL>
int launch_one(const KernelArgs& a, int grid, int threads, int lds_bytes, hipStream_t s)
{
    // accumulators (KW * LP * V floats) plus the reads in flight have to fit a 128-register wavefront
    if constexpr ((LP > 1 && KW * LP * V > 32) || KW * V > 64 || (REAL && LP > 1)) {
        return (int)hipErrorInvalidValue;
    } else {
    auto fn = tile_kernel<T, V, KW, LP, COMPACT, REAL>;
    if (lds_bytes > 64 * 1024) {
        // more than 64 KB of dynamic LDS has to be allowed per kernel and device: once, for the whole 160 KB
        static std::atomic<unsigned long long> allowed{0};   // one bit per device ordinal
        int dev = 0;
        hipError_t e = hipGetDevice(&dev);
        if (e != hipSuccess) return (int)e;
        const unsigned long long bit = dev < 64 ? 1ull << dev : 0ull;
        if (!(allowed.load(std::memory_order_relaxed) & bit)) {
            e = hipFuncSetAttribute(reinterpret_cast<const void*>(fn),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
            if (e != hipSuccess) return (int)e;
            allowed.fetch_or(bit, std::memory_order_relaxed);
        }
    }
    hipLaunchKernelGGL(fn, dim3(grid), dim3(threads), lds_bytes, s, a);
    return (int)hipGetLastError();
    }
}

// one-word entries or not, lanes as outputs or as lattice positions
template <typename T, int V, int KW, int LP>
int pick(const KernelArgs& a, int grid, int threads, int lds, hipStream_t s)
{
    if (a.real)
        return a.compact ? launch_one<T, V, KW, LP, true, true>(a, grid, threads, lds, s)
                         : launch_one<T, V, KW, LP, false, true>(a, grid, threads, lds, s);
    return a.compact ? launch_one<T, V, KW, LP, true, false>(a, grid, threads, lds, s)
                     : launch_one<T, V, KW, LP, false, false>(a, grid, threads, lds, s);
}

template <typename T, int V>
int launch_kw(int KW, int LP, const KernelArgs& a, int grid, int threads, int lds, hipStream_t s)
{
    switch (KW * 8 + LP) {
        case 1 * 8 + 1: return pick<T, V, 1, 1>(a, grid, threads, lds, s);
        case 2 * 8 + 1: return pick<T, V, 2, 1>(a, grid, threads, lds, s);
        case 4 * 8 + 1: return pick<T, V, 4, 1>(a, grid, threads, lds, s);
        case 8 * 8 + 1: return pick<T, V, 8, 1>(a, grid, threads, lds, s);
        case 16 * 8 + 1: return pick<T, V, 16, 1>(a, grid, threads, lds, s);
        case 1 * 8 + 2: return pick<T, V, 1, 2>(a, grid, threads, lds, s);
        case 2 * 8 + 2: return pick<T, V, 2, 2>(a, grid, threads, lds, s);
        case 4 * 8 + 2: return pick<T, V, 4, 2>(a, grid, threads, lds, s);
        case 8 * 8 + 2: return pick<T, V, 8, 2>(a, grid, threads, lds, s);
    }
    return (int)hipErrorInvalidValue;
}

}  // namespace

// Device memory for callers that must not allocate (sparse_conv_forward_static): one array per GPU,
// part of the loaded code object, held until the process ends.  In host code the array's name is
// only a handle for hipGetSymbolAddress; its device address differs from GPU to GPU and is looked
// up once per device, with that device current.
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

int static_scratch(void** ptr)
{
    static std::mutex lock;
    static void* address_on[64] = {};   // per device ordinal
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return (int)e;
    if (dev < 0 || dev >= 64) return (int)hipErrorInvalidDevice;
    std::lock_guard<std::mutex> hold(lock);
    if (!address_on[dev]) {
        void* p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return (int)e;
        if (!p) return (int)hipErrorInvalidSymbol;
        address_on[dev] = p;
    }
    *ptr = address_on[dev];
    return 0;
}

int launch_tile_kernel(int dtype, int V, int KW, int LP, const KernelArgs& a, int grid, int threads,
                       int lds_bytes, void* stream)
{
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (dtype == 0) {
        switch (V) {
            case 1: return launch_kw<float, 1>(KW, LP, a, grid, threads, lds_bytes, s);
            case 2: return launch_kw<float, 2>(KW, LP, a, grid, threads, lds_bytes, s);
            case 4: return launch_kw<float, 4>(KW, LP, a, grid, threads, lds_bytes, s);
        }
    } else {
        switch (V) {
            case 1: return launch_kw<_Float16, 1>(KW, LP, a, grid, threads, lds_bytes, s);
            case 2: return launch_kw<_Float16, 2>(KW, LP, a, grid, threads, lds_bytes, s);
            case 4: return launch_kw<_Float16, 4>(KW, LP, a, grid, threads, lds_bytes, s);
            case 8: return launch_kw<_Float16, 8>(KW, LP, a, grid, threads, lds_bytes, s);
        }
    }
    return (int)hipErrorInvalidValue;
}

}  // namespace sc
