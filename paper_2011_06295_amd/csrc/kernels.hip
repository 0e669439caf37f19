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
// the rows they touch, for Cc channels at a time, in LDS.  A lane owns one
// position: tap (r, s) of channel c is the LDS element at
// position + c*CS + r*Wp + s, so the 64 lanes of a wavefront always read 64
// consecutive, naturally aligned V-vectors (one ds_read_b128 for 4 fp32 or
// 8 fp16 images), free of bank conflicts whatever the tap.  Positions that fall
// on padding compute a value nobody stores.  A wavefront owns KW output
// channels whose accumulators stay in registers across the channel chunks.
// Stored weights arrive as (weight, LDS offset) pairs, wave-uniform, fetched in
// batches of kBatch through the scalar path with one batch of look-ahead; per
// pair a lane does one vector LDS read and V fused multiply-adds in fp32.
#include <hip/hip_runtime.h>

#include "internal.h"

namespace sc {

constexpr int kStage = 4;  // tile elements a thread stages per round (loads in flight: kStage * V)

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
#pragma clang diagnostic pop

// n / d for 0 <= n < 2^31 with the multiplier prepared on the host.
__device__ __forceinline__ int fdiv(int n, const FastDiv& f)
{
    return f.d == 1 ? n : (int)(__umulhi((unsigned)n, f.mul) >> f.shift);
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

template <typename T, int V, int KW>
__global__ __launch_bounds__(1024) void tile_kernel(const KernelArgs a)
{
    using VT = Vec<T, V>;
    using vec = typename VT::type;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    vec* tile = reinterpret_cast<vec*>(smem);

    const int tid = threadIdx.x;
    const int nthreads = blockDim.x;

    // Workgroup -> (tile, channel block).  Consecutive workgroup ids go round
    // the 8 XCDs.  Each XCD gets one contiguous range of tiles and all their
    // channel blocks, so a tile's rows, which its neighbours and its other
    // channel blocks stage again, are fetched into a single L2.
    const int bid = blockIdx.x;
    const int xcd = bid & 7;
    const int qb = bid >> 3;
    const int kb = qb % a.kblocks;
    const int tile_id = xcd * ((a.ntiles + 7) >> 3) + qb / a.kblocks;
    if (tile_id >= a.ntiles || qb / a.kblocks >= ((a.ntiles + 7) >> 3)) return;

    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lane = tid & 63;
    const int wp = wave % a.WP;
    const int wk = wave / a.WP;

    // The tile covers lattice positions [q0, q0 + span); its row 0 is lattice row Y0.
    const long long q0 = (long long)tile_id * a.span;
    const int Y0 = fdiv((int)q0, a.fd_Wp);      // the host guarantees fewer than 2^31 positions
    const int lq0 = (int)q0 - Y0 * a.Wp;

    // lane -> position -> output element (if any)
    const int lpos = lq0 + wp * 64 + lane;      // tile-local element index of the position
    const int lposb = lpos * (int)sizeof(vec);
    const int Yl = fdiv(lpos, a.fd_Wp);
    const int X = lpos - Yl * a.Wp;
    const int Y = Y0 + Yl;
    const int g = fdiv(Y, a.fd_Hs);
    const int yy = Y - g * a.Hs;
    const int oi = yy / a.stride;
    const int oj = X / a.stride;
    const bool valid = g < a.ngroups && oi * a.stride == yy && oj * a.stride == X && oi < a.E && oj < a.F;

    float acc[KW][V];
#pragma unroll
    for (int kk = 0; kk < KW; ++kk)
#pragma unroll
        for (int v = 0; v < V; ++v) acc[kk][v] = 0.f;

    // padding rows/columns and absent images stay zero for the whole kernel
    for (int u = tid; u < a.tile_elems; u += nthreads) tile[u] = VT::zero();

    const T* __restrict__ x = static_cast<const T*>(a.x);
    const int chan_stride = a.H * a.W;
    const int img_stride = a.C * chan_stride;   // the host guarantees N*C*H*W < 2^31

    // Staging map.  The tile's real (non-padding) elements are enumerated group
    // by group, inside a group channel by channel, inside a channel row by row
    // (RW row slots per channel, RW = min(H, Hb)): in that order one image's
    // elements are contiguous in memory across rows and channels, so consecutive
    // lanes load consecutive addresses even when a feature map is only a few
    // pixels large.  Slots whose row lies outside the tile are skipped.  Thread `tid` owns elements tid,
    // tid + nthreads, ...  Decoding an element gives:
    //   src  input element offset of image 0 of the group at chunk channel 0, or -1 for none
    //   dc   tile element index | channel << 17 | (valid images - 1) << 28
    const int g_first = fdiv(Y0, a.fd_Hs);
    const int g_count = fdiv(Y0 + a.Hb - 1, a.fd_Hs) - g_first + 1;
    const int chan_slots = a.RW * a.W;          // a group holds at most RW rows of the tile
    const int group_slots = a.Cc * chan_slots;
    const int units = g_count * group_slots;    // enumerated slots of a full chunk (some fall outside the tile)
    auto decode = [&](int u, int& src, int& dc) {
        const int gi = fdiv(u, a.fd_group);
        const int rem = u - gi * group_slots;
        const int c = fdiv(rem, a.fd_chan);
        const int r2 = rem - c * chan_slots;
        const int yr = fdiv(r2, a.fd_W);
        const int xx = r2 - yr * a.W;
        const int gs = g_first + gi;
        int r_lo = Y0 - gs * a.Hs - a.pad;      // first input row of group gs inside the tile
        int r_hi = r_lo + a.Hb;
        if (r_lo < 0) r_lo = 0;
        if (r_hi > a.H) r_hi = a.H;
        const int ys = r_lo + yr;
        const int Yt = gs * a.Hs + a.pad + ys - Y0;
        const int left = a.N - gs * V;
        const int nv = left < V ? left : V;
        const bool ok = u < units && gs < a.ngroups && ys < r_hi;
        src = ok ? gs * V * img_stride + c * chan_stride + ys * a.W + xx : -1;
        dc = ok ? ((c * a.CS + Yt * a.Wp + a.pad + xx) | (c << 17) | ((nv - 1) << 28)) : 0;
    };
    const int round_units = kStage * nthreads;

    // Per (channel block, chunk, wavefront) descriptor: first plan entry, then the
    // batch count of each of the KW rows; the KW segments are contiguous in the
    // entry table.  The descriptor of the next chunk and the first batch of this
    // chunk are requested before staging starts, so their latency is hidden.
    const SC_CONSTANT int* sg = as_constant(a.seg) + ((size_t)kb * a.nchunks * a.WK + wk) * (KW + 1);
    const size_t sg_step = (size_t)a.WK * (KW + 1);
    int d_start = sg[0];
    int d_nb[KW];
#pragma unroll
    for (int kk = 0; kk < KW; ++kk) d_nb[kk] = sg[1 + kk];

    for (int ch = 0; ch < a.nchunks; ++ch) {
        const SC_CONSTANT Entry* e = as_constant(a.entries) + d_start;
        int nb[KW];
#pragma unroll
        for (int kk = 0; kk < KW; ++kk) nb[kk] = d_nb[kk];
        Entry cur[kBatch];
#pragma unroll
        for (int u = 0; u < kBatch; ++u) {  // the table ends in kBatch slack entries
            cur[u].wbits = e[u].wbits;
            cur[u].off = e[u].off;
        }
        if (ch + 1 < a.nchunks) {
            sg += sg_step;
            d_start = sg[0];
#pragma unroll
            for (int kk = 0; kk < KW; ++kk) d_nb[kk] = sg[1 + kk];
        }

        __syncthreads();  // zero fill done / previous chunk fully consumed
        // ---- stage the chunk: all loads of a round are issued before the first LDS write
        const int c0 = ch * a.Cc;
        const int cn = (a.C - c0) < a.Cc ? (a.C - c0) : a.Cc;
        const T* __restrict__ xc = x + (size_t)c0 * chan_stride;
        for (int r0 = 0; r0 < units; r0 += round_units) {
            int src[kStage], dc[kStage];
#pragma unroll
            for (int t = 0; t < kStage; ++t) {
                decode(r0 + tid + t * nthreads, src[t], dc[t]);
                if (((dc[t] >> 17) & 0x7ff) >= cn) src[t] = -1;
            }
            vec val[kStage];
#pragma unroll
            for (int t = 0; t < kStage; ++t) {
                const int nv = ((dc[t] >> 28) & 7) + 1;
#pragma unroll
                for (int v = 0; v < V; ++v)
                    VT::set(val[t], v, (src[t] >= 0 && v < nv) ? xc[(size_t)src[t] + (size_t)v * img_stride] : T(0));
            }
#pragma unroll
            for (int t = 0; t < kStage; ++t)
                if (src[t] >= 0) tile[dc[t] & 0x1ffff] = val[t];
        }
        __syncthreads();

        // ---- gather-FMA over this wavefront's KW rows
#pragma unroll
        for (int kk = 0; kk < KW; ++kk) {
            for (int b = 0; b < nb[kk]; ++b) {
                vec xv[kBatch];
#pragma unroll
                for (int u = 0; u < kBatch; ++u)  // entry offsets are in bytes: one VOP2 add per read
                    xv[u] = *reinterpret_cast<const vec*>(smem + (lposb + cur[u].off));
                e += kBatch;
                Entry nxt[kBatch];  // look-ahead fetch of the next batch (possibly the next row's first)
#pragma unroll
                for (int u = 0; u < kBatch; ++u) {
                    nxt[u].wbits = e[u].wbits;
                    nxt[u].off = e[u].off;
                }
                __builtin_amdgcn_sched_barrier(0);  // keep the LDS reads ahead of the arithmetic
#pragma unroll
                for (int u = 0; u < kBatch; ++u) {
                    const float w = __uint_as_float(cur[u].wbits);
#pragma unroll
                    for (int v = 0; v < V; ++v)
                        acc[kk][v] = __builtin_fmaf(w, (float)VT::get(xv[u], v), acc[kk][v]);
                }
#pragma unroll
                for (int u = 0; u < kBatch; ++u) cur[u] = nxt[u];
            }
        }
    }

    // ---- store: one writer per output element
    if (valid) {
        T* __restrict__ y = static_cast<T*>(a.y);
        const SC_CONSTANT int* kr = as_constant(a.krow) + ((size_t)kb * a.WK + wk) * KW;
        const size_t plane = (size_t)a.E * a.F;
        const size_t pix = (size_t)oi * a.F + oj;
#pragma unroll
        for (int kk = 0; kk < KW; ++kk) {
            const int k = kr[kk];
            if (k < 0) continue;
#pragma unroll
            for (int v = 0; v < V; ++v) {
                const int n = g * V + v;
                if (n < a.N) y[((size_t)n * a.K + k) * plane + pix] = (T)acc[kk][v];
            }
        }
    }
}

namespace {

template <typename T, int V, int KW>
int launch_one(const KernelArgs& a, int grid, int threads, int lds_bytes, hipStream_t s)
{
    auto fn = tile_kernel<T, V, KW>;
    if (lds_bytes > 64 * 1024) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(fn),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes);
        if (e != hipSuccess) return (int)e;
    }
    hipLaunchKernelGGL(fn, dim3(grid), dim3(threads), lds_bytes, s, a);
    return (int)hipGetLastError();
}

template <typename T, int V>
int launch_kw(int KW, const KernelArgs& a, int grid, int threads, int lds, hipStream_t s)
{
    switch (KW) {
        case 1: return launch_one<T, V, 1>(a, grid, threads, lds, s);
        case 2: return launch_one<T, V, 2>(a, grid, threads, lds, s);
        case 4: return launch_one<T, V, 4>(a, grid, threads, lds, s);
        case 8: return launch_one<T, V, 8>(a, grid, threads, lds, s);
        case 16: return launch_one<T, V, 16>(a, grid, threads, lds, s);
    }
    return (int)hipErrorInvalidValue;
}

}  // namespace

int launch_tile_kernel(int dtype, int V, int KW, const KernelArgs& a, int grid, int threads,
                       int lds_bytes, void* stream)
{
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (dtype == 0) {
        switch (V) {
            case 1: return launch_kw<float, 1>(KW, a, grid, threads, lds_bytes, s);
            case 2: return launch_kw<float, 2>(KW, a, grid, threads, lds_bytes, s);
            case 4: return launch_kw<float, 4>(KW, a, grid, threads, lds_bytes, s);
        }
    } else {
        switch (V) {
            case 1: return launch_kw<_Float16, 1>(KW, a, grid, threads, lds_bytes, s);
            case 2: return launch_kw<_Float16, 2>(KW, a, grid, threads, lds_bytes, s);
            case 4: return launch_kw<_Float16, 4>(KW, a, grid, threads, lds_bytes, s);
            case 8: return launch_kw<_Float16, 8>(KW, a, grid, threads, lds_bytes, s);
        }
    }
    return (int)hipErrorInvalidValue;
}

}  // namespace sc
