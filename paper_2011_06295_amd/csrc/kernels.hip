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
    // the 8 XCDs; all channel blocks of one tile are kept on one XCD so the
    // tile's input is fetched into a single L2.
    const int bid = blockIdx.x;
    const int xcd = bid & 7;
    const int qb = bid >> 3;
    const int kb = qb % a.kblocks;
    const int tile_id = (qb / a.kblocks) * 8 + xcd;
    if (tile_id >= a.ntiles) return;

    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int nwaves = nthreads >> 6;
    const int lane = tid & 63;
    const int wp = wave % a.WP;
    const int wk = wave / a.WP;

    // The tile covers lattice positions [q0, q0 + span); its row 0 is lattice row Y0.
    const long long q0 = (long long)tile_id * a.span;
    const int Y0 = (int)(q0 / a.Wp);
    const int lq0 = (int)(q0 - (long long)Y0 * a.Wp);

    // lane -> position -> output element (if any)
    const int lpos = lq0 + wp * 64 + lane;      // tile-local element index of the position
    const int Yl = lpos / a.Wp;
    const int X = lpos - Yl * a.Wp;
    const int Y = Y0 + Yl;
    const int g = Y / a.Hs;
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
    const size_t chan_stride = (size_t)a.H * a.W;
    const size_t img_stride = (size_t)a.C * chan_stride;
    const int hbw = a.Hb * a.W;

    for (int ch = 0; ch < a.nchunks; ++ch) {
        __syncthreads();  // zero fill done / previous chunk fully consumed
        // ---- stage the chunk.  A lane owns fixed (row, column) cells of the tile
        // and walks the channels assigned to its wavefront; consecutive lanes read
        // consecutive input elements of V images and write one V-vector each.
        const int c0 = ch * a.Cc;
        const int cn = (a.C - c0) < a.Cc ? (a.C - c0) : a.Cc;
        for (int cell = lane; cell < hbw; cell += 64) {
            const int Yt = cell / a.W;
            const int xx = cell - Yt * a.W;
            const int Ys = Y0 + Yt;
            const int gs = Ys / a.Hs;
            const int ys = Ys - gs * a.Hs - a.pad;
            if (gs >= a.ngroups || ys < 0 || ys >= a.H) continue;  // a zero row
            const int n0 = gs * V;
            const T* src = x + (size_t)n0 * img_stride + (size_t)c0 * chan_stride + (size_t)ys * a.W + xx;
            vec* dst = tile + Yt * a.Wp + a.pad + xx;
            int c = wave;
            for (; c + 3 * nwaves < cn; c += 4 * nwaves) {
                vec val[4];
#pragma unroll
                for (int t = 0; t < 4; ++t)
#pragma unroll
                    for (int v = 0; v < V; ++v)
                        VT::set(val[t], v, (n0 + v) < a.N ? src[(size_t)v * img_stride + (size_t)(c + t * nwaves) * chan_stride] : T(0));
#pragma unroll
                for (int t = 0; t < 4; ++t) dst[(size_t)(c + t * nwaves) * a.CS] = val[t];
            }
            for (; c < cn; c += nwaves) {
                vec val;
#pragma unroll
                for (int v = 0; v < V; ++v)
                    VT::set(val, v, (n0 + v) < a.N ? src[(size_t)v * img_stride + (size_t)c * chan_stride] : T(0));
                dst[(size_t)c * a.CS] = val;
            }
        }
        __syncthreads();

        // ---- gather-FMA over this wavefront's KW rows
        const SC_CONSTANT int* sg = as_constant(a.seg) + (((size_t)kb * a.nchunks + ch) * a.WK + wk) * (KW * 2);
#pragma unroll
        for (int kk = 0; kk < KW; ++kk) {
            const int start = sg[2 * kk];
            const int nb = sg[2 * kk + 1];
            const SC_CONSTANT Entry* e = as_constant(a.entries) + start;
            Entry cur[kBatch];
#pragma unroll
            for (int u = 0; u < kBatch; ++u) {  // the table ends in kBatch slack entries
                cur[u].wbits = e[u].wbits;
                cur[u].off = e[u].off;
            }
            for (int b = 0; b < nb; ++b) {
                vec xv[kBatch];
#pragma unroll
                for (int u = 0; u < kBatch; ++u) xv[u] = tile[lpos + cur[u].off];
                e += kBatch;
                Entry nxt[kBatch];  // look-ahead fetch of the next batch
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
