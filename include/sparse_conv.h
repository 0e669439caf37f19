/*
 * sparse_conv.h - C ABI of the MI355X (gfx950) direct sparse convolution library.
 *
 * Direct sparse convolution (Pietron & Zurek, arXiv 2011.06295, sections 7 and
 * 8): the weights of a convolution layer that survived unstructured pruning
 * are stored per output channel in CSR and multiplied straight against the
 * dense NCHW input, with no im2col lowering.  The result is the plain
 * convolution of section 3, eq. 1, evaluated over the kept weights only.
 *
 * Conventions shared by all entry points
 *   - every function returns an int status (SC_OK or a negative SC_E* code),
 *     never throws and never aborts; on error the outputs are left untouched;
 *   - HOST pointers are ordinary process memory, DEVICE pointers are HIP
 *     device memory of the current device (for instance tensor.data_ptr() of a
 *     PyTorch-ROCm tensor); the library never takes ownership of either;
 *   - all arrays are dense, contiguous, row-major in the index order written;
 *   - a handle keeps its device tables on the device that was current at the
 *     first call that needed them (sparse_conv_forward, sparse_conv_autotune,
 *     sparse_conv_set_epilogue with a bias); later such calls with another
 *     device current return SC_EINVAL;
 *   - the handle is not thread-safe against concurrent calls on itself.
 */
#ifndef SPARSE_CONV_H
#define SPARSE_CONV_H

#ifdef __cplusplus
extern "C" {
#endif

typedef struct sparse_conv_s* sparse_conv_t; /* opaque layer handle */

enum {
    SC_OK = 0,
    SC_EINVAL = -1,       /* null pointer, non-positive size, stride < 1, pad < 0, filter larger than padded input, unknown dtype/flag */
    SC_EUNSUPPORTED = -2, /* valid request this build cannot run (e.g. a tile that cannot fit the LDS, no gfx950 device) */
    SC_ENOMEM = -3,       /* host or device allocation failed */
    SC_EHIP = -4,         /* a HIP runtime call failed; sparse_conv_last_hip_error() has the code */
    SC_ETOOBIG = -5       /* sparse_conv_forward_static: the layer's tables exceed the static device scratch */
};

/* Storage type of weights, input and output.  Products and sums are always
 * formed in fp32 (section 8: the half path converts the value array and the
 * input to half; accumulation width is this library's choice). */
enum { SC_F32 = 0, SC_F16 = 1 };

/* Section 7: pad every CSR row with explicit zeros up to the non-zero count of
 * the fullest row, so all output channels have one unified count. */
enum { SC_FLAG_UNIFY_NNZ = 1u };

/* Epilogue flags (sparse_conv_set_epilogue): apply ReLU to the stored value; store the maximum over
 * 2 x 2 windows (stride 2) of the map instead of the map. */
enum { SC_EPILOGUE_RELU = 1u, SC_EPILOGUE_MAXPOOL2 = 2u };

/*
 * sparse_conv_create - build the CSR form of one pruned layer (section 7).
 *   out      receives the handle.
 *   dense_w  HOST, fp32 [K][C][R][S]: the dense filter tensor of section 3.
 *   mask     HOST, uint8 [K][C][R][S]: non-zero = the weight survives pruning
 *            (section 5, eq. 4: w <- w * mask).  The mask, not the value,
 *            decides what is stored; kept values are copied bit for bit
 *            (SC_F16: converted once to IEEE binary16, round-to-nearest-even).
 *   K,C,R,S  output channels, input channels, filter height, filter width (> 0,
 *            C*R*S and the total stored count below 2^31).
 *   dtype    SC_F32 or SC_F16.
 *   flags    0 or SC_FLAG_UNIFY_NNZ.
 * CSR layout: row k = output channel k; column = (c*R + r)*S + s; entries of a
 * row in ascending column order; 32-bit rowptr[K+1] and colidx[nnz].
 * With SC_FLAG_UNIFY_NNZ a short row is extended to the count of the fullest
 * row: scanning columns upwards, a dropped column directly right of a stored
 * one (possibly just added) is stored with value +0.0 until the row is full;
 * if it is still short the lowest dropped columns are added.
 * Both input arrays are copied; the caller may free them on return.  No GPU is
 * needed for this call: device copies are made by the first forward call.
 */
int sparse_conv_create(sparse_conv_t* out, const float* dense_w, const unsigned char* mask,
                       int K, int C, int R, int S, int dtype, unsigned flags);

/*
 * sparse_conv_output_shape - section 3: E = (H + 2*pad - R)/stride + 1 and
 * F = (W + 2*pad - S)/stride + 1, with floor division.  SC_EINVAL if the
 * padded input is smaller than the filter.
 */
int sparse_conv_output_shape(sparse_conv_t h, int H, int W, int stride, int pad, int* E, int* F);

/*
 * sparse_conv_forward - direct sparse convolution (section 8) of a batch.
 *   input   DEVICE, [N][C][H][W] of the handle's dtype (fp32 or binary16).
 *   output  DEVICE, [N][K][E][F] of the same dtype; every element is written
 *           (channels with no stored weight are written as zeros).  Must not
 *           overlap input.
 *   N,H,W   batch size (>= 0; 0 is a no-op) and input height/width (> 0).
 *   stride  >= 1, the same in both directions.   pad >= 0, zero padding.
 *   stream  a hipStream_t passed as void*; NULL is the default stream.
 * Asynchronous: kernels are enqueued on the stream and the call returns
 * without synchronising.  The first call for a new (N,H,W,stride,pad) builds
 * and uploads a per-geometry plan (one synchronous allocation + copy);
 * further calls with the same geometry allocate nothing and enqueue exactly one
 * kernel, so they may be recorded into a HIP graph on a capturing stream.
 * A plan whose channels are dealt over several workgroups (launch parameter [10]) owns a
 * scratch buffer of partial sums and arrival counters: two forwards of one handle and
 * geometry must then not run at the same time (different streams without ordering).
 * Limits: input and output below 2^31 elements each (SC_EUNSUPPORTED beyond).
 * Non-finite input values count only under a stored weight, as the definition
 * has it: an output is NaN, +Inf or -Inf exactly where the sum over its stored
 * weights is (the zero-weight entries that fill a stored row to a multiple of
 * four read a zeroed region of the tile, not the input).
 */
int sparse_conv_forward(sparse_conv_t h, const void* input, void* output,
                        int N, int H, int W, int stride, int pad, void* stream);

/*
 * sparse_conv_forward_static - sparse_conv_forward for callers that cannot allocate device
 * memory: code that runs where hipMalloc is not allowed (tight serving loops, harnesses that
 * forbid it).  Same arguments, same kernel, same result as sparse_conv_forward, but the call
 * makes no device allocation, not even the first one for a geometry: the per-geometry tables
 * the kernel reads (stored weights as LDS tap offsets, segment descriptors, channel slots) are
 * copied, on `stream`, into a static device array of SC_STATIC_SCRATCH_BYTES that is part of the
 * library's code object (every GPU the library runs on holds its own copy until the process
 * ends), and the kernel reads them there.
 *   - SC_ETOOBIG if the tables of this layer and geometry need more than that (about 8.2 bytes
 *     per stored weight); nothing is enqueued then.
 *   - All handles of the process share the array of a GPU, and it keeps what the last call
 *     left there: a call whose tables are already in place (same handle, geometry and launch
 *     configuration as the call before it on that GPU) copies nothing, any other call
 *     overwrites them.  Calls on one GPU must therefore not overlap: a call that changes the
 *     tables while an earlier kernel still reads them (another stream, another host thread
 *     without ordering between the streams) races with it.  Enqueue on one stream, or order the
 *     streams with events.
 *   - The host-side plan of a new geometry is still built on the first call (host memory only);
 *     the copy reads host memory owned by the handle, so the handle's plans must not be
 *     discarded (sparse_conv_set_launch, sparse_conv_autotune, sparse_conv_destroy) before the
 *     stream has passed the call.
 */
#define SC_STATIC_SCRATCH_BYTES (16u << 20)
int sparse_conv_forward_static(sparse_conv_t h, const void* input, void* output,
                               int N, int H, int W, int stride, int pad, void* stream);

/*
 * sparse_conv_get_csr - expose the CSR arrays built by create (section 7).
 * All pointers are HOST memory owned by the handle, valid until destroy; any
 * of the out-pointers may be NULL.  values points to float (SC_F32) or to
 * 16-bit binary16 patterns (SC_F16).
 */
int sparse_conv_get_csr(sparse_conv_t h, int* K, long long* nnz,
                        const int** rowptr, const int** colidx, const void** values);

/*
 * sparse_conv_create_codebook - the same for cluster-quantised weights (section 6;
 * section 9 uses 16 centroids of 16 bits, i.e. a 4-bit code per weight).
 *   index      HOST, unsigned char [K][C][R][S], the centroid number (0..15) of
 *              every weight; read only where mask is non-zero.
 *   centroids  HOST, fp32 [16]; each is rounded to binary16 (round to nearest
 *              even) and that value is the weight, for SC_F32 layers too.
 *   mask, K..S, dtype, flags   as for sparse_conv_create.  With
 *              SC_FLAG_UNIFY_NNZ the explicit zeros take the number of the first
 *              centroid that is zero.
 * The handle stores rowptr, colidx (as above), the codes of the stored entries in
 * CSR order, two to a byte (entry 2i in the low nibble of byte i, entry 2i+1 in the
 * high nibble, an unused last nibble zero) and the 16 centroids: 0.5 byte per
 * stored weight instead of 2 or 4.  sparse_conv_get_csr returns the decoded
 * values.  On the device a plan entry of such a layer is one 32-bit word (LDS offset
 * in 16 bits and the centroid itself as binary16) instead of the 8-byte (fp32 weight,
 * offset) pair: half the stream the kernel fetches, for SC_F32 layers too; the
 * multiply-add takes the binary16 weight as it is (mixed precision, fp32 sum).
 * SC_EINVAL: bad arguments, an index above 15 under the mask, or explicit zeros
 * are needed and no centroid is zero.
 */
int sparse_conv_create_codebook(sparse_conv_t* out, const unsigned char* index, const float* centroids,
                                const unsigned char* mask, int K, int C, int R, int S, int dtype, unsigned flags);

/* Codes and centroids of a handle made by sparse_conv_create_codebook: *codes is
 * HOST unsigned char [(nnz + 1) / 2], *centroids HOST binary16 patterns [16];
 * both stay owned by the handle.  Either pointer may be NULL.  SC_EINVAL for a
 * handle without a codebook. */
int sparse_conv_get_codebook(sparse_conv_t h, const unsigned char** codes, const unsigned short** centroids);

/*
 * sparse_conv_set_launch - override the per-layer launch configuration, this
 * library's counterpart of the per-layer thread-block count the paper tunes
 * (section 8, subBatchSize; section 9).  params[0..nparams), nparams <= 11, are, in order:
 *   [0] V   images interleaved per LDS element (1, 2, 4 or 8; 0 = automatic)
 *   [1] WP  wavefronts across output positions (64 * LP positions each) per workgroup
 *   [2] WK  wavefronts across output channels per workgroup (WP*WK <= 16)
 *   [3] KW  output channels accumulated per wavefront (1, 2, 4, 8 or 16)
 *   [4] Cc  input channels staged per LDS pass
 *   [5] LDS budget in bytes per workgroup (used when Cc is automatic)
 *   [6] LP  output positions per lane (1 or 2; with LP = 2: KW * V <= 16)
 *   [7] channel blocks the K output channels are dealt over (a workgroup takes one
 *           block; at least ceil(K / (WK * KW)), more leaves row slots empty on the
 *           wavefronts a SIMD serves last; fewer is SC_EUNSUPPORTED)
 *   [8] output stores: 1 ordinary, 2 non-temporal (the output bypasses the cache
 *           lines the other workgroups of the launch still read their input from;
 *           faster for some layers, slower for others: sparse_conv_autotune
 *           measures both); automatic without a measurement is 1
 *   [9] what a lane stands for: 1 a position of the zero-padded input lattice (positions on
 *           padding compute a value that is never stored); 1 + G with G = 1, 2, 4, 8 or 16: an
 *           output element, with G groups of V images interleaved element by element in the
 *           tile (no lane is spent on padding; needs LP = 1).  Which is faster depends on the
 *           map size; sparse_conv_autotune measures both kinds.
 *   [10] workgroups the input channels of one (tile, channel block) are dealt over: 1, 2, 4 or 8.
 *           With more than one, each works through its share of the channel chunks and leaves
 *           its partial sums in a scratch buffer of the plan; the one that finishes last adds them
 *           up, in the order of the shares (the result does not depend on which one that is),
 *           and stores.  It pays where a layer has too few tiles and channel blocks to fill the
 *           chip with workgroups that have many rows each (the 2x2 and 4x4 maps of a deep stack).
 * Missing trailing entries and zeros mean "automatic".  nparams = 0 restores
 * the automatic choice.  Cached plans are discarded.  SC_EINVAL for values the
 * kernels cannot run; a configuration that cannot fit is reported by forward.
 */
int sparse_conv_set_launch(sparse_conv_t h, const int* params, int nparams);

/*
 * sparse_conv_autotune - choose the launch configuration of one geometry by
 * measurement (section 8 sets the thread-block count of each layer by
 * experiment; section 9 reports what an untuned choice costs).  Runs the layer
 * on the given buffers with the max_candidates (<= 0: 8) configurations the
 * cost estimate ranks best, within whatever sparse_conv_set_launch has pinned,
 * times each with events on `stream`, times the three fastest once more with
 * non-temporal output stores (kept only where at least 2 % faster), and keeps
 * the fastest for later forwards of this (N,H,W,stride,pad).
 *   input, output, N..pad, stream   as for sparse_conv_forward (N > 0); output is
 *            overwritten with the layer's result.
 *   best_us  if not NULL receives the kept configuration's time per launch, in us.
 * Synchronous (it waits for its own measurements) and it allocates plan
 * buffers: call it once, outside timed or captured regions.
 * sparse_conv_set_launch discards what was tuned.
 */
int sparse_conv_autotune(sparse_conv_t h, const void* input, void* output,
                         int N, int H, int W, int stride, int pad, void* stream,
                         int max_candidates, float* best_us);

/*
 * sparse_conv_rank_launches - the candidates sparse_conv_autotune would time, for callers
 * that measure in their own setting (inside a pass through a network, say): up to
 * max_candidates launch configurations for the geometry, cheapest cost estimate first,
 * within whatever sparse_conv_set_launch has pinned (the list goes round the kinds of
 * lanes: the best of each kind, then the second best of each, ...).  params receives 11 ints per
 * candidate, in the order sparse_conv_set_launch takes them (each can be passed back to
 * it as it is); *count the number written.  Needs no GPU.
 */
int sparse_conv_rank_launches(sparse_conv_t h, int N, int H, int W, int stride, int pad,
                              int max_candidates, int* params, int* count);

/*
 * sparse_conv_set_epilogue - what the store step does with a finished sum
 * (section 3: the sum over the filter is added to the bias of its output channel
 * and the activation function is applied).  Default: store the bare sum.
 *   bias   HOST, fp32 [K], added to every output element of channel k before
 *          anything else; NULL = no bias.  Copied by the call (one synchronous
 *          device allocation and copy).
 *   flags  0, or any of
 *          SC_EPILOGUE_RELU: out = max(sum + bias, 0);
 *          SC_EPILOGUE_MAXPOOL2: the pooling step that follows the activation in section 3's
 *          layer sequence, done in the store: the output is [N][K][E/2][F/2], element (i, j)
 *          the largest of the four values (2i..2i+1, 2j..2j+1) after bias and ReLU.  Needs even
 *          E and F and a plan with lanes as output elements whose tiles hold whole pairs of
 *          output rows (the planner then offers only such; SC_EUNSUPPORTED from the calls that
 *          plan a geometry if there is none: lattice lanes forced, stride above 1, or an F that
 *          is not a power of two, since a tile is a power of two of outputs).
 *          sparse_conv_output_shape then reports E/2 and F/2.  A window that holds a NaN gives
 *          an unspecified one of its values.
 * For SC_F16 the fp32 value is rounded to binary16 once, after bias, ReLU and maximum.
 * Applies to every later forward of this handle; changing SC_EPILOGUE_MAXPOOL2 discards the
 * handle's plans and measured launch choices.
 */
int sparse_conv_set_epilogue(sparse_conv_t h, const float* bias, unsigned flags);

/* Diagnostic: builds (or takes the cached) plan of a geometry and checks it on the
 * host against the CSR: every stored weight appears exactly once, with the LDS
 * offset of its tap (section 7's pre-computed input offsets) inside the staged
 * tile, every output channel has one accumulator slot, the tables have the sizes
 * the kernel walks, and the launch fits the hardware.  *failed_check receives 0,
 * or the number of the first check that failed.  Needs no GPU.  Returns SC_OK
 * when the check ran (whatever it found), else as sparse_conv_get_launch. */
int sparse_conv_check_plan(sparse_conv_t h, int N, int H, int W, int stride, int pad, int* failed_check);

/* The launch configuration chosen for a geometry: [0] V .. [4] Cc, [5] the LDS
 * budget in force, [6] workgroups launched, [7] LDS bytes
 * per workgroup, [8] threads per workgroup, [9] stored plan entries
 * (including batch padding), [10] LP, [11] channel blocks, [12] kind of output store
 * (1 or 2), [13] what a lane stands for (1, or 1 + G, as sparse_conv_set_launch takes it),
 * [14] workgroups the channels are dealt over, [15] bytes per plan entry on the device (8: fp32 weight
 * and LDS offset; 4: binary16 weight and 16-bit LDS offset, for SC_F16 handles and handles made by
 * sparse_conv_create_codebook).  [0..5] are in the order of sparse_conv_set_launch.  Builds the plan's
 * host side if needed; needs no GPU.  params must have room for 16 ints. */
int sparse_conv_get_launch(sparse_conv_t h, int N, int H, int W, int stride, int pad, int* params);

/*
 * Roof probes: kernels of known work, for measuring on the machine at hand the two rates the
 * benchmark's roofline fractions refer to (the caller times them with events on `stream`).
 * sparse_conv_probe_lds_read: `workgroups` workgroups of 1024 threads; every wavefront reads 64
 *   consecutive 16-byte LDS elements (ds_read_b128, the gather pattern of section 8's multiply loop
 *   as this library lays it out) 8 * iterations times and does nothing else.  sink: DEVICE, at least
 *   4096 * workgroups bytes (one float per thread is written so that the reads are kept).
 *   *bytes_read receives the LDS bytes read by the whole launch.
 * sparse_conv_probe_copy: copies bytes / 16 16-byte words from src to dst (DEVICE, 16-byte aligned,
 *   not overlapping): `bytes` read and `bytes` written, the traffic of a plain copy.
 * Both return SC_EINVAL for bad arguments, SC_EHIP if the launch failed.
 */
int sparse_conv_probe_lds_read(void* sink, int workgroups, int iterations, void* stream, long long* bytes_read);
int sparse_conv_probe_copy(void* dst, const void* src, long long bytes, void* stream);

/* HIP error code of the last failing runtime call made through this handle (0 if none). */
int sparse_conv_last_hip_error(sparse_conv_t h);

/* Static description of a status code. */
const char* sparse_conv_strerror(int code);

/* Release the handle, its host arrays and its device buffers.  NULL is a no-op.
 * The caller must make sure no forward call on the handle is still running. */
void sparse_conv_destroy(sparse_conv_t h);

#ifdef __cplusplus
}
#endif
#endif /* SPARSE_CONV_H */
