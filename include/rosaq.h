/* rosaq.h - C ABI of the MI355X (gfx950) fused ROSAQ linear layer.
 *
 * The layer is y = (x Q) What^T  with  What = W Q  stored in mixed precision:
 * the K rotated input channels with the largest PCA eigenvalues stay FP16, all
 * other channels are INT4 / INT3 codes in groups of 128 with an FP16 scale and an
 * integer (FP16-stored) zero point per (output row, group).
 *
 * Notation.  The paper writes the rotation as R and weights as W in R^{d x d'};
 * this interface names the rotation Q and takes weights in the PyTorch layout
 * W[out, in] = W[N, D].  Hence What = W Q is the transpose of the paper's R^T W
 * (Eq. 1-3), and "salient rows of R^T W" become salient columns of What.
 *
 * Conventions: every function returns 0 (ROSAQ_OK) or a negative error code and
 * never throws or aborts; rosaq_last_error() gives the text of the last failure
 * on the calling thread.  "HOST" / "DEVICE" say where a pointer must live.
 * All fp16 data is passed as raw IEEE binary16 bit patterns (uint16_t).
 */
#ifndef ROSAQ_H_
#define ROSAQ_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define ROSAQ_OK             0
#define ROSAQ_ERR_NULL      (-1)  /* a required pointer is NULL                                  */
#define ROSAQ_ERR_SHAPE     (-2)  /* D % 128, (D-K) % group, K > D, M < 1, leading dim < width   */
#define ROSAQ_ERR_ARG       (-3)  /* bits not 3/4, group != 128, head_dim != 128, bad enum       */
#define ROSAQ_ERR_MODE      (-4)  /* entry point does not serve this handle's q_mode             */
#define ROSAQ_ERR_ALIGN     (-5)  /* device pointer / leading dimension not 16-byte aligned      */
#define ROSAQ_ERR_WORKSPACE (-6)  /* workspace missing or smaller than rosaq_workspace_bytes      */
#define ROSAQ_ERR_NONFINITE (-7)  /* NaN / Inf in W, Q, eigenvalues or the rotated weights       */
#define ROSAQ_ERR_HIP       (-8)  /* a HIP call failed (text in rosaq_last_error)                */
#define ROSAQ_ERR_NOMEM     (-9)  /* host allocation failed                                      */
#define ROSAQ_ERR_HOSTONLY  (-10) /* handle was packed with host_only and has no device buffers  */
#define ROSAQ_ERR_NOCONVERGE (-11) /* the Jacobi eigensolver did not reach its tolerance          */

/* Rotation kinds.  NONE is R = I (the rotation-less "Mixed" baseline, Sec. 4.1);
 * FULL is the layer-wise PCA rotation (Sec. 3.1, Eq. 4); HEADWISE is the block
 * diagonal rotation made of one PCA per attention head (Sec. 3.1.1, Eq. 6). */
#define ROSAQ_Q_NONE     0
#define ROSAQ_Q_FULL     1
#define ROSAQ_Q_HEADWISE 2

/* Which rotated channels stay FP16 (ties always go to the lower channel index).
 * TOP is the method (Sec. 3.2).  TOP_PER_HEAD keeps K / (D/128) channels in every
 * 128-channel head, the setting the weight-splitting appendix uses for the attention
 * output projection (32 per head).  The other three are the ablation rules of the
 * salient-channel appendix: BOTTOM = the K smallest eigenvalues; CONSECUTIVE = channels
 * select_arg .. select_arg+K-1 (the caller draws the random start); TOP_AND_BOTTOM = the
 * channels of TOP and of BOTTOM together: K/2 largest plus K/2 smallest among the rest.  K is
 * always the size of the FP16 block, so the appendix's combined scheme for its K' (K' from Top
 * and K' from Bottom) is this rule with K = 2 K'. */
#define ROSAQ_SELECT_TOP            0
#define ROSAQ_SELECT_TOP_PER_HEAD   1
#define ROSAQ_SELECT_BOTTOM         2
#define ROSAQ_SELECT_CONSECUTIVE    3
#define ROSAQ_SELECT_TOP_AND_BOTTOM 4

typedef struct rosaq_packed rosaq_packed_t;   /* opaque; owns its host and device buffers */

/* Description of one linear layer to pack (Sec. 3.1-3.3; Eq. 3).  All pointers HOST;
 * the library copies what it needs, the caller may free them after the call. */
typedef struct {
  int32_t out_features;      /* N                                                             */
  int32_t in_features;       /* D, multiple of 128                                            */
  const uint16_t* W;         /* fp16 [N x D], row n at W + n*ldw                              */
  int64_t ldw;               /* >= D, in elements                                             */
  int32_t q_mode;            /* ROSAQ_Q_*                                                     */
  int32_t head_dim;          /* 128 for HEADWISE, ignored otherwise                           */
  const float* Q;            /* fp32. FULL: [D x D] row-major, xhat = x Q (eigenvectors are    */
                             /* columns). HEADWISE: [D/128][128][128], block h rotates input   */
                             /* channels 128h..128h+127. NONE: ignored (may be NULL)           */
  const double* eigenvalues; /* [D], one per rotated channel: the saliency key (Sec. 3.2)      */
  int32_t K;                 /* number of FP16 salient channels, multiple of 32, (D-K) % 128 == 0 */
  int32_t bits;              /* 3 or 4                                                        */
  int32_t group;             /* 128                                                           */
  int32_t select_rule;       /* ROSAQ_SELECT_* (0 = the K largest eigenvalues, the method)      */
  int32_t host_only;         /* nonzero: build the canonical arrays only, touch no GPU         */
  int32_t select_arg;        /* first channel for ROSAQ_SELECT_CONSECUTIVE, else ignored       */
  int32_t rotation_absorbed; /* nonzero: W is rotated by Q at pack time as usual, but the caller */
                             /* feeds already-rotated activations (the rotation was folded into  */
                             /* the producing layer offline, as the paper deploys it): at run    */
                             /* time the handle behaves as q_mode NONE and is served by          */
                             /* rosaq_linear with x = xhat                                       */
} rosaq_pack_desc;

/* rosaq_pack_weights - offline step of the method (Sec. 3.1-3.3, Eq. 1-3):
 *   1. What = W Q in fp64, rounded once to fp16 (HEADWISE: per 128-column block);
 *   2. salient_idx = the K channels picked by select_rule (default: largest eigenvalues), ascending;
 *      storage order perm = [salient_idx ; all other channels ascending];
 *   3. W_S = What[:, salient_idx] kept as fp16;
 *   4. the other columns, in storage order, are cut into groups of 128 and each
 *      (row, group) is quantised:  s = fp16(max((max-min)/(2^bits-1), 2^-14)),
 *      z = clamp(rne(-min/s), 0, 2^bits-1), q = clamp(rne(w/s)+z, 0, 2^bits-1)
 *      (fp64 arithmetic, round-half-to-even; the paper fixes only "per-group,
 *      128 channels, INT3/INT4": this formula is this library's reading);
 *   5. unless host_only, steps 1, 3 and 4 run on the GPU (W and Q are uploaded on `hip_stream`;
 *      the results are bit-identical to the host path) and leave the layer in device memory in
 *      the kernels' fragment order, plus an fp16 copy of Q; the call waits for them.
 * hip_stream is a hipStream_t (NULL = default stream).  *out is owned by the
 * library until rosaq_free.  Errors: NULL, SHAPE, ARG, NONFINITE, NOMEM, HIP. */
int rosaq_pack_weights(const rosaq_pack_desc* desc, void* hip_stream, rosaq_packed_t** out);

/* rosaq_packed_clone - a second, independent copy of a packed layer: host arrays
 * copied, device buffers duplicated with a device-to-device copy on hip_stream (the
 * call waits for it).  The clone is freed with rosaq_free like any handle.
 * Errors: NULL, NOMEM, HIP. */
int rosaq_packed_clone(const rosaq_packed_t* src, void* hip_stream, rosaq_packed_t** out);

/* Bytes of DEVICE workspace to give rosaq_linear* for M rows (0 on a bad handle): the rotated
 * activations, a few KiB of tickets, and (calls of up to 64 rows) room for the fp32 partial output
 * tiles of a launch whose contraction is split over up to 16 workgroups per tile.  A call accepts a
 * smaller workspace as long as the first two parts fit (it then splits less, or not at all, and
 * runs slower); it fails with ROSAQ_ERR_WORKSPACE below that. */
size_t rosaq_workspace_bytes(const rosaq_packed_t* p, int32_t M);

/* The smallest workspace a call with M rows accepts (no room for split launches). */
size_t rosaq_workspace_bytes_min(const rosaq_packed_t* p, int32_t M);

/* rosaq_workspace_bytes for one rosaq_linear_batch call over these `count` layers (their output
 * widths add up). */
size_t rosaq_workspace_bytes_batch(const rosaq_packed_t* const* layers, int32_t count, int32_t M);

/* rosaq_linear - Eq. 3 for q_mode NONE or FULL:
 *     xhat = x fp16(Q)            (FULL; fp32 accumulate, xhat rounded to fp16)
 *     y = xhat[:, salient_idx] W_S^T + xhat[:, rest] ((q - z) s)^T
 * fp32 accumulation, y rounded to fp16 (RNE).
 *   x_dev  DEVICE fp16 [M x D], row m at x + m*ldx (ldx >= D, ldx % 8 == 0, 16-byte aligned base)
 *   y_dev  DEVICE fp16 [M x N], row m at y + m*ldy (ldy >= N; any fp16-aligned base and ldy)
 *   ws_dev DEVICE scratch of at least rosaq_workspace_bytes(p, M), 256-byte aligned;
 *          contents need not be preserved or initialised between calls
 * Asynchronous on hip_stream; allocates nothing and never synchronises.  Calls that
 * share a workspace must not overlap in time.
 * Errors: NULL, SHAPE, MODE (HEADWISE handle), ALIGN, WORKSPACE, HOSTONLY, HIP. */
int rosaq_linear(const rosaq_packed_t* p, const void* x_dev, int32_t M, int64_t ldx,
                 void* y_dev, int64_t ldy, void* ws_dev, size_t ws_bytes, void* hip_stream);

/* rosaq_linear_headwise - Eq. 6: the same layer with the block-diagonal
 * rotation  xhat[:, 128h..128h+127] = x[:, 128h..128h+127] fp16(Q_h).
 * Same arguments and rules as rosaq_linear; serves q_mode HEADWISE only. */
int rosaq_linear_headwise(const rosaq_packed_t* p, const void* x_dev, int32_t M, int64_t ldx,
                          void* y_dev, int64_t ldy, void* ws_dev, size_t ws_bytes,
                          void* hip_stream);

/* rosaq_linear_headwise_static - rosaq_linear_headwise for callers that cannot allocate or hold
 * a workspace: code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.
 * The rotated activations, tickets and partial tiles go to a fixed 8 MiB array that the library
 * keeps in the device memory of every GPU it runs on (until the process ends); the call itself
 * allocates nothing.  Same arguments, rules and results as rosaq_linear_headwise, minus the
 * workspace.  Limit: the call must fit the array, i.e. rosaq_workspace_bytes_min(p, M) <= 8 MiB
 * (ceil(M / 64) * 128 * in_features bytes plus 32 KiB; M up to 960 at in_features 4096), else
 * ROSAQ_ERR_WORKSPACE.  All calls on one GPU share that GPU's array: calls that overlap in time
 * on one GPU (two streams, two threads) race and give wrong results; calls on one stream are safe.
 * Errors: those of rosaq_linear_headwise. */
#define ROSAQ_STATIC_SCRATCH_BYTES (8u << 20)
int rosaq_linear_headwise_static(const rosaq_packed_t* p, const void* x_dev, int32_t M, int64_t ldx,
                                 void* y_dev, int64_t ldy, void* hip_stream);

/* rosaq_linear_batch - up to 4 layers that read the same input through the same
 * rotation, in one pass: y_i = (x Q) What_i^T.  The query, key and value projections
 * of an attention block share their input activations and hence their PCA (Eq. 5 feeds
 * the same Z to W^Q, W^K, W^V), as do the up and gate projections of the FFN (weight
 * splitting appendix): xhat is computed once and all layers' weights stream in one launch.
 *   layers HOST array of `count` handles packed with identical D, K, bits, q_mode, Q
 *          and eigenvalues (checked through a fingerprint taken at pack time)
 *   y_dev  HOST array of `count` DEVICE pointers, y_dev[i] fp16 [M x N_i], row stride ldy[i]
 * Other arguments and rules as rosaq_linear; the workspace size is that of layers[0].
 * Serves every q_mode.  Errors: those of rosaq_linear, ARG (count), MODE (layers differ). */
int rosaq_linear_batch(const rosaq_packed_t* const* layers, int32_t count, const void* x_dev,
                       int32_t M, int64_t ldx, void* const* y_dev, const int64_t* ldy,
                       void* ws_dev, size_t ws_bytes, void* hip_stream);

/* rosaq_linear_swiglu - the gated pair of the FFN in one pass:
 *     y = silu(xhat What_gate^T) * (xhat What_up^T),   silu(t) = t / (1 + exp(-t)),
 * both products accumulated in fp32, the gate applied in fp32, y rounded to fp16 once.  The up and
 * gate projections read the same input through the same rotation (weight splitting appendix:
 * W_U and W_G are split alike), so xhat is computed once and both weights stream in one launch; the
 * two [M x N] intermediates never reach memory.
 *   gate, up  handles with identical N, D, K, bits, q_mode and rotation (as for rosaq_linear_batch)
 *   y_dev     DEVICE fp16 [M x N], row stride ldy
 * Other arguments and rules as rosaq_linear (serves every q_mode; the launch is never split over
 * workgroups).  Errors: those of rosaq_linear, MODE (the layers differ). */
int rosaq_linear_swiglu(const rosaq_packed_t* gate, const rosaq_packed_t* up, const void* x_dev, int32_t M,
                        int64_t ldx, void* y_dev, int64_t ldy, void* ws_dev, size_t ws_bytes,
                        void* hip_stream);

/* rosaq_mlp_swiglu - the gated FFN block of a decoder layer in three launches:
 *     y = h What_down^T,   h = silu(xhat What_gate^T) * (xhat What_up^T)   (rosaq_linear_swiglu),
 * for a down projection that needs no rotation at run time (packed with q_mode NONE, the paper's
 * setting for W_D, or with rotation_absorbed).  The gated product is rounded to fp16 once and
 * written straight into the down projection's input fragments, each channel at the storage
 * position that layer's salient-channel split assigns it (Sec. 3.2), so h never exists in
 * row-major form and no permutation launch runs in front of the down projection.  The result
 * equals, bit for bit, rosaq_linear_swiglu followed by rosaq_linear(down).
 *   gate, up  as for rosaq_linear_swiglu
 *   down      handle with in_features = gate's out_features and q_mode NONE at run time
 *   x_dev     DEVICE fp16 [M x gate.in_features], row stride ldx
 *   y_dev     DEVICE fp16 [M x down.out_features], row stride ldy
 *   ws_dev    DEVICE scratch of at least rosaq_workspace_bytes_mlp(gate, up, down, M) bytes
 *             (256-byte aligned; that size includes room for a split launch of the down projection)
 * Errors: those of rosaq_linear, MODE (gate / up differ, or down rotates at run time), SHAPE (down's
 * input width). */
size_t rosaq_workspace_bytes_mlp(const rosaq_packed_t* gate, const rosaq_packed_t* up,
                                 const rosaq_packed_t* down, int32_t M);
int rosaq_mlp_swiglu(const rosaq_packed_t* gate, const rosaq_packed_t* up, const rosaq_packed_t* down,
                     const void* x_dev, int32_t M, int64_t ldx, void* y_dev, int64_t ldy, void* ws_dev,
                     size_t ws_bytes, void* hip_stream);

/* Shape and storage facts of a handle (any output pointer may be NULL). */
int rosaq_packed_info(const rosaq_packed_t* p, int32_t* N, int32_t* D, int32_t* K,
                      int32_t* bits, int32_t* group, int32_t* q_mode,
                      size_t* device_bytes /* packed weights + scales + fp16 Q on the GPU */);

/* rosaq_packed_export - copy the canonical (layout-independent) arrays of Eq. 3 to
 * HOST buffers; any pointer may be NULL to skip it.
 *   salient_idx int32 [K]            ascending rotated-channel indices
 *   W_S         fp16  [N x K]        row-major
 *   codes       uint8 [N x (D-K)]    one code per byte, storage order
 *   scales      fp16  [N x (D-K)/group]
 *   zeros       fp16  [N x (D-K)/group]  (integer valued)                         */
int rosaq_packed_export(const rosaq_packed_t* p, int32_t* salient_idx, uint16_t* W_S,
                        uint8_t* codes, uint16_t* scales, uint16_t* zeros);

/* rosaq_pca_headwise - calibration step of the method on the GPU (Sec. 3.1 Eq. 4 applied per
 * attention head, Sec. 3.1.1): for every block of 128 input channels the eigenvectors of the
 * uncentred second moment C_h = X_h^T X_h / n_cal, found as the right singular vectors of X_h by
 * one-sided Jacobi rotations in fp64 (pairs of columns are rotated until all are mutually orthogonal;
 * C_h is never formed; eigenvalue c = |column c of X_h V|^2 / n_cal), until the off-diagonal norm of
 * the implied C_h is <= 1e-13 ||C_h||_F in every head.  Results, ready for rosaq_pack_weights:
 *   Q_host            HOST fp32 [D/128][128][128], eigenvectors as columns, sorted by eigenvalue
 *                     (descending; each column signed so that its largest entry is positive)
 *   eigenvalues_host  HOST fp64 [D], descending inside every head, >= 0
 *   X_dev             DEVICE fp16 [n_cal x D] calibration activations, row r at X + r*ldx
 * Allocates its own device scratch and waits for the result (calibration time, not the hot path).
 * Errors: NULL, SHAPE, ALIGN, HIP, NOCONVERGE (tolerance not reached within 60 sweeps). */
int rosaq_pca_headwise(const void* X_dev, int32_t n_cal, int32_t D, int64_t ldx, float* Q_host,
                       double* eigenvalues_host, void* hip_stream);

/* rosaq_pca_full - the same calibration step for a layer-wise rotation (Sec. 3.1, Eq. 4): the
 * eigenvectors of C = X^T X / n_cal over all D input channels, found as the right singular vectors
 * of X by one-sided Jacobi rotations in fp64 on the GPU (pairs of columns of X are rotated until
 * all are mutually orthogonal; C is never formed; eigenvalue c = |column c of X V|^2 / n_cal).
 * Stops when the off-diagonal norm of the implied C is <= 1e-13 ||C||_F.  Results as for
 * rosaq_pca_headwise:
 *   Q_host            HOST fp32 [D x D] row-major, eigenvectors as columns (xhat = x Q), sorted by
 *                     eigenvalue descending, each signed so that its largest entry is positive; with
 *                     fewer calibration rows than channels the null space comes out as an orthonormal
 *                     completion (any one is valid)
 *   eigenvalues_host  HOST fp64 [D], descending, >= 0
 *   X_dev             DEVICE fp16 [n_cal x D], row r at X + r*ldx
 * D a multiple of 128 up to 8192 (a sweep is D - 1 launches; a 1024-channel layer takes a few
 * tenths of a second).  Allocates its own device scratch (8 D (n_cal + D) bytes and 4 D^2 bytes of
 * bookkeeping) and waits for the result.  Errors: NULL, SHAPE, ALIGN, HIP, NOCONVERGE. */
int rosaq_pca_full(const void* X_dev, int32_t n_cal, int32_t D, int64_t ldx, float* Q_host,
                   double* eigenvalues_host, void* hip_stream);

/* rosaq_stream_probe - measurement aid, no arithmetic of the method: one launch of
 * `workgroups` x `threads` in which every wave reads its own contiguous share of
 * src_dev (src_bytes in total, 1 KiB per load) and every workgroup then reads
 * shared_bytes_per_workgroup from the start region of shared_dev (a buffer all
 * workgroups share, as they share the rotated activations in the GEMM).  Nothing is
 * written unless the data matches a magic pattern.  Timing it next to the GEMM gives
 * the memory system's own ceiling for a launch of that size and shape.
 * All pointers DEVICE, 16-byte aligned; src_bytes a multiple of 1 KiB per wave;
 * sink_dev at least 16 bytes per thread.  Errors: NULL, ARG, SHAPE, WORKSPACE, ALIGN, HIP. */
int rosaq_stream_probe(const void* src_dev, size_t src_bytes, const void* shared_dev,
                       size_t shared_bytes, size_t shared_bytes_per_workgroup, int32_t workgroups,
                       int32_t threads, void* sink_dev, size_t sink_bytes, void* hip_stream);

/* Tuning aid for benchmarks; affects later rosaq_linear* calls in this process.
 *   "mt", "nt"  16-row / 16-channel MFMA tiles per workgroup (0 = heuristic, 1, 2, 4; nt also 3 and 6
 *             for low-bit layers with mt >= 2)
 *   "rot_mt", "rot_nt", "rot_depth"  the same three knobs for the dense-rotation launch
 *   "wpb"     waves per workgroup splitting the contraction (0 = default, 4, 8, 16; variants that
 *             would not fit the register file fall back to 8)
 *   "depth"   units (a group, or four fp16 k-steps) a wave keeps in flight (0 = default, 1-4; clamped to
 *             what the chosen tile fits without spilling)
 *   "splits"  workgroups sharing one output tile of the main GEMM, each over its own part of the
 *             contraction (0 = heuristic, 1 = never split, 2-16; calls of up to 64 rows only)
 *   "rot_splits"  the dense rotation of calls of 17 to 64 rows as n = 2-16 slabs of the contraction
 *             whose partial tiles a second launch adds (0, 1 = the single-launch rotation, the
 *             default; a count whose slabs exceed 32 k-steps also keeps the single launch)
 *   "stages"  3 = whole call (default), 1 = prologue kernels only, 2 = main GEMM only
 *             (2 reuses the rotated activations a previous call left in the workspace)
 * For benchmarks and tests only: the settings are process-wide and not synchronised, so no other
 * thread may be inside a rosaq_linear* call while they change, and "stages" other than 3 makes
 * every later call skip part of its work while still returning ROSAQ_OK. */
int rosaq_tune(const char* key, int32_t value);

/* Reports, without launching anything (no GPU needed), the workgroup shape the main GEMM of a call
 * would get: M rows, `channels` output channels in total over the layers of the launch (each layer
 * rounded up to whole 16-channel tiles by the caller: pass the sum of 16 * ceil(N_i / 16)),
 * `in_features` = D, `bits` 3 or 4 (16 for an all-fp16 layer), under the current rosaq_tune settings.
 * shape_out (HOST, 5 ints) receives mt, nt (tiles of 16 rows / 16 channels per workgroup), waves per
 * workgroup, units in flight per wave and the number of workgroups that split one tile's contraction
 * (given a workspace of rosaq_workspace_bytes_batch size).  Errors: ROSAQ_ERR_NULL, ROSAQ_ERR_SHAPE (M, channels < 1,
 * channels or D not a multiple of 16 / 128), ROSAQ_ERR_ARG (bits). */
int rosaq_launch_shape(int32_t M, int32_t channels, int32_t in_features, int32_t bits, int32_t* shape_out);

/* Testing aid, host only: the weight image exactly as the kernels read it, rebuilt from the handle's
 * canonical arrays (which = 2 / 3: the same two images copied back from the device buffers the kernels
 * read; needs a handle packed without host_only).  which = 0: fp16 salient fragments [tiles][K/32][64 lanes][8 halves]; which = 1:
 * low-bit records [tiles][G] of 1088 bytes (INT4: [64 lanes][4 dwords] codes, then 16 dwords
 * scale | zero << 16) or 832 bytes (INT3: [64 lanes][3 dwords]); tiles = 8 * ceil(N / 128).
 * Lane l of tile t holds output channel 16 t + l % 16 and, per 32-channel k-step, the 8 storage-order
 * channels 8 (l / 16) .. + 7.  out_host may be NULL to query the size; *bytes is capacity in, size out.
 * Errors: ROSAQ_ERR_NULL, ROSAQ_ERR_ARG, ROSAQ_ERR_WORKSPACE (buffer too small; *bytes set to the need),
 * ROSAQ_ERR_HOSTONLY, ROSAQ_ERR_HIP (which = 2 / 3). */
int rosaq_packed_image(const rosaq_packed_t* p, int32_t which, void* out_host, size_t* bytes);

/* Testing aid, host only: the main GEMM's map from workgroup index to (channel chunk, row group) for a
 * launch of `chunks` x `row_groups` tiles (workgroup % 8 is the XCD; inside an XCD consecutive workgroups
 * form blocks of 8 chunks x 4 row groups).  workgroup < 0: returns the grid size (>= chunks * row_groups;
 * the surplus are padding workgroups that exit at once).  Otherwise returns 1 and the pair, or 0 (and -1,
 * -1) for a padding workgroup.  Errors (negative): ROSAQ_ERR_SHAPE, ROSAQ_ERR_NULL. */
int rosaq_block_map(int32_t workgroup, int32_t chunks, int32_t row_groups, int32_t* chunk_out,
                    int32_t* row_group_out);

void rosaq_free(rosaq_packed_t* p);

/* Text of the last error on this thread ("" if none). */
const char* rosaq_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* ROSAQ_H_ */
