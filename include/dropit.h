/*
 * dropit.h -- C ABI of the MI355X (gfx950) DropIT hot path.
 *
 * Two operations of "DropIT: Dropping Intermediate Tensors for Memory-Efficient
 * DNN Training" (arXiv 2202.13808):
 *
 *   forward  : a^ = D(a) = {a_Xr, Xr}   min-k dropping of a layer's cached
 *              input (Sec. 3.2; Sec. 3.3, min-k strategy; Sec. 4.1,
 *              implementation details)                      -> dropit_compress
 *   backward : grad(theta) ~= grad(z) * dl(R(a^), theta)/dtheta, the weight
 *              gradient taken on the zero-filled recovered tensor R(a^)
 *              (Sec. 3.2, Eq. conv_backward_elem / Eq. fc_backward_elem_save)
 *                                                           -> dropit_weight_grad
 *
 * General conventions
 *   - Every pointer named x, vals, idx, dY, dW, workspace is a DEVICE pointer
 *     owned by the caller.  The library allocates nothing, frees nothing and
 *     keeps no state between calls.  `shape` / `x_shape` / `conv` are HOST
 *     pointers read during the call only.
 *   - All work is enqueued on `hip_stream` (a hipStream_t passed as void*;
 *     NULL = the default stream).  No call synchronises the host or copies
 *     device memory to the host: the output length k is a host-side function
 *     of (numel, gamma), see dropit_keep_count.
 *   - Tensors are contiguous row-major; a "flat index" is the 0-based
 *     row-major element offset, stored as int32 (App. A.7 assumes int32
 *     indices), hence numel <= 2^31 - 1.
 *   - bf16 data are raw 16-bit patterns (top half of an IEEE fp32).
 *   - Arguments are validated before any HIP call; errors are returned as
 *     status codes, nothing aborts.  Results are bit-reproducible run to run.
 *   - Concurrent calls must use distinct workspaces.
 */
#ifndef DROPIT_H
#define DROPIT_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* In C an enumeration is an int and any int may arrive in one; C++ callers and this library's own (C++) sources
 * get the same guarantee from a fixed underlying type, so an unknown code is an error value, never undefined. */
#ifdef __cplusplus
#define DROPIT_ENUM(name) enum name : int
#else
#define DROPIT_ENUM(name) enum name
#endif

typedef DROPIT_ENUM(dropit_dtype) { DROPIT_F32 = 0, DROPIT_BF16 = 1 } dropit_dtype;

typedef DROPIT_ENUM(dropit_status) {
    DROPIT_OK = 0,
    DROPIT_EINVAL = 1,        /* null / misaligned pointer, bad shape, gamma outside [0,1], numel > 2^31-1 */
    DROPIT_EWORKSPACE = 2,    /* workspace smaller than the matching *_workspace_bytes query */
    DROPIT_EUNSUPPORTED = 3,  /* reserved: a geometry that is not implemented (none at present) */
    DROPIT_EHIP = 4           /* a HIP launch failed */
} dropit_status;

/* Human-readable name of a status code (static storage, never NULL). */
const char *dropit_status_string(dropit_status s);

/*
 * Number of retained elements for dropping rate gamma (Sec. 3.3, min-k strategy: the
 * gamma fraction of smallest magnitude is dropped; Sec. 4.1: the top-k keeps a
 * share of 1 - gamma):  k = floor((1 - gamma) * numel), evaluated in IEEE double as
 * numel - ceil(gamma * numel).  gamma = 0 keeps everything (the baseline row of
 * Table 2), gamma = 1 keeps nothing.
 * Returns -1 if numel < 0, numel > 2^31-1, or gamma is NaN / outside [0,1].
 */
int64_t dropit_keep_count(int64_t numel, double gamma);

/* Bytes of device workspace dropit_compress needs for a tensor of `numel`
 * elements of type `dt` (0 on invalid arguments). */
size_t dropit_compress_workspace_bytes(int64_t numel, dropit_dtype dt);

/*
 * Min-k dropping D(a) (Sec. 3.2; Sec. 3.3, min-k strategy; Sec. 4.1).
 *
 * Keeps the k = dropit_keep_count(numel, gamma) elements of x with the largest
 * absolute magnitude, ranked over the whole tensor (one ranking per call, i.e.
 * per mini-batch tensor).  Magnitude order is the unsigned order of the bit
 * pattern with the sign bit cleared: -0 ties with +0, denormals are ordered
 * exactly, inf ranks above all finite values and NaN above inf.  Elements that
 * tie at the threshold magnitude are kept in order of lowest flat index.
 *
 *   x      [in]  device, contiguous row-major tensor of `shape` (ndim >= 1,
 *                all dims >= 1), 16-byte aligned
 *   shape  [in]  host, ndim extents
 *   vals   [out] device, k elements of type dt: exact bit copies x[idx[j]]
 *   idx    [out] device, k int32 flat indices, strictly ascending
 *   workspace    device, 256-byte aligned, >= dropit_compress_workspace_bytes;
 *                contents on entry are irrelevant, undefined on exit
 *
 * k == 0 writes nothing.  vals/idx may be NULL only if k == 0.
 */
dropit_status dropit_compress(const void *x, const int64_t *shape, int ndim, dropit_dtype dt,
                              double gamma, void *vals, int32_t *idx,
                              void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * dropit_compress without a workspace argument, for callers that cannot allocate device memory
 * and have none to spare: code under HIP graph capture, tight serving loops, harnesses that
 * forbid hipMalloc.  The select's exchange area (about 170 KB, independent of the tensor size)
 * is a static device array inside the library, one copy per GPU, held until the process ends.
 * The call itself allocates and frees nothing, on the device or through any library.
 *
 * Arguments, outputs, alignment and error behaviour as for dropit_compress; tensors of up to
 * DROPIT_STATIC_MAX_NUMEL elements (the limit of the int32 index; larger shapes give
 * DROPIT_EINVAL), DROPIT_EHIP if the runtime cannot give the array's device address.
 * All calls on one GPU share the one array (it keeps the last call's contents; the kernels clear
 * what they need): calls that overlap in time on the same GPU, from any stream or thread, race
 * with each other -- order them, or give the others a workspace through dropit_compress.
 */
#define DROPIT_STATIC_MAX_NUMEL 2147483647
dropit_status dropit_compress_static(const void *x, const int64_t *shape, int ndim, dropit_dtype dt,
                                     double gamma, void *vals, int32_t *idx, void *hip_stream);

/* Bytes of device workspace dropit_compress_random needs (0 on invalid arguments). */
size_t dropit_compress_random_workspace_bytes(int64_t numel, dropit_dtype dt);

/*
 * Random dropping D(a) (Sec. 3.3, random strategy: a gamma fraction of the
 * elements of the mini-batch tensor is dropped at random; the paper's baseline
 * strategy beside min-k).
 *
 * Keeps exactly k = dropit_keep_count(numel, gamma) elements, a uniformly random
 * k-subset fixed by `seed` alone (not by the values of x): element i draws the
 * 32-bit word (i mod 4) of Philox4x32-10 (Salmon et al., SC'11) at counter
 * (floor(i/4), 0, 0, 0) under key (seed mod 2^32, seed div 2^32); the k elements
 * with the largest draw, shifted right by one bit, are kept, equal draws going to
 * the lowest flat index.  Callers that want a fresh subset per iteration pass a
 * fresh seed.
 *
 * Arguments, outputs (ascending idx, vals[j] = x[idx[j]] bit for bit), alignment
 * and error behaviour as for dropit_compress; the workspace must hold
 * dropit_compress_random_workspace_bytes (it keeps one 32-bit draw per element).
 * The pairs feed dropit_weight_grad unchanged.
 */
dropit_status dropit_compress_random(const void *x, const int64_t *shape, int ndim, dropit_dtype dt,
                                     double gamma, uint64_t seed, void *vals, int32_t *idx,
                                     void *workspace, size_t workspace_bytes, void *hip_stream);

/* Convolution geometry for dropit_weight_grad (cross-correlation, zero padding,
 * 0-based: input row = out_row*stride_h - pad_h + u*dil_h). */
typedef struct {
    int64_t kh, kw, stride_h, stride_w, pad_h, pad_w, dil_h, dil_w;
} dropit_conv2d;

/* Bytes of device workspace dropit_weight_grad needs for k retained pairs (0 on
 * invalid or unsupported arguments).  Arguments as for dropit_weight_grad. */
size_t dropit_weight_grad_workspace_bytes(const int64_t *x_shape, int ndim, dropit_dtype dt,
                                          int64_t k, int64_t c_out, const dropit_conv2d *conv);

/* Which kernels dropit_weight_grad runs for these arguments (arguments as there; host-only, no GPU work):
 * DROPIT_PATH_NONE for invalid or unsupported arguments. */
typedef DROPIT_ENUM(dropit_wgrad_path) {
    DROPIT_PATH_NONE = 0,
    DROPIT_PATH_FC_MFMA = 1,        /* recover + split-K bf16 MFMA GEMM */
    DROPIT_PATH_CONV_BANDS = 2,     /* 3x3/s1/p1 bf16: row bands in LDS, implicit im2col on the matrix cores */
    DROPIT_PATH_CONV_GEMM = 3,      /* 3x3/s1/p1 bf16, small planes with many channels: explicit im2col rows + the FC GEMM */
    DROPIT_PATH_FMA = 4,            /* exact fp32 multiply-add kernels (fp32 inputs, odd shapes) */
    DROPIT_PATH_CONV_IM2COL = 5,    /* bf16, any geometry and either layout: zero-filled im2col rows written from the pairs + the FC GEMM */
    DROPIT_PATH_FC_SMALL = 6,       /* fully-connected layers of at most 16384 input elements: recover in LDS and exact fp32 multiply-adds, one launch */
    DROPIT_PATH_FC_FUSED = 7        /* the FC_MFMA product with the recover step inside it (only after dropit_set_fc_recover(1)) */
} dropit_wgrad_path;
dropit_wgrad_path dropit_weight_grad_path(const int64_t *x_shape, int ndim, dropit_dtype dt, int64_t k,
                                          int64_t c_out, const dropit_conv2d *conv);

/*
 * Weight gradient from the sparsified cache (Sec. 3.2): the recover step R(a^)
 * (zeros at dropped positions) followed by the ordinary dense weight gradient;
 * the dense product is kept on purpose (Sec. 3.2: sparsity is used for
 * storage only).
 *
 * conv == NULL, fully-connected layer (Eq. fc_backward_elem_save):
 *     x_shape = [..., C_in]; all leading dims are tokens (N_tok = numel/C_in)
 *     dY  [N_tok, c_out] row-major, type dt
 *     dW  [c_out, C_in] row-major fp32:  dW[j][c] = sum_n dY[n][j] * R(a^)[n][c]
 * conv != NULL, 2-d convolution (Eq. conv_backward_elem):
 *     x_shape = [N, C, H, W] (NCHW);  dY [N, c_out, OH, OW] with
 *     OH = (H + 2*pad_h - dil_h*(kh-1) - 1)/stride_h + 1 (OW alike), type dt
 *     dW  [c_out, C, kh, kw] fp32:
 *     dW[j][c][u][v] = sum_{n,oy,ox} dY[n][j][oy][ox] * R(a^)[n][c][oy*sh-ph+u*dh][ox*sw-pw+v*dw]
 *     bf16 with c_out % 8 == 0 and C*kh*kw <= 32768 runs on the matrix cores
 *     (3x3 / stride 1 / pad 1 in forms of its own, every other geometry through
 *     explicit im2col rows in the workspace, at most 1 GiB of them; see
 *     dropit_weight_grad_path); fp32 and the remaining shapes (kernel extents up
 *     to 1024, stride / pad / dilation up to 65535) take an exact but slow fp32 kernel.
 *     DROPIT_EINVAL if the window does not fit the padded input.
 *
 *   vals, idx [in]  device, the k pairs written by dropit_compress for a tensor
 *                   of x_shape (idx strictly ascending, in range; not checked)
 *   dY        [in]  device, 16-byte aligned
 *   dW        [out] device fp32, 16-byte aligned, fully overwritten
 *   workspace       device, 256-byte aligned, >= dropit_weight_grad_workspace_bytes
 *
 * bf16 inputs are multiplied exactly and accumulated in fp32; fp32 inputs use
 * true fp32 multiply-adds.  k == 0 gives dW = 0.  The bias gradient does not
 * depend on the cached input and is not computed here.
 */
dropit_status dropit_weight_grad(const void *vals, const int32_t *idx, int64_t k,
                                 const int64_t *x_shape, int ndim, dropit_dtype dt,
                                 const void *dY, int64_t c_out, const dropit_conv2d *conv,
                                 float *dW, void *workspace, size_t workspace_bytes,
                                 void *hip_stream);

/*
 * The same weight gradient for channels-last tensors (Sec. 3.2, Eq. conv_backward_elem; the
 * paper's method does not depend on the memory layout, the flat indices of dropit_compress
 * simply index the NHWC tensor):
 *     x_shape = [N, H, W, C] (4 extents),  dY [N, OH, OW, c_out],  conv != NULL
 *     dW [c_out, kh, kw, C] fp32 (the channels-last layout of a [c_out, C, kh, kw] weight)
 * Everything else (arguments, alignment, workspace, errors, arithmetic) as for
 * dropit_weight_grad; bf16 with c_out % 8 == 0 runs on the matrix cores (DROPIT_PATH_CONV_IM2COL; a
 * 1x1 / stride 1 / unpadded convolution is a fully-connected layer over the N*H*W positions in this
 * layout and takes those kernels, DROPIT_PATH_FC_MFMA).
 */
dropit_wgrad_path dropit_weight_grad_nhwc_path(const int64_t *x_shape, dropit_dtype dt, int64_t k, int64_t c_out,
                                               const dropit_conv2d *conv);
size_t dropit_weight_grad_nhwc_workspace_bytes(const int64_t *x_shape, dropit_dtype dt, int64_t k, int64_t c_out,
                                               const dropit_conv2d *conv);
dropit_status dropit_weight_grad_nhwc(const void *vals, const int32_t *idx, int64_t k, const int64_t *x_shape,
                                      dropit_dtype dt, const void *dY, int64_t c_out, const dropit_conv2d *conv,
                                      float *dW, void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * Row form of the cache: cheaper indices (Sec. 4.3 counts the indices as the
 * method's memory cost; the appendix on choosing gamma prices an int32 index like
 * an fp32 activation).  The tensor is read as rows of its last dimension
 * (row_len = shape[ndim-1] <= 65536, rows = numel / row_len).  A retained element
 * keeps its 16-bit position in its row, and each row one offset:
 *     col[j]    = idx[j] mod row_len                       (k uint16)
 *     rowptr[r] = number of retained elements before row r  (rows + 1 int32;
 *                 row r owns pairs rowptr[r] .. rowptr[r+1]-1, rowptr[rows] = k)
 * i.e. 2k + 4(rows+1) bytes of indices instead of 4k, lossless.
 *
 * dropit_compress_rows: same selection, same vals as dropit_compress (min-k,
 * ties to the lowest index, ascending order); col / rowptr [out] device.
 * rowptr is always written, also for k == 0 (all zeros).  DROPIT_EINVAL if the
 * last dimension exceeds 65536.  Workspace: dropit_compress_rows_workspace_bytes
 * (the select's area plus 4k bytes for the flat indices it converts).
 *
 * dropit_weight_grad_rows: dropit_weight_grad from (vals, col, rowptr); same
 * kernels, same results bit for bit.  The table is trusted like idx is (a
 * malformed one gives a wrong gradient, never an out-of-bounds write into the
 * workspace).  Workspace: dropit_weight_grad_rows_workspace_bytes.
 */
size_t dropit_compress_rows_workspace_bytes(int64_t numel, int64_t k, dropit_dtype dt);
dropit_status dropit_compress_rows(const void *x, const int64_t *shape, int ndim, dropit_dtype dt,
                                   double gamma, void *vals, uint16_t *col, int32_t *rowptr,
                                   void *workspace, size_t workspace_bytes, void *hip_stream);
size_t dropit_weight_grad_rows_workspace_bytes(const int64_t *x_shape, int ndim, dropit_dtype dt,
                                               int64_t k, int64_t c_out, const dropit_conv2d *conv);
dropit_status dropit_weight_grad_rows(const void *vals, const uint16_t *col, const int32_t *rowptr,
                                      int64_t k, const int64_t *x_shape, int ndim, dropit_dtype dt,
                                      const void *dY, int64_t c_out, const dropit_conv2d *conv,
                                      float *dW, void *workspace, size_t workspace_bytes,
                                      void *hip_stream);

/*
 * Bit-mask form of the cache (Sec. 4.3 counts the index bytes as part of the method's memory;
 * the appendix on choosing gamma prices an int32 index at one fp32 activation).  Instead of idx:
 *     mask[ceil(numel/32)]  uint32, bit (i mod 32) of word (i div 32) set iff element i is retained
 *                           (bits past numel are 0);
 *     blockptr[ceil(numel/DROPIT_MASK_BLOCK) + 1]  int32, the number of retained elements before
 *                           element b * DROPIT_MASK_BLOCK (the last entry is k).
 * numel/8 bytes whatever k: smaller than int32 indices when more than 1/32 of the tensor is kept.
 * vals is what dropit_compress writes (ascending flat index).  The encoding is lossless:
 * dropit_weight_grad_mask gives bit for bit what dropit_weight_grad gives on the flat indices.
 * Arguments not named here, alignment and error behaviour as for dropit_compress /
 * dropit_weight_grad; mask and blockptr are device pointers, 4-byte aligned; each workspace also
 * holds the flat indices (the *_mask_workspace_bytes queries say how much).
 */
#define DROPIT_MASK_BLOCK 1024
size_t dropit_compress_mask_workspace_bytes(int64_t numel, int64_t k, dropit_dtype dt);
dropit_status dropit_compress_mask(const void *x, const int64_t *shape, int ndim, dropit_dtype dt,
                                   double gamma, void *vals, uint32_t *mask, int32_t *blockptr,
                                   void *workspace, size_t workspace_bytes, void *hip_stream);
size_t dropit_weight_grad_mask_workspace_bytes(const int64_t *x_shape, int ndim, dropit_dtype dt,
                                               int64_t k, int64_t c_out, const dropit_conv2d *conv);
dropit_status dropit_weight_grad_mask(const void *vals, const uint32_t *mask, const int32_t *blockptr,
                                      int64_t k, const int64_t *x_shape, int ndim, dropit_dtype dt,
                                      const void *dY, int64_t c_out, const dropit_conv2d *conv,
                                      float *dW, void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * How dropit_compress runs its select (per host thread):
 *   0 (default)  one persistent kernel (it also clears its own exchange area), one workgroup per
 *                compute unit, grid barriers between its phases, launched as an ordinary kernel
 *                after checking that the grid fits the device at once; falls back to mode 1 if
 *                it does not.  Its barriers wait a
 *                bounded time; if the workgroups do not all become resident (a device shared
 *                with other persistent kernels) the kernel redoes the selection serially in its
 *                last workgroup, so the result is complete either way, only late.
 *   1            the same select as separate ordinary kernels (no grid barriers, no memset
 *                nodes): for callers that must not depend on co-residency at all.  Use it when
 *                other kernels that hold compute units or LDS for long (another select on a
 *                second stream, a persistent kernel) run on the device at the same time: mode 0
 *                then waits out its patience (milliseconds) and redoes the selection serially,
 *                correct but orders of magnitude later than its usual 25 - 50 us.
 *   2            mode 0's kernel through a cooperative launch: the runtime then guarantees
 *                co-residency, at the price of tens of microseconds of queue switching per
 *                call; cannot be recorded into a HIP graph (falls back to mode 0's launch).
 *   3            test hook: mode 0 with zero patience at the grid barriers, which forces the
 *                serial redo; every kernel still exits normally.
 * Modes 0, 1 and 3 use only ordinary kernel launches and can be captured into a HIP graph.
 * Returns DROPIT_EINVAL for any other mode.
 */
dropit_status dropit_set_select_mode(int mode);

/*
 * Where the recover step R(a^) of a bf16 fully-connected layer happens (Sec. 3.2; Fig. 1: the zero-filled
 * tensor is only ever an operand of the weight gradient).  Per host thread, like the select mode.
 *   0  (default) R(a^) is written as a dense bf16 operand into the workspace and the product reads it
 *      (DROPIT_PATH_FC_MFMA).  The faster form on MI355X by 10 - 15 us per layer at the ViT shapes; the
 *      workspace holds one tensor the size of the layer's input for the duration of the call.
 *   1  R(a^) is built tile by tile in LDS inside the product and never exists in device memory
 *      (DROPIT_PATH_FC_FUSED): the workspace holds one 4-byte word per kept pair instead of the dense tensor
 *      (0.2 of its bytes at gamma = 0.9).  Same dW, bit for bit.  Shapes the form does not cover (c_out <= 128,
 *      C_in > 32768) keep taking form 0; query with dropit_weight_grad_path.
 * dropit_weight_grad_workspace_bytes / _path answer for the form set on the calling thread.
 * Returns DROPIT_EINVAL for any other value.
 */
dropit_status dropit_set_fc_recover(int form);

/*
 * Measurement aid (not part of the method): per-kernel timing marks.
 * `events` is a HOST array of `count` hipEvent_t handles created by the caller.
 * The next dropit_compress / dropit_weight_grad call made from this host thread
 * records events[0] before its first kernel, events[i] before its (i+1)-th
 * kernel and one after its last, on the call's stream, until the array is
 * used up.  Pass (NULL, 0) to switch it off.  The handles stay owned by the
 * caller; these per-thread settings are the only state the library keeps.
 */
void dropit_trace_events(void **events, int count);

#ifdef __cplusplus
}
#endif
#endif /* DROPIT_H */
