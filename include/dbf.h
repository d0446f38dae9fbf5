/*
 * libdbf -- Double Binary Factorization (DBF) layer products on AMD MI355X (gfx950).
 *
 * One DBF layer stands for a weight matrix W (n_out x n_in) through
 *
 *     W' = diag(a) * A * diag(m) * B * diag(b)
 *
 * with sign matrices A (n_out x k) and B (k x n_in), entries in {-1,+1}, and
 * fp16 vectors a (n_out), m (k), b (n_in).  The layer product is
 *
 *     Y = X * W'^T = ((((X . b^T) B^T) . m^T) A^T) . a^T          (batch x n_out)
 *
 * (paper, section 3: the factorisation, the forward-pass expression that follows
 * it, and "Middle dimension size" for the shapes).  Inside the two sign products
 * only additions and subtractions are needed (section 3.1, "Inference costs").
 *
 * Conventions common to every entry point
 *   - Plain C ABI.  Every function that can fail returns one of the DBF_* codes
 *     below and never throws or aborts.  Arguments are validated before any GPU
 *     call, so all argument errors are reported even on a machine without a GPU.
 *   - "host" pointers are ordinary process memory; "device" pointers are HIP
 *     device memory of the GPU the layer was packed on.  The caller owns every
 *     buffer it passes in; the library owns what a dbf_layer / dbf_stack holds
 *     until dbf_free / dbf_stack_free.
 *   - fp16 values cross the boundary as IEEE binary16 bit patterns (uint16_t on
 *     the host, 2-byte elements on the device).
 *   - Launching entry points (dbf_gemv*, dbf_gemm, dbf_stack_gemv) are
 *     asynchronous on the caller's HIP stream (a hipStream_t passed as void*,
 *     NULL = the default stream), allocate nothing and do not synchronise.  A
 *     layer holds scratch for its middle activations and, for batches of 2 and
 *     more, for its quantised stage inputs, so one layer must not run on two
 *     streams at the same time, be it directly or through stacks that hold it.
 *   - Non-finite activations give unspecified (but memory-safe) results.
 *
 * Canonical sign-bit format (the paper defines none; this is the interchange
 * format): row-major, reduction dimension fastest; element c of a row is bit
 * (c & 31), least significant first, of 32-bit word (c >> 5) of that row; a set
 * bit means +1, a clear bit -1; unused high bits of a row's last word are zero.
 * A is n_out rows of ceil(k/32) words, B is k rows of ceil(n_in/32) words.
 */
#ifndef DBF_H
#define DBF_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct dbf_layer dbf_layer; /* one packed layer; opaque; owns device memory */
typedef struct dbf_stack dbf_stack; /* a group of layers run in one launch; opaque  */

enum {
    DBF_OK = 0,
    DBF_EINVAL = -1,     /* null pointer, bad enum value, batch/T out of range     */
    DBF_ESHAPE = -2,     /* n_in, n_out or k < 1, or beyond the supported maximum  */
    DBF_ENOTSIGN = -3,   /* a sign entry other than -1/+1, or dirty tail bits      */
    DBF_ENOMEM = -4,     /* host or device allocation failed                       */
    DBF_EHIP = -5,       /* a HIP runtime call or kernel launch failed             */
    DBF_EWORKSPACE = -6  /* workspace missing, misaligned or too small             */
};

/* Which decode kernel dbf_gemv_kind runs. */
enum {
    DBF_GEMV_AUTO = 0, /* what dbf_gemv uses.  Batch 1: DBF_GEMV_MFMA for a group of layers whose B stage
                          alone fills the chip (1024 workgroups: 64 layers of 4096 x 4096,
                          k = 2048), DBF_GEMV_MFMA_SPLIT for a single layer and shorter groups (measured
                          faster there: in one launch their A-stage workgroups would all sit waiting
                          next to the B stage), long rows of short launches cut into column pieces.
                          Batches of 2 and more -- and groups of layers with long stage inputs at
                          batch 1 too, see DBF_TUNE_LONG_ROWS -- quantise each stage input once per
                          call: four launches (quantise x, B stage, quantise t, A stage).  Every
                          choice gives the same bits as DBF_GEMV_MFMA and DBF_GEMV_MFMA_SPLIT     */
    DBF_GEMV_VALU = 1, /* fp32 add/subtract per sign bit on the vector ALU (exact fp32 sums) */
    DBF_GEMV_MFMA = 2, /* sign bytes fed to the int8 matrix cores as the adder; the input
                          vector of each stage is rounded once to 16-bit fixed point.  Both
                          stages run in ONE launch: A-stage workgroups wait on the device for
                          their layer's B stage                                             */
    DBF_GEMV_MFMA_SPLIT = 3 /* the same kernel in two launches (B stage, then A stage)      */
};

#define DBF_MAX_BATCH 16       /* largest batch dbf_gemv / dbf_stack_gemv accept */
#define DBF_MAX_DIM (1 << 20)  /* largest n_in, n_out or k                       */
/* Longest stage input (n_in for the B stage, k for the A stage) the integer matrix-core paths take.  They add the
 * 16-bit fixed-point inputs (|q| <= 32512) in int32: a sum over more than 66051 inputs need not fit, whatever the
 * order.  Layers with a longer stage input are decoded by the vector-ALU kernel (fp32 sums) under DBF_GEMV_AUTO;
 * the kinds that name the matrix-core kernel, and the prefill beyond what dbf_gemm hands to the decode kernels
 * (32 tokens; dbf_gemm_static: any), return DBF_ESHAPE. */
#define DBF_INT_PATH_MAX_COLS 65536

/* ---- packing (offline, once per layer) -------------------------------------------------
 * Section 3 ("Double binary factorization"): the five operands of a layer.
 *
 * dbf_pack: A_pm1 (host, n_out*k int8, row-major) and B_pm1 (host, k*n_in int8, row-major)
 * hold -1/+1; a, m, b (host) hold n_out, k, n_in fp16 bit patterns.  Converts the signs to
 * bits, re-tiles them into the device layout, uploads everything to the current HIP device
 * and returns a new layer in *out.  Any k >= 1 is accepted (padding is internal).
 * Errors: DBF_EINVAL (null), DBF_ESHAPE, DBF_ENOTSIGN (entry not -1/+1), DBF_ENOMEM,
 * DBF_EHIP (no usable GPU).  On error *out is set to NULL.
 *
 * dbf_pack_bits: the same from canonical packed words (host).  DBF_ENOTSIGN if a row's
 * unused tail bits are not zero.
 *
 * dbf_unpack_bits: inverse of dbf_pack_bits; copies the layer back from the device into
 * host buffers of the canonical sizes (any output pointer may be NULL to skip it).
 * Synchronises the device.  Bit-exact round trip.
 */
int dbf_pack(int n_in, int n_out, int k, const int8_t* A_pm1, const int8_t* B_pm1,
             const uint16_t* a, const uint16_t* m, const uint16_t* b, dbf_layer** out);
int dbf_pack_bits(int n_in, int n_out, int k, const uint32_t* A_bits, const uint32_t* B_bits,
                  const uint16_t* a, const uint16_t* m, const uint16_t* b, dbf_layer** out);
int dbf_unpack_bits(const dbf_layer* layer, uint32_t* A_bits, uint32_t* B_bits,
                    uint16_t* a, uint16_t* m, uint16_t* b);
/* Shapes and the device memory the layer holds (any output pointer may be NULL). */
int dbf_dims(const dbf_layer* layer, int* n_in, int* n_out, int* k, size_t* device_bytes);
void dbf_free(dbf_layer* layer); /* NULL is allowed */

/* ---- host-side layout helpers (no GPU needed) ------------------------------------------
 * The device layout of a rows x cols sign matrix (reduction over cols): rows are padded to
 * a multiple of 128 and cols to a multiple of 64 with zero bits; the matrix is cut into
 * tiles of 128 rows x 64 cols stored row-tile major, 1024 bytes each.  In a tile, byte
 * (256*g + 16*r + j), 0<=g<4, 0<=r<16, 0<=j<16, holds in its bit s (0<=s<8) the sign of
 * element (row 16*s + r, col 16*g + j) of the tile.  A wavefront reads one tile with one
 * coalesced 16-byte load per lane and owns, per lane, sixteen columns of eight rows.
 *
 * dbf_tiled_bytes: size of the tiled image (0 if rows or cols is out of range).
 * dbf_signs_to_bits_host: int8 -1/+1 (rows*cols) -> canonical words; DBF_ENOTSIGN otherwise.
 * dbf_tile_host / dbf_untile_host: canonical words <-> tiled image (both host), bit-exact
 * inverses of each other; dbf_tile_host returns DBF_ENOTSIGN for dirty tail bits.
 */
size_t dbf_tiled_bytes(int rows, int cols);
int dbf_signs_to_bits_host(int rows, int cols, const int8_t* pm1, uint32_t* bits);
int dbf_tile_host(int rows, int cols, const uint32_t* bits, uint8_t* tiled);
int dbf_untile_host(int rows, int cols, const uint8_t* tiled, uint32_t* bits);

/* ---- decode: Y = X W'^T for a few tokens -----------------------------------------------
 * The forward-pass expression of section 3, evaluated in two stages: the B stage
 * t = ((x . b) B^T) . m (the middle rescale is fused into its epilogue), then the A stage
 * y = (t A^T) . a.  fp32 (or exact integer) accumulation, fp32 middle activations.  How many
 * launches a call makes depends on the kind (see DBF_GEMV_AUTO); all are issued on `hip_stream`.
 *
 * x_dev: device, fp16 [batch][n_in] row-major, tightly packed.
 * y_dev: device, fp16 [batch][n_out] row-major, written in full.
 * batch: 1..DBF_MAX_BATCH.  Errors: DBF_EINVAL, DBF_ESHAPE (a kind that names the matrix-core kernel on a layer
 * with n_in or k above DBF_INT_PATH_MAX_COLS), DBF_EHIP.
 * dbf_gemv_kind selects the kernel variant (DBF_GEMV_*); dbf_gemv is DBF_GEMV_AUTO.
 */
int dbf_gemv(const dbf_layer* layer, const void* x_dev, void* y_dev, int batch, void* hip_stream);
int dbf_gemv_kind(const dbf_layer* layer, const void* x_dev, void* y_dev, int batch, int kind,
                  void* hip_stream);
/* The bounded wait of the one-launch kernel.  An A-stage workgroup waits on the device for the B stage of
 * its layer, for at most DBF_TUNE_WAIT_LIMIT_US microseconds (default 250 000) of the GPU's constant-rate
 * clock.  The bound is never expected to be hit: a B-stage workgroup never waits and is always dispatched
 * before any A-stage one.  If it is hit, the workgroup gives up: every fp16 output it owns is written as a
 * quiet NaN (0x7E00), so the failure is visible in y itself, with no extra call and no synchronisation; a
 * sticky counter is raised as well.  The device-side counters stay consistent (they only ever grow), so
 * later calls on the same layer or stack are not affected.
 * dbf_sync_timeouts / dbf_stack_sync_timeouts synchronise the device and return the sticky counter in
 * *timeouts (0 = no wait was ever given up).  Errors: DBF_EINVAL, DBF_EHIP. */
int dbf_sync_timeouts(const dbf_layer* layer, int* timeouts);

/* ---- prefill: the same product for T tokens as two matrix-core contractions ------------
 * (The paper times batch 1 only, section 4.4; rows of X are independent, so the product is
 * defined for any T by the same expression, section 3.)
 *   DBF_GEMM_I8  the int8 matrix cores as the adder.  X.b, and later the middle activations, are rounded
 *                per token to 16-bit fixed point (q = rint(u * 32512 / max|u|)) and split into two int8
 *                planes; the masked sign bytes are the other operand; the sums are exact integers; the
 *                middle activations stay in fp32.
 *   DBF_GEMM_AUTO (dbf_gemm): DBF_GEMM_I8; calls of up to 2 * DBF_MAX_BATCH tokens are run as one or two
 *                decode batches (dbf_gemv), which give the same bits at a third to two thirds of the latency.
 *
 * X_dev: device fp16 [T][n_in]; Y_dev: device fp16 [T][n_out]; T >= 1 (at most 65535 * 64).
 * workspace_dev: device scratch of at least dbf_gemm_workspace_bytes(layer, T) bytes (up to 512 tokens that
 * includes room for the integer sums of stages whose columns are cut into shares over more workgroups: calls of
 * few tokens would otherwise leave most of the chip idle; same bits), 256-byte aligned, contents need not be
 * anything on entry and are undefined on return.  Asynchronous on the
 * stream; allocates nothing.  Errors: DBF_EINVAL (NULL pointer, T < 1 or too large, unknown
 * kind), DBF_EWORKSPACE (NULL, misaligned or short workspace), DBF_ESHAPE (more than 2 * DBF_MAX_BATCH tokens
 * on a layer with n_in or k above DBF_INT_PATH_MAX_COLS), DBF_EHIP.
 * dbf_gemm_workspace_bytes returns 0 for a NULL layer or T < 1.
 */
enum { DBF_GEMM_AUTO = 0, DBF_GEMM_I8 = 2 };
size_t dbf_gemm_workspace_bytes(const dbf_layer* layer, int T);
int dbf_gemm(const dbf_layer* layer, const void* X_dev, void* Y_dev, int T,
             void* workspace_dev, size_t workspace_bytes, void* hip_stream);
int dbf_gemm_kind(const dbf_layer* layer, const void* X_dev, void* Y_dev, int T,
                  void* workspace_dev, size_t workspace_bytes, int kind, void* hip_stream);

/* dbf_gemm_static: dbf_gemm for callers that cannot allocate or pass a workspace -- code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  The same kernels and the same bits as
 * dbf_gemm_kind(..., DBF_GEMM_I8, ...), for every T >= 1, with the scratch (quantised activations, fp32 middle
 * activations) in a static device array of DBF_GEMM_STATIC_BYTES that each GPU the library runs on holds
 * until the process ends.  Calls no hipMalloc / hipFree or any allocating routine.
 *   Limit: every call with dbf_gemm_workspace_bytes(layer, T) <= DBF_GEMM_STATIC_BYTES is taken, and so is a
 *   call of up to 512 tokens that fits without the room for the sums of column shares (it then runs unsplit);
 *   else DBF_EWORKSPACE and nothing is launched (T = 512 at 11008 -> 4096, k = 5970 needs 28.4 MiB unsplit; 1024
 *   tokens of a 4096 x 4096, k = 2048 layer 20 MiB).  The current device must be the layer's (DBF_EINVAL).
 *   The first call on a device looks up the array's address (hipGetSymbolAddress); make it outside graph capture.
 *   Every call on a GPU uses that GPU's one array: calls that may overlap in time on one GPU (two streams,
 *   two threads) race and give wrong results; calls on one stream are ordered and safe.  Nothing in the array
 *   has to be zero and nothing is kept between calls.
 * Asynchronous on hip_stream.  Errors: DBF_EINVAL, DBF_EWORKSPACE, DBF_ESHAPE (n_in or k above
 * DBF_INT_PATH_MAX_COLS), DBF_EHIP. */
#define DBF_GEMM_STATIC_BYTES (32u << 20)
int dbf_gemm_static(const dbf_layer* layer, const void* X_dev, void* Y_dev, int T, void* hip_stream);

/* ---- middle-channel pruning (paper, section 3.5 "Nonuniform layer compression ratios") ------
 * The paper treats the middle dimension as channels and keeps those with the highest scores
 * (the scores need gradients and are the caller's business).  dbf_prune_middle makes the new,
 * smaller layer on the device, in the packed tile layout, without unpacking:
 *     A' = A[:, keep],  B' = B[keep, :],  m' = m[keep],  a' = a,  b' = b,   k' = n_keep,
 * i.e. W'_new = sum over kept j of m_j A[:,j] B[j,:] (the old W' with the dropped m_j set to 0).
 * keep: HOST array of n_keep middle indices, strictly increasing, each in [0, k); 1 <= n_keep <= k.
 * The current device must be the layer's.  *out is a new, independent layer (free it with
 * dbf_free; the old layer is untouched).  Synchronous: allocates, runs the gather kernels and
 * returns when they have finished.  Errors: DBF_EINVAL (null, bad or unsorted indices, wrong
 * device), DBF_ENOMEM, DBF_EHIP. */
int dbf_prune_middle(const dbf_layer* layer, const int32_t* keep, int n_keep, dbf_layer** out);

/* ---- SVID projection (paper, section 3.2 "Computing Double Binary Factorization") ------------
 * SVID(Z) = a . Sign(Z) . m^T, with a m^T the rank-one decomposition of |Z| by power iteration:
 * the projection step of the ADMM iteration that computes the factorisation.  Readings where the
 * paper is silent: Sign(0) = +1; the iteration starts from the constant unit vector and runs
 * `iters` (>= 1) rounds of  u <- |Z| v / ||.||,  v <- |Z|^T u,  sigma <- ||v||,  v <- v / sigma;
 * a = sigma u, m = v (so ||m|| = 1).  (The kernels keep the iterate unnormalised between the passes
 * and divide at the end: the same values up to fp32 rounding.)
 *   Z_dev:    device, fp32 [rows][cols] row major (read only); NaNs are not supported.
 *   a_dev:    device, fp32 [rows] out;   m_dev: device, fp32 [cols] out (also used as the iterate).
 *   bits_dev: device, dbf_tiled_bytes(rows, cols) bytes out: Sign(Z) in the tile layout of this
 *             library (dbf_untile_host turns a host copy into canonical words), padding bits zero.
 *   workspace_dev: device, 256-byte aligned, >= dbf_svid_workspace_bytes(rows, cols) bytes.
 * Asynchronous on hip_stream, allocates nothing; all reductions have a fixed order (results do not
 * depend on scheduling).  Errors: DBF_EINVAL (null / misaligned pointers, sizes out of range,
 * iters < 1), DBF_EWORKSPACE, DBF_EHIP. */
size_t dbf_svid_workspace_bytes(int rows, int cols); /* 0 if the sizes are out of range */
int dbf_svid(const void* Z_dev, int rows, int cols, int iters, void* a_dev, void* m_dev, void* bits_dev,
             void* workspace_dev, size_t workspace_bytes, void* hip_stream);

/* ---- one ADMM update (paper, section 3.2, the three-line update that follows the SVID definition) ----
 * The compression solves min ||B X - W|| with X constrained to the SVID form a . S . m^T by ADMM (the
 * alternating minimisation's subproblem min_A ||A B - W|| has this form after transposition):
 *     W_hat = (B^T B + rho I)^-1 (B^T W + rho (A - U)),   A' = SVID(W_hat + U),   U' = U + W_hat - A'.
 * B and W do not change during the inner iterations, so the two constant matrices are formed once
 *     Minv = (B^T B + rho I)^-1   (q x q),      C = B^T W   (q x r)
 * (dbf_admm_prepare below does that on the device from the packed fixed factor; any other source will do)
 * and this call does what is repeated, on the device, with the iterate kept in its factored form:
 *     Z = Minv^T (C + rho (a . S . m^T - U)) + U;   (S, a, m) <- SVID(Z);   U <- Z - a . S . m^T.
 * (Minv is symmetric in exact arithmetic; it is applied transposed, i.e. read by rows of the summation
 * index, so the result is defined for whatever the caller's inverse holds.)
 *   Minv_dev: device, fp32 [q][q] row major (read only).    C_dev: device, fp32 [q][r] row major (read only).
 *   rho: penalty factor, > 0 (the paper uses 1).   svid_iters: rounds of the power iteration, >= 1.
 *   a_dev: device, fp32 [q];  m_dev: device, fp32 [r];  bits_dev: device, dbf_tiled_bytes(q, r) bytes, the
 *          signs S in the tile layout (as dbf_svid writes them);  U_dev: device, fp32 [q][r].
 *          All four are read as the current iterate and overwritten with the next one.
 *   workspace_dev: device, 256-byte aligned, >= dbf_admm_workspace_bytes(q, r) bytes (two q x r fp32
 *          matrices and the SVID workspace).
 * Asynchronous on hip_stream, allocates nothing; results do not depend on scheduling.  NaNs unsupported.
 * Errors: DBF_EINVAL (null or misaligned pointers, sizes out of range, rho <= 0 or not finite,
 * svid_iters < 1), DBF_EWORKSPACE, DBF_EHIP. */
size_t dbf_admm_workspace_bytes(int q, int r); /* 0 if the sizes are out of range */
int dbf_admm_step(const void* Minv_dev, const void* C_dev, int q, int r, float rho, int svid_iters,
                  void* a_dev, void* m_dev, void* bits_dev, void* U_dev, void* workspace_dev,
                  size_t workspace_bytes, void* hip_stream);

/* dbf_admm_prepare: the two constant matrices of that update, formed on the device with the fixed factor left in
 * its packed form (section 3.2: B and W do not change during the inner iterations; section 3.2 "alternating
 * minimisation": the fixed factor is itself a sign matrix with two scale vectors).  In the least-squares form
 * min ||B X - W|| the fixed factor is
 *     B = diag(b) S^T diag(m2)   (p x q),   i.e.  B[l][j] = b[l] * S[j][l] * m2[j],
 * with S (q x p, entries +-1) the packed sign matrix (for the left-factor update of a layer: S = the layer's B
 * signs, q = k, p = n_in, b its input scales, m2 the part of the middle scales that stays with it).  Computes
 *     C = B^T W  (q x r)     and     Minv = (B^T B + rho I)^-1  (q x q)
 * by fp32 matrix-core contractions that read the sign tiles directly (B is never stored densely), a blocked
 * Cholesky factorisation B^T B + rho I = R^T R (blocks of 128), the inverse of the factor and one more
 * contraction.  The outputs are what dbf_admm_step takes (Minv is symmetric up to rounding).
 *   bits_dev: device, dbf_tiled_bytes(q, p) bytes: S in the tile layout, rows q, columns p (read only).
 *   m2_dev: device fp32 [q];  b_dev: device fp32 [p];  W_dev: device fp32 [p][r] row major (all read only).
 *   rho > 0.   Minv_dev: device fp32 [q][q] out;   C_dev: device fp32 [q][r] out.
 *   workspace_dev: device, 256-byte aligned, >= dbf_admm_prepare_workspace_bytes(p, q, r) bytes (a q x q matrix
 *          and the inverses of the diagonal blocks).
 *   not_positive_definite_dev: device int (4-byte aligned) or NULL: set to the number of diagonal blocks whose
 *          factorisation met a non-positive pivot (0 = fine; with rho > 0 the matrix is positive definite and
 *          this only happens when rounding swamps rho).  Read it with an ordinary stream-ordered copy.
 * Asynchronous on hip_stream, allocates nothing, results do not depend on scheduling.
 * Errors: DBF_EINVAL (null or misaligned pointers, sizes out of range, rho <= 0 or not finite), DBF_EWORKSPACE, DBF_EHIP. */
size_t dbf_admm_prepare_workspace_bytes(int p, int q, int r); /* 0 if the sizes are out of range */
int dbf_admm_prepare(const void* bits_dev, const void* m2_dev, const void* b_dev, const void* W_dev, int p, int q, int r,
                     float rho, void* Minv_dev, void* C_dev, void* workspace_dev, size_t workspace_bytes,
                     int* not_positive_definite_dev, void* hip_stream);

/* ---- a group of independent layer products in one launch -------------------------------
 * Decode of several layers whose inputs do not depend on each other (q/k/v, gate/up, or a
 * benchmark stream of layers): the B and A stages of all layers run in one launch (two for
 * DBF_GEMV_VALU, DBF_GEMV_MFMA_SPLIT and short groups under DBF_GEMV_AUTO, four where DBF_GEMV_AUTO
 * quantises the stage inputs once per call), so the sign bits stream from HBM without a launch gap per layer.
 *
 * dbf_stack_create: layers[0..n_layers) must stay alive while the stack exists; the stack
 * only holds a device table describing them.  n_layers >= 1.  A layer may appear only once
 * in a stack (its scratch would be shared by two products of one launch): DBF_EINVAL.
 * dbf_stack_gemv: x_dev is the concatenation over layers of fp16 [batch][n_in_i] blocks,
 * y_dev the concatenation of fp16 [batch][n_out_i] blocks; layer i's blocks start at
 * element offsets batch * (sum of n_in_j, j<i) and batch * (sum of n_out_j, j<i), which
 * dbf_stack_offsets also reports.
 *
 * dbf_stack_create_grouped: the same with groups of consecutive layers that read ONE input
 * block (the projections of one activation vector: q, k, v; gate, up -- section 3 defines the
 * product per layer, the grouping only says which x a layer is given).  group_sizes[0..n_groups)
 * are positive and sum to n_layers; the layers of a group must have equal n_in (DBF_ESHAPE).
 * x_dev then holds one fp16 [batch][n_in] block per GROUP, in group order; dbf_stack_offsets
 * reports the same x offset for every layer of a group (and, at layer_index == n_layers, the
 * total), y offsets as before.  group_sizes == NULL: every layer its own group.
 */
int dbf_stack_create(const dbf_layer* const* layers, int n_layers, dbf_stack** out);
int dbf_stack_create_grouped(const dbf_layer* const* layers, int n_layers, const int* group_sizes,
                             int n_groups, dbf_stack** out);
int dbf_stack_offsets(const dbf_stack* stack, int layer_index, int batch,
                      size_t* x_offset_elems, size_t* y_offset_elems);
int dbf_stack_gemv(const dbf_stack* stack, const void* x_dev, void* y_dev, int batch, int kind,
                   void* hip_stream);
int dbf_stack_sync_timeouts(const dbf_stack* stack, int* timeouts); /* as dbf_sync_timeouts */
void dbf_stack_free(dbf_stack* stack); /* NULL is allowed */

/* Measurement aid: dbf_stack_gemv with HIP events recorded on `hip_stream` around its
 * launches.  Blocks until the last launch has finished.  *ms_first is the elapsed time of the
 * first kernel (the whole pass for DBF_GEMV_MFMA, the B stage for the two-launch kinds),
 * *ms_second that of the second kernel (0 for DBF_GEMV_MFMA).  Either pointer may be NULL.
 * Same arguments and errors as dbf_stack_gemv. */
int dbf_stack_gemv_timed(const dbf_stack* stack, const void* x_dev, void* y_dev, int batch,
                         int kind, void* hip_stream, float* ms_first, float* ms_second);

/* Measurement aid: launches a kernel on `hip_stream` that reads the first
 * floor(bytes / 65536) * 65536 bytes of src_dev (device, 16-byte aligned, bytes >= 65536) once
 * with 16-byte per-lane loads and does nothing else; timing it gives the practical HBM read
 * ceiling the decode kernels are compared with.  sink_dev: device, 4 bytes, or NULL.
 * Asynchronous.  Errors: DBF_EINVAL, DBF_EHIP. */
int dbf_probe_read(const void* src_dev, size_t bytes, void* sink_dev, void* hip_stream);

/* Measurement aid: launches a kernel on `hip_stream` that issues int8 matrix instructions on
 * independent accumulators and nothing else: `iters` iterations of 128 accumulator registers'
 * worth of instructions (2^19 multiply-adds for wide = 0, 2^18 for wide = 1) per wavefront,
 * wavefronts_per_simd (1..4) wavefronts on every SIMD of the current device.
 *   wide = 0: v_mfma_i32_16x16x64_i8 (the prefill stage kernel's instruction); 1: v_mfma_i32_32x32x32_i8.
 *   with_ands != 0: the sign operand is remade by 4 ANDs for every group of matrix instructions that
 *     the prefill kernel feeds from one masked operand (4 for wide = 0, 2 for wide = 1).
 * Timing it gives what the matrix pipe sustains for that instruction mix, next to the data-sheet
 * peak.  *ops (host, may be NULL) receives the integer operations of the launch (2 per
 * multiply-add).  sink_dev: device, 4 bytes, or NULL.  Asynchronous.  Errors: DBF_EINVAL, DBF_EHIP. */
int dbf_probe_mfma(int wide, int with_ands, int wavefronts_per_simd, int iters, void* sink_dev,
                   void* hip_stream, double* ops);

/* ---- tuning and test hooks ---------------------------------------------------------------
 * Process-wide integers that steer how launch plans are cut and how launches behave.  The defaults are
 * what the measurements in this repository were taken with; the hooks exist so that tests can force the
 * rarely taken code paths (column pieces on short rows, the bounded wait giving up) and so that the cuts
 * can be re-tuned on other shapes.  The library reads no environment variables.
 * A knob is read when a plan is built (dbf_pack*, dbf_prune_middle, dbf_stack_create*: the PLAN knobs)
 * or when a launch is issued (the LAUNCH knobs); changing one never affects plans that already exist.
 * Not thread safe against concurrent pack / create / launch calls.
 *   dbf_tuning_set:   DBF_EINVAL for an unknown knob or a value outside the stated range.
 *   dbf_tuning_get:   the current value, or INT_MIN for an unknown knob.
 *   dbf_tuning_reset: every knob back to its default. */
enum {
    /* PLAN knobs */
    DBF_TUNE_COL_PIECES = 0,          /* -1 (default): cut long rows of small launches into column pieces by the
                                         built-in rule; 0: never cut; N in 1..64: cut into N wherever N pieces of
                                         at least 8 column tiles fit                                              */
    DBF_TUNE_PIECE_TARGET = 1,        /* 0 (default): built-in (256 workgroups per stage, 1024 if the stage already
                                         has more than 256 row tiles); else that many workgroups per stage, 1..65536 */
    DBF_TUNE_PIECE_MIN_TILES = 2,     /* smallest piece in column tiles, 1..4096 (default 24)                      */
    DBF_TUNE_PIECE_NEVER_TILES = 3,   /* rows of at most this many column tiles are never cut, 0..65536 (default 64) */
    DBF_TUNE_PIECE_MAX_ROW_TILES = 4, /* plans with more row tiles per stage are never cut, 0..2^20 (default 768)   */
    DBF_TUNE_STACK_SPAN_B = 5,        /* row tiles per B-stage workgroup in stacks: 0 (default) = chosen per layer  */
    DBF_TUNE_STACK_SPAN_A = 6,        /*   from the launch size, else 1..16; the same for the A stage              */
    /* LAUNCH knobs */
    DBF_TUNE_SHARED_Q = 7,            /* batches >= 2: -1 (default) built-in choice; 0: every workgroup quantises its
                                         own input; 1: input quantised once per call and copied to LDS; 2: read from
                                         memory tile by tile; 3: the same with a row tile per wavefront             */
    DBF_TUNE_SHARED_MIN_BATCH = 8,    /* smallest batch that takes the once-per-call quantisation, 1..17 (default 2) */
    DBF_TUNE_SHARED_LDS_KB = 9,       /* LDS budget per workgroup for the copied input, 16..64 KiB (default 52)     */
    DBF_TUNE_WAIT_LIMIT_US = 10,      /* bound of the device-side wait in microseconds, 0..10 000 000 (default
                                         250 000); 0 makes every wait that is not already satisfied give up        */
    /* PLAN knob */
    DBF_TUNE_LONG_ROWS = 11,          /* -1 (default): plans of several layers, most of whose sign bytes are in layers
                                         with one stage input longer than 6144 values and the other longer than 4096,
                                         quantise every stage input once per call at batch 1 too (four launches per
                                         call instead of one); 0: no plan does; 1: every plan does                  */
    /* LAUNCH knob */
    DBF_TUNE_GEMM_SPLITS = 12,        /* dbf_gemm / dbf_gemm_static of up to 512 tokens: -1 (default): a stage that
                                         would start at most 64 workgroups (256 rows x 64 tokens each; 128 if it
                                         has 8192 columns or more) cuts its columns into 4 shares; 1: never; N in
                                         2..1024: N shares (at most one per 64 columns)                            */
    DBF_TUNE_FUSED_MIN_B_ITEMS = 13,  /* DBF_GEMV_AUTO at batch 1 runs both stages of a group of layers in one launch
                                         only if the B stage has at least this many workgroups, else in a launch per
                                         stage; 0..2^20 (default 1024: what the chip holds at once)                  */
    DBF_TUNE_WIDE_WG_MAX_ITEMS = 14,  /* a launch of at most this many self-quantising whole-row workgroups at batch
                                         1..8, over stage inputs of 2048 columns or more, gives each 8 wavefronts
                                         instead of 4; 0..2^20 (default 256: one workgroup per compute unit at most) */
    DBF_TUNE_FP4_MAX_ITEMS = 15,      /* batch-1 launches of at most this many whole-row workgroups over stage inputs of at
                                         most 4096 columns (2048 at least), all readable in 16-byte pieces, feed the matrix cores fp4
                                         sign operands and bf6 digits of the input (same bits out, half the
                                         instructions per tile, but two workgroups per compute unit at most: for
                                         launches that do not fill the chip); 0..2^20 (default 256), 0: never       */
    DBF_TUNE_COUNT_ = 16
};
int dbf_tuning_set(int knob, int value);
int dbf_tuning_get(int knob);
void dbf_tuning_reset(void);

const char* dbf_strerror(int code);

#ifdef __cplusplus
}
#endif
#endif /* DBF_H */
