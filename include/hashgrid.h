/*
 * hashgrid.h - C ABI of the multiresolution hash encoding for AMD MI355X (gfx950).
 *
 * The encoding y = enc(x; theta) is the one of Section 3 of "Instant Neural
 * Graphics Primitives with a Multiresolution Hash Encoding" (Eq. 2-4, Fig. 3):
 * for each of L levels of resolution N_l = floor(N_min * b^l) (Eq. 2-3) the
 * point x in [0,1)^d is scaled by N_l, the 2^d corners of its voxel are mapped
 * to entries of that level's feature array (1:1 where (N_l+1)^d <= T, else by
 * the spatial hash of Eq. 4), the F-wide feature vectors are gathered and
 * d-linearly interpolated with weights w_l = x_l - floor(x_l), and the L
 * results are concatenated.  The backward pass accumulates dL/dy times the
 * interpolation weight into the gathered entries (Fig. 3 caption).
 *
 * Conventions shared by every entry point
 *   - Every data pointer is a DEVICE pointer owned by the caller; the library
 *     never allocates, frees or copies device memory and never synchronises.
 *     Work is enqueued on `stream` (a hipStream_t passed as void*; NULL is the
 *     default stream) and the call returns at once.
 *   - x is fp32, row-major [B, d], every coordinate finite and in [0,1).  This
 *     is a precondition; coordinates outside the range give unspecified values
 *     but never an out-of-bounds access.
 *   - Tables (theta) are one flat array [n_entries, F] of `param_dtype`:
 *     level-major, entry-major, feature-minor; level l starts at entry
 *     `entry_offset` reported by hashgrid_level_info and holds `n_entries`
 *     entries, with no padding between levels.
 *   - y and dL/dy are row-major [B, L*F] of `io_dtype`, level-major inside a row
 *     (the concatenation of Fig. 3, step 4).
 *   - Table gradients have the shape of theta and are of `grad_dtype`: fp32, or fp16 as the paper
 *     accumulates them (Section 4, "Performance considerations"; Fig. 5).  An fp16 gradient buffer
 *     must start on a 4-byte boundary and its allocation must extend to one (packed two-half
 *     atomics).  fp16 sums lose precision with every rounded addition; the sorted pass
 *     (hashgrid_encode_bwd_ws) sums exactly and rounds once per call where one workgroup owns the
 *     chunk.  hashgrid_adam_step takes fp32 gradients, hashgrid_adam_step_half_grad fp16 ones.
 *   - Alignment: x 4 bytes; tables, y, dL/dy and gradients one entry (F scalars of their type) or
 *     16 bytes, whichever is smaller; anything less is HG_ERR_INVALID_ARG.  The fastest kernels
 *     want 16 bytes and rows of y that are a multiple of 16 bytes; other cases take a slower path.
 *   - Errors are returned as status codes; nothing aborts or throws.  B = 0 is
 *     HG_OK and launches nothing.
 *   - Every entry point only launches kernels on the caller's stream (no allocation, no memset,
 *     no synchronisation), so calls can be recorded into a HIP graph.  What a call derives on the
 *     host from its scalar arguments travels as kernel arguments and is fixed at capture: a
 *     replayed hashgrid_adam_step repeats the bias correction of the `step` it was recorded with
 *     (callers that replay update the node's arguments or record one node per step).
 */
#ifndef HASHGRID_H
#define HASHGRID_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define HG_MAX_LEVELS 32u
#define HG_MAX_BATCH (1u << 28) /* points per call; larger B returns HG_ERR_UNSUPPORTED */

typedef struct hashgrid hashgrid_t; /* opaque, host memory, owned by the library */

typedef enum {
  HG_OK = 0,
  HG_ERR_INVALID_ARG = 1, /* NULL pointer, zero size, N_max < N_min, level out of range ... */
  HG_ERR_UNSUPPORTED = 2, /* d > 3, F not in {1,2,4,8}, L > HG_MAX_LEVELS, table too large      */
  HG_ERR_ALLOC = 3,       /* host allocation of the handle failed                               */
  HG_ERR_DEVICE = 4       /* the HIP runtime refused a launch                                   */
} hg_status;

typedef enum { HG_F32 = 0, HG_F16 = 1 } hg_dtype;

typedef enum {
  HG_INTERP_LINEAR = 0,    /* Section 3: weights w and 1-w                                        */
  HG_INTERP_SMOOTHSTEP = 1 /* Appendix A: weights S(w) = w^2 (3-2w), levels shifted by 1/(2 N_l)  */
} hg_interp;

typedef enum {
  HG_BWD_COUNTED = 1,  /* the workspace already holds the counts of these points (hashgrid_encode_fwd_ws) */
  HG_BWD_OVERWRITE = 2 /* grad_params = the gradient of this batch, not += (no need to clear it first)   */
} hg_bwd_flags;

typedef struct {
  uint32_t d;           /* input dimensions: 1, 2 or 3 (Eq. 4 defines three primes)              */
  uint32_t L;           /* levels, 1..HG_MAX_LEVELS (Table 1: 16)                                */
  uint32_t F;           /* features per entry: 1, 2, 4 or 8 (Table 1: 2)                         */
  uint32_t T;           /* maximum entries per level (Table 1: 2^14 .. 2^24); any value >= 1    */
  uint32_t N_min;       /* coarsest resolution (Table 1: 16)                                    */
  uint32_t N_max;       /* finest resolution, >= N_min (Table 1: 512 .. 524288)                 */
  uint32_t param_dtype; /* hg_dtype of the tables                                               */
  uint32_t io_dtype;    /* hg_dtype of y and dL/dy                                              */
  uint32_t interp;      /* hg_interp                                                            */
  uint32_t grad_dtype;  /* hg_dtype of the table gradients: HG_F32, or HG_F16 as in the paper   */
} hashgrid_config;

/* Builds the level table of Eq. 2-3 on the host: N_l, the 1:1-or-hashed decision
 * of Section 3 and the entry offsets.  No device work.  *out is set on HG_OK only. */
hg_status hashgrid_create(const hashgrid_config* cfg, hashgrid_t** out);

/* Frees the handle (NULL is accepted).  The caller must have finished every
 * stream that still runs work enqueued through it: kernels hold no reference
 * to the handle, so this is only about the caller's own bookkeeping. */
void hashgrid_destroy(hashgrid_t* hg);

/* Sum over levels of the entries per level; the tables hold n_entries * F scalars
 * (Section 3: bounded by T * L * F).  0 for a NULL handle. */
uint64_t hashgrid_n_entries(const hashgrid_t* hg);

/* Level l of the table of Eq. 2-3: resolution N_l, first entry, entry count
 * ((N_l+1)^d when 1:1, else T) and whether the level is 1:1 indexed.  Output
 * pointers may be NULL. */
hg_status hashgrid_level_info(const hashgrid_t* hg, uint32_t l, uint32_t* N_l, uint64_t* entry_offset,
                              uint32_t* n_entries, int* is_dense);

/* Forward pass (Section 3; Fig. 3 steps 1-4): y[b, l*F+f] = sum over the 2^d
 * corners of weight * theta_l[index(corner)][f].
 *   x      [B, d]          fp32, device, read
 *   params [n_entries, F]  param_dtype, device, read
 *   y      [B, L*F]        io_dtype, device, written in full */
hg_status hashgrid_encode_fwd(const hashgrid_t* hg, uint32_t B, const float* x, const void* params, void* y,
                              void* stream);

/* Backward pass to the tables (Fig. 3 caption; collisions are summed):
 * grad_params[offset_l + index(corner), f] += weight * dLdy[b, l*F+f].
 *   dLdy        [B, L*F]        io_dtype, device, read
 *   grad_params [n_entries, F]  grad_dtype, device, ACCUMULATED INTO with atomic adds
 *                               (zeroing it is the caller's job; the summation
 *                               order, hence the last bits, varies run to run) */
hg_status hashgrid_encode_bwd(const hashgrid_t* hg, uint32_t B, const float* x, const void* dLdy,
                              void* grad_params, void* stream);

/* Size in bytes of the scratch buffer hashgrid_encode_bwd_ws needs for a batch of
 * B points, or 0 when that variant does not serve this configuration or batch
 * (it needs at most 4096 chunks of 4096 entries per level, 2048 entries at F = 8, i.e. levels of
 * at most 2^24 (2^23) entries, at most 4096 (2048) vertices per axis on the 1:1 levels of a
 * power-of-two T, and fewer than 2^32 records).  The buffer holds one record of 8 + F *
 * sizeof(dLdy scalar) bytes (rounded up to 4) per pair of corners along dimension 0,
 * B*L*2^(d-1) of them, or per corner, B*L*2^d of them, where the two corners of a pair are not
 * neighbours in memory (T not a power of two: Eq. 4's mod T; d = 1), plus 4 bytes per (tile of
 * 512 points, chunk), tiles of 4096 points where there are more than 16384 chunks in all:
 * 195 MiB at Table 1's sizes with 2^18 points, 1.6 GiB at T = 2^24 with 2^21. */
uint64_t hashgrid_bwd_workspace_bytes(const hashgrid_t* hg, uint32_t B);

/* 1 when hashgrid_encode_bwd_ws serves this configuration and batch and is expected to be the
 * faster of the two backward passes, else 0: it visits every chunk of the gradient whatever the
 * batch, so below some ten thousand points (at Table 1's sizes) the atomic pass wins, except
 * where a level is so small that the atomic requests of the batch queue up on a few of its
 * entries (a host-side estimate from sizes alone; points are taken as evenly spread). */
int hashgrid_bwd_ws_pays(const hashgrid_t* hg, uint32_t B);

/* Backward pass to the tables, same result as hashgrid_encode_bwd (Fig. 3
 * caption), computed without device-wide atomics on the hot path: the
 * weight * dLdy contributions are bucket-sorted by destination chunk into
 * `workspace` and each chunk is summed on-chip by one owner.  Sums are exact
 * 64-bit fixed point scaled to the largest |dLdy| of the call (each summand is
 * rounded to about 2^-38 of that value or finer), so the result does not depend
 * on the order of execution, except on coarse 1:1 levels whose few chunks are
 * shared by several workgroups and combined with fp32 atomic adds.  The sorted
 * records carry the interpolation weights with relative precision (2^-20; along
 * dimension 0 exactly, except 2^-17 in the first voxel): a gradient entry differs
 * from the exact sum by at most 1e-5 of the sum of the absolute values of its
 * summands, as hashgrid_encode_bwd's does, plus the fixed-point rounding above.
 *   workspace  device, 256-byte aligned, at least hashgrid_bwd_workspace_bytes(hg, B)
 *              bytes, owned by the caller; contents are scratch: undefined on
 *              entry and on exit.  Calls that overlap in time need separate
 *              workspaces.
 *   flags      0, or any of: HG_BWD_COUNTED when hashgrid_encode_fwd_ws has just run on the same
 *              hg, B, x and workspace (see there); HG_BWD_OVERWRITE to have every entry of
 *              grad_params written with what the call without this flag leaves in a buffer of
 *              zeros (untouched entries become 0), which spares the caller the clearing pass
 *              and this call the reading of the old values.
 * Returns HG_ERR_UNSUPPORTED when hashgrid_bwd_workspace_bytes is 0 and
 * HG_ERR_INVALID_ARG when the buffer is missing, misaligned or too small or a flag is
 * unknown.  x and dLdy must not be written while the call is in flight. */
hg_status hashgrid_encode_bwd_ws(const hashgrid_t* hg, uint32_t B, const float* x, const void* dLdy,
                                 void* grad_params, void* workspace, uint64_t workspace_bytes, uint32_t flags,
                                 void* stream);

/* hashgrid_encode_bwd_ws for callers that cannot allocate and have no scratch buffer to pass: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments,
 * result and error codes, minus the workspace: the scratch is a fixed array of
 * HG_STATIC_SCRATCH_BYTES in device memory that belongs to the library (each GPU the library runs on
 * holds its own copy from the time the library is loaded until the process ends).  The call itself
 * allocates and frees nothing, on the host or on the device.
 *   flags  0 or HG_BWD_OVERWRITE (HG_BWD_COUNTED needs a caller-owned workspace: HG_ERR_INVALID_ARG)
 * Returns HG_ERR_UNSUPPORTED when hashgrid_bwd_workspace_bytes(hg, B) is 0 or larger than
 * HG_STATIC_SCRATCH_BYTES (at Table 1's sizes: batches beyond about 87 000 points), HG_ERR_DEVICE
 * when the array cannot be located on the current device.
 * All calls on one GPU share that GPU's array: two calls that overlap in time on one GPU (different
 * streams, or different threads) race; calls on one stream, or otherwise ordered, are fine.  The
 * array keeps what the last call left; nothing in it needs clearing between calls. */
#define HG_STATIC_SCRATCH_BYTES (64u << 20)
hg_status hashgrid_encode_bwd_static(const hashgrid_t* hg, uint32_t B, const float* x, const void* dLdy,
                                     void* grad_params, uint32_t flags, void* stream);

/* Forward pass, the arithmetic of hashgrid_encode_fwd (Section 3; Fig. 3 steps 1-4; an fp16 output
 * that is an exact tie may differ from that call's in its last bit), that also does
 * the first step of hashgrid_encode_bwd_ws for the same points while it gathers: it counts, per
 * tile of points and chunk of the gradient, the corner pairs that the backward pass will sort,
 * and leaves the counts in `workspace`.  A following hashgrid_encode_bwd_ws on the same hg, B, x
 * and workspace may then pass HG_BWD_COUNTED and skips its own counting pass.  Nothing else may
 * write the workspace in between, and x must be unchanged.
 * Where the counting cannot ride along (batches too small to give every compute unit a full
 * workgroup, configurations whose records are per corner) the call runs hashgrid_encode_fwd and
 * the counting pass one after the other, with the same result.
 * (What the counting costs this call depends on the order of the points: a few percent of it on
 * batches in random order, against a counting pass of a seventh of it; on batches whose
 * neighbours share voxels, samples in ray order, the forward waits less for the tables and the
 * counting costs as much as the separate pass: there hashgrid_encode_fwd and no flag is as fast.)
 * Returns HG_ERR_UNSUPPORTED when hashgrid_bwd_workspace_bytes is 0, when y or params are not
 * 16-byte / entry aligned, or when the configuration has more than 16384 chunks in all (callers
 * then use hashgrid_encode_fwd and pass no flag); HG_ERR_INVALID_ARG as hashgrid_encode_bwd_ws. */
hg_status hashgrid_encode_fwd_ws(const hashgrid_t* hg, uint32_t B, const float* x, const void* params, void* y,
                                 void* workspace, uint64_t workspace_bytes, void* stream);

/* Gradient with respect to the input position (chain rule on the weight
 * definition of Section 3; S' of Appendix A for the smoothstep variant):
 * dLdx[b, j] = sum_{l,f} dLdy[b, l*F+f] * d y[b, l*F+f] / d x_j.
 *   dLdx [B, d] fp32, device, written in full */
hg_status hashgrid_encode_bwd_input(const hashgrid_t* hg, uint32_t B, const float* x, const void* params,
                                    const void* dLdy, float* dLdx, void* stream);

/* The integer decisions of one level, for bit-exact checks: level-local entry
 * indices idx [B, 2^d] uint32 (corner m is the upper corner along dimension i
 * when bit i of m is set) and fractional positions w [B, d] fp32 (before any
 * smoothstep).  Either output may be NULL. */
hg_status hashgrid_debug_indices(const hashgrid_t* hg, uint32_t B, const float* x, uint32_t level, uint32_t* idx,
                                 float* w, void* stream);

/* The precondition of every call above, checked on request (Appendix E.1 bounds scenes to the unit
 * cube; the kernels clamp instead of checking): adds to *count the number of coordinates of x that
 * are not in [0,1), NaN and infinities included.
 *   count  one uint32, device, 4-byte aligned, ADDED TO (clear it first) */
hg_status hashgrid_debug_count_outside(const hashgrid_t* hg, uint32_t B, const float* x, uint32_t* count,
                                       void* stream);

/* Hyper-parameters of the optimiser step below (paper Section 4, "Training": Adam with
 * beta1 = 0.9, beta2 = 0.99, eps = 1e-15; learning rate 1e-2, 1e-4 for signed distance
 * functions; an L2 regularisation of factor 1e-6 on the network's weights and none on table
 * entries: l2_reg * value is added to every gradient scalar, 0 switches it off). */
typedef struct {
  float lr, beta1, beta2, eps;
  float l2_reg;
} hashgrid_adam_config;

/* One Adam step (Kingma & Ba, Algorithm 1, with bias correction for the 1-based global
 * `step`) on n_scalars table scalars or network weights, following Section 4 of the paper: a
 * scalar whose gradient (with the regulariser's term, if any) is exactly 0 is skipped (value and
 * both moments untouched); the full-precision
 * master copy is updated and, when params_half is not NULL, rounded (nearest even) into the
 * half-precision working copy the encoding kernels read.  All arithmetic fp32.
 *   params_master [n] fp32  device, 16-byte aligned, read and written
 *   params_half   [n] fp16  device, 8-byte aligned, written where updated; may be NULL
 *   grad          [n] fp32  device, 16-byte aligned, read; set to 0 where it was not when
 *                           zero_grad != 0 (so the next backward pass can accumulate into it)
 *   m, v          [n] fp32  device, 16-byte aligned, first and second moment, read and written
 * Returns HG_ERR_INVALID_ARG for step == 0, betas outside [0,1), negative eps or l2_reg, NULL or
 * misaligned pointers.  n_scalars == 0 is HG_OK. */
hg_status hashgrid_adam_step(uint64_t n_scalars, float* params_master, void* params_half, float* grad, float* m,
                             float* v, const hashgrid_adam_config* cfg, uint32_t step, int zero_grad, void* stream);

/* The same step (Section 4, "Training", as above) on a half-precision gradient, as the backward
 * passes write it with grad_dtype = HG_F16 (Section 4, "Performance considerations": half-precision
 * tables and gradients, a full-precision master copy for the update).  Every gradient scalar is
 * converted to fp32 and multiplied by grad_scale before use: 1, or the reciprocal of the factor by
 * which the caller scaled the loss to keep small half-precision gradients out of the subnormal
 * range (a power of two keeps the product exact).
 *   grad_half  [n] fp16  device, 8-byte aligned, read; set to 0 where it was not when zero_grad != 0
 *   grad_scale           finite and positive, else HG_ERR_INVALID_ARG
 * Everything else as hashgrid_adam_step. */
hg_status hashgrid_adam_step_half_grad(uint64_t n_scalars, float* params_master, void* params_half, void* grad_half,
                                       float* m, float* v, const hashgrid_adam_config* cfg, uint32_t step,
                                       int zero_grad, float grad_scale, void* stream);

/* The encoding followed by the paper's network (Section 4, "Architecture": two hidden layers of 64
 * neurons, ReLU on the hidden layers, a linear output layer), in one kernel: the encoded features
 * never reach memory.  out[b, i] = sum_k W3[i,k] h2[k], h2 = relu(W2 h1), h1 = relu(W1 y),
 * y = enc(x_b; params).  Half-precision operands on the matrix cores with fp32 accumulation: y, h1
 * and h2 are rounded to fp16 (nearest even) where they are stored, out is fp32.
 *   params  [n_entries, F]  fp16 (param_dtype must be HG_F16), device, read
 *   W1      [64, L*F]       fp16, device, 8-byte aligned (as W2, W3), read; row = neuron
 *   W2      [64, 64]        fp16
 *   W3      [n_out, 64]     fp16, 1 <= n_out <= 32
 *   out     [B, n_out]      fp32, device, written in full
 * A network with one hidden layer (the density network of the paper's radiance fields, Section 4,
 * "Architecture") is this one with W2 = identity: relu(h1) = h1 exactly, in every entry point below too.
 * HG_ERR_UNSUPPORTED unless d is 2 or 3, T a power of two, L*F a multiple of 8 and at most 64 and
 * the tables fp16; HG_ERR_INVALID_ARG for NULL or misaligned pointers or n_out == 0. */
hg_status hashgrid_encode_mlp_fwd(const hashgrid_t* hg, uint32_t B, const float* x, const void* params,
                                  const void* W1, const void* W2, const void* W3, uint32_t n_out, float* out,
                                  void* stream);

/* hashgrid_encode_mlp_fwd for training: the same call, which also writes the encoded features as the
 * network saw them (rounded to fp16) for the backward pass of the network below.
 *   y  [B, L*F]  fp16, device, 16-byte aligned, written in full */
hg_status hashgrid_encode_mlp_fwd_train(const hashgrid_t* hg, uint32_t B, const float* x, const void* params,
                                        const void* W1, const void* W2, const void* W3, uint32_t n_out, float* out,
                                        void* y, void* stream);

/* That network alone (Section 4, "Architecture"), on features that are in memory: for a second
 * network whose inputs are not (only) this encoding's output, or to re-evaluate the network on kept
 * features.  Same arithmetic as the network part of hashgrid_encode_mlp_fwd: y is read as fp16, h1 and
 * h2 are rounded to fp16, products accumulate in fp32 on the matrix cores.
 *   y    [B, n_in]   fp16, device, 16-byte aligned, read
 *   W1 [64, n_in], W2 [64, 64], W3 [n_out, 64]   fp16, device, 8-byte aligned, read
 *   out  [B, n_out]  fp32, device, written in full
 * HG_ERR_UNSUPPORTED unless n_in is a multiple of 8 and at most 64 and n_out at most 32;
 * HG_ERR_INVALID_ARG for NULL or misaligned pointers, n_in == 0 or n_out == 0.  B == 0 is HG_OK. */
hg_status hashgrid_mlp_fwd(uint32_t B, uint32_t n_in, uint32_t n_out, const void* y, const void* W1, const void* W2,
                           const void* W3, float* out, void* stream);

/* Backward pass of that network (Section 4, "Architecture"; chain rule through the three layers,
 * ReLU passing the gradient where its output is positive), in one kernel on the matrix cores.  The
 * hidden activations are recomputed from y.  Half-precision operands with fp32 accumulation: dL/dout
 * and the two hidden-layer gradients are rounded to fp16 where they enter the next product (callers
 * that train in half precision scale their loss accordingly).
 *   y       [B, n_in]   fp16, device, 16-byte aligned, read: the encoded features (n_in = L*F)
 *   W1, W2, W3          as in hashgrid_encode_mlp_fwd, read
 *   dLdout  [B, n_out]  fp32, device, read
 *   dLdy    [B, n_in]   fp16, device, 8-byte aligned, written in full: what hashgrid_encode_bwd[_ws]
 *                       takes as dL/dy (io_dtype fp16)
 *   dW1 [64, n_in], dW2 [64, 64], dW3 [n_out, 64]   fp32, device, ACCUMULATED INTO (sums over the
 *                       batch; fp32 atomic adds, so the last bits vary from run to run)
 * HG_ERR_UNSUPPORTED unless n_in is a multiple of 8 and at most 64 and n_out at most 32;
 * HG_ERR_INVALID_ARG for NULL or misaligned pointers, n_in == 0 or n_out == 0.  B == 0 is HG_OK. */
hg_status hashgrid_mlp_bwd(uint32_t B, uint32_t n_in, uint32_t n_out, const void* y, const void* W1, const void* W2,
                           const void* W3, const float* dLdout, void* dLdy, float* dW1, float* dW2, float* dW3,
                           void* stream);

/* Training losses (Section 4, "Training"): the squared error (p - t)^2 the paper uses for images and
 * radiance fields, and the mean absolute percentage error |p - t| / (|t| + 0.01) it uses for signed
 * distance functions.  (Its luminance-relative loss for radiance caching is defined elsewhere and
 * is not offered.) */
typedef enum { HG_LOSS_L2 = 0, HG_LOSS_MAPE = 1 } hg_loss;

/* The loss's derivative with respect to the network's output, per scalar and times `scale`, as
 * hashgrid_mlp_bwd takes it:  dLdout[i] = scale * 2 (p_i - t_i)  or  scale * sign(p_i - t_i) /
 * (|t_i| + 0.01), sign(0) = 0.  The paper's losses are means over the batch: callers pass
 * scale = 1/n, times the factor by which they scale the loss for half-precision gradients.
 * Arithmetic fp32.
 *   prediction, target [n] fp32  device, 4-byte aligned, read (n = B * n_out scalars)
 *   dLdout             [n] fp32  device, 4-byte aligned, written in full
 *   loss_sum           one fp64  device, 8-byte aligned, may be NULL: the UNSCALED loss values of the
 *                      n scalars are ADDED to it (clear it first; one atomic addition per
 *                      workgroup, so the last bits vary from run to run)
 * 16-byte aligned arrays are read and written four scalars at a time.  HG_ERR_INVALID_ARG for an
 * unknown loss, a scale that is not finite, NULL or misaligned pointers.  n == 0 is HG_OK. */
hg_status hashgrid_loss_grad(uint64_t n, const float* prediction, const float* target, uint32_t loss, float scale,
                             float* dLdout, double* loss_sum, void* stream);

/* Static, NUL-terminated description of a status code. */
const char* hashgrid_strerror(hg_status s);

#ifdef __cplusplus
}
#endif
#endif /* HASHGRID_H */
