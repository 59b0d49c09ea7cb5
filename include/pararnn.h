/*
 * pararnn.h -- C ABI of the MI355X (gfx950) implementation of the
 * sequence-parallel application of a nonlinear RNN (ParaRNN, arXiv 2510.21450).
 *
 * The library applies h_l = f(h_{l-1}, u_l), l = 1..L (Sec. 2, Eq. (1)) to all
 * L timesteps at once: the L equations are stacked into one nonlinear system
 * (Eq. (2)) and solved with Newton's method (Eq. (3), Alg. 1a); every Newton
 * iteration evaluates residuals and Jacobians for all timesteps in parallel
 * and solves the block bi-diagonal linear system with a prefix scan over
 * affine maps (the role of Alg. 1b).  The backward pass is the matching
 * reverse scan with transposed Jacobians (Eq. (6)).
 *
 * All data pointers are DEVICE pointers unless stated otherwise.  The caller
 * owns every buffer; the library allocates nothing and only enqueues work on the
 * given HIP stream (hipStream_t passed as void*, NULL = the default stream).
 * Results are valid once the stream has been synchronised.  Calls that share a
 * workspace must be ordered on one stream.
 *
 * State.  A call keeps nothing on the device beyond its workspace.  On the host
 * the library has a handful of process-wide tuning and test switches (the
 * pararnn_set_* functions below and the environment variable PARARNN_TILE, read
 * once): they are plain variables, NOT thread-safe, meant to be set before the
 * calls they affect and not while another thread is inside the library.  They
 * change the launch plan and with it the workspace size: query
 * pararnn_workspace_bytes again after any of them.  Code that wants per-call
 * choices, or calls from several threads, uses pararnn_forward_ex, whose options
 * travel with the call.
 *
 * Layouts (H is always the contiguous axis):
 *   u          [B][L][G][H]  pre-activations u_l = B x_l + b of the G gates
 *   h, dL_dh   [B][L][S][H]  states / loss gradients, S values per channel
 *   h0, dL_dh0 [B][S][H]
 *   params     always fp32.  Diagonal cells: [2][G][H] = recurrent weights,
 *              then biases (PARALSTM_DIAG: [8][H], see below).  Dense cell:
 *              W[H][H] row-major.
 * Gate order: GRU (z, r, c); LSTM (i, f, o, g).  LSTM state order (c, h).
 */
#ifndef PARARNN_H
#define PARARNN_H

#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Cells.  G gates, S state values per channel.
 *  GRU_DIAG   (G=3,S=1): Sec. 3, Eq. (7a) with diagonal A_* (Eq. (9)):
 *             z = sig(a_z h + u_z + b_z), r = sig(a_r h + u_r + b_r),
 *             c = tanh(a_c (r h) + u_c + b_c), h' = (1-z) h + z c.
 *             Jacobian: Eq. (8a), a scalar per channel.
 *  LSTM_DIAG  (G=4,S=2): i,f,o = sig(w_* h + u_* + b_*), g = tanh(w_g h + u_g + b_g),
 *             c' = f c + i g, h' = o tanh(c').  2x2 Jacobian block per channel
 *             (the structure of Eq. (8b)).
 *  TANH_DENSE (G=1,S=1): h' = tanh(W h + u), dense Jacobian diag(1-h'^2) W
 *             (the generic dense case of Sec. 2.1).
 *  LINEAR_DIAG(G=1,S=1): h' = a h + u + b, the linear SSM of the footnote in
 *             Sec. 2; used to test that one Newton solve is exact.
 *  PARALSTM_DIAG (G=3,S=2): the paper's ParaLSTM, Sec. 3, Eq. (7b) with diagonal
 *             A_*, C_* (Eq. (9)): f = sig(a_f h + u_f + c_f c + b_f),
 *             z = tanh(a_z h + u_z + b_z), c' = f c + (1-f) z,
 *             o = sig(a_o h + u_o + c_o c' + b_o), h' = o tanh(c'); Jacobian
 *             blocks Eq. (8b).  Gates (f, z, o); params [8][H] = a_f, a_z, a_o,
 *             c_f, c_o, b_f, b_z, b_o. */
typedef enum {
    PARARNN_GRU_DIAG = 0,
    PARARNN_LSTM_DIAG = 1,
    PARARNN_TANH_DENSE = 2,
    PARARNN_LINEAR_DIAG = 3,
    PARARNN_PARALSTM_DIAG = 4
} pararnn_cell_t;

/* Storage type of u, h0, h, dL_dh, dL_du, dL_dh0.  With BF16 all arithmetic,
 * the Newton iterate, scan carries and dL_dparams stay fp32; the iterate is
 * rounded to bf16 (nearest-even) once, when h is written. */
typedef enum { PARARNN_F32 = 0, PARARNN_BF16 = 1 } pararnn_dtype_t;

typedef enum {
    PARARNN_OK = 0,
    PARARNN_NOT_CONVERGED = 1,       /* device status only: max_iter reached */
    PARARNN_INVALID_ARG = 2,
    PARARNN_WORKSPACE_TOO_SMALL = 3,
    PARARNN_HIP_ERROR = 4,
    PARARNN_NONFINITE = 5,           /* device status only: max|dh| became inf/nan */
    PARARNN_UNSUPPORTED = 6,         /* valid request the library has no kernel for */
    PARARNN_INTERNAL = 7             /* device status only: a bounded wait ran out */
} pararnn_status_t;

/* Human-readable name of a status code (static string, host). */
const char *pararnn_status_string(int status);

/* Library version, major*10000 + minor*100 + patch. */
int pararnn_version(void);

/*
 * What the HIP runtime reports for the current device (host only; used by the
 * benchmark to print the machine's own figures beside the published peaks its
 * rooflines use).  info[0..5] = compute units, core clock in kHz, memory clock
 * in kHz, memory bus width in bits, L2 size in bytes, LDS bytes a workgroup may
 * use; -1 where the runtime gives no answer.  Returns the number of entries
 * written (6), or -1 if info is NULL, capacity is below 6 or no device is
 * current.
 */
int pararnn_device_info(int *info, int capacity);

/* Tuning / test hook (host, process-wide, not thread-safe): force the tile
 * shape of the scan kernels for all later calls -- vec channels per lane, ll
 * segments along L per wave, c timesteps per thread, w waves per workgroup.
 * Only shapes compiled into the library are accepted (else UNSUPPORTED); a
 * call whose H or pointer alignment does not allow `vec` keeps the automatic
 * choice.  vec = 0 restores the automatic choice.  Query workspace sizes
 * after setting it.  The environment variable PARARNN_TILE="vec,ll,c,w" has
 * the same effect at start-up. */
int pararnn_set_tile(int vec, int ll, int c, int w);

/* Gates G and state values S of a cell; -1 for an unknown cell. */
int pararnn_cell_gates(int cell);
int pararnn_cell_state(int cell);

/* Bytes of device workspace pararnn_forward (backward = 0) or
 * pararnn_backward (backward = 1) needs for this problem; 0 on invalid
 * arguments.  The workspace needs 256-byte alignment and no initialisation. */
size_t pararnn_workspace_bytes(int cell, int dtype, int B, int L, int H, int backward);

/* Workspace size that lets a fixed-count solve (tol < 0, 1 <= n_iters <= 8) run
 * all its iterations in ONE launch (the paper's "fully fused" mode, Sec. 4 item 3:
 * u is read once and h written once): one carry-record slot per iteration.  Never
 * smaller than pararnn_workspace_bytes(.., 0).  pararnn_forward takes the
 * one-launch path whenever tol < 0, max_iter <= 8 and the workspace it is given
 * is at least this large; otherwise it launches one kernel per iteration.  Both
 * paths compute the same iterations (results agree to fp32 rounding). */
size_t pararnn_workspace_bytes_fused(int cell, int dtype, int B, int L, int H, int n_iters);

/* Test hook (host, process-wide): the number of times a tile polls its
 * predecessor's carry record before it gives up (polls = 0: the default, about
 * two million, i.e. seconds).  A tile that gives up uses a zero carry, the call's
 * device status becomes PARARNN_INTERNAL and every wave still exits: with a tiny
 * limit this path can be exercised without any wait that does not end. */
int pararnn_set_spin_limit(unsigned int polls);

/* Test / tuning hook (host, process-wide): enable = 0 makes pararnn_forward
 * always launch one kernel per iteration (fixed-count solves and solves to a
 * tolerance alike); the returned h is then exactly the iterate of the stopping
 * iteration. */
int pararnn_set_fused(int enable);

/* Test / tuning hook (host, process-wide; default 1): enable = 0 keeps the kernels
 * from copying their inputs straight from memory into LDS ahead of their use:
 * the backward kernel of the diagonal cells (bf16 storage, rows 16-byte
 * aligned, H % 8 == 0), the forward and dx products of the input projection
 * (d_h >= 128; either storage type) and its weight-gradient sums (bf16 storage,
 * d_h = 192, 256, 448 and up).  They then load through registers.  The
 * backward kernel gives the same bits either way; the projection's kernels sum
 * in different orders and agree to fp32 rounding. */
int pararnn_set_staging(int enable);

/* Test / tuning hook (host, process-wide; default 0).  The kernels that run at
 * the speed of the memory (one Newton iteration per launch; the backward pass
 * for bf16 storage) can mark their tile accesses as streamed, which keeps
 * them out of the way of what the device's memory-side cache holds from the
 * launch before.  mode 0: chosen per call from the sizes of the tensors (u is
 * streamed once u and the fp32 iterate together exceed that cache, the iterate
 * and the backward pass's tensors once they exceed twice its size); 1: never;
 * 2: always.  The results are the same bits in every mode.  Returns
 * PARARNN_INVALID_ARG for another mode. */
int pararnn_set_streaming(int mode);

/* Tuning hook (host, process-wide): a solve to a tolerance (tol >= 0) runs its
 * first min(n_iters, max_iter) iterations in ONE launch of the fused kernel (u
 * read once, the iterate kept in registers), then blocks of 1, 2, 4, ...
 * iterations (at most n_iters each) until max_iter; a block of more than one
 * iteration is again one fused launch, resumed from the iterate.  The stopping
 * test still sees m_k of every iteration: `iters`, the status and delta_trace
 * are those of the per-iteration solve.  When the tolerance is met at an
 * iteration before the end of a launch, the returned h is the iterate at the
 * END of that launch -- the converged iterate refined by the Newton iterations
 * that were already in flight -- so it differs from the per-iteration path's h
 * by less than tol.  0 <= n_iters <= 8; 0 turns
 * it off; default 5.  Query workspace sizes after setting it (a workspace
 * that is too small for the record slots falls back to one launch per
 * iteration). */
int pararnn_set_fused_head(int n_iters);

/* Tuning / test hook (host, process-wide, not thread-safe; default 1): the blocks
 * of a solve to a tolerance that follow its second launch (the first fused
 * block, then one iteration of the per-iteration kernel) run in ONE more launch
 * of the fused kernel, which walks the rest of the plan on the device (grid-wide
 * barriers between blocks; the grid is what the device holds at once, and a
 * barrier wait is bounded like the look-back waits: pararnn_set_spin_limit) and
 * returns at once when the tolerance was met before.  enable = 0: every block is
 * a launch of its own, and the launches after the one that met the tolerance
 * return at once.  `iters`, status and delta_trace are the same either way. */
int pararnn_set_fused_tail(int enable);

/* Tuning hook (host, process-wide, not thread-safe; default 0).  enable = 1 is a
 * promise by the caller: between two calls of this library that are handed the
 * same workspace address on the same device, nothing but this library writes to
 * that memory (it is not freed and allocated anew, not used as scratch by
 * anybody else, not shared by calls that run at the same time).  pararnn_forward
 * and pararnn_backward of the diagonal and block-diagonal cells (user cells
 * included) then note, per device and address, the layout of the last call and
 * a call number, put the number into the tags of the carry records, and skip
 * the clearing of the records when the next call on that workspace has the same
 * layout: records of the earlier call carry another number and read as empty.
 * The records are cleared as always when the layout differs, for a new address,
 * every 2^20 calls, when max_iter > 1000, while the stream is being captured
 * into a graph (a captured launch sequence would replay one number), and after
 * any other entry point of the library or a failed call has used the workspace.
 * Results are bit-identical either way.  What it saves: the zero-fill, 0.26 ms of
 * a forward solve and 0.10 ms of a backward pass at 2^30 timestep-channels in
 * bf16 storage.  A broken promise can make a tile accept a stale record as its
 * predecessor's: wrong results without an error. */
int pararnn_set_workspace_reuse(int enable);

/* The blocks of Newton iterations pararnn_forward runs for a solve with these
 * settings when the workspace is of the size pararnn_workspace_bytes reports
 * (host only, no device work): writes the number of iterations of each block to
 * block_sizes[0 .. capacity) and returns the number of blocks (which may exceed
 * capacity), or -1 on invalid arguments.  The sizes add up to max_iter.  The
 * stopping test is evaluated for every iteration and acted on between blocks.
 * The first two blocks are launches of their own; the following ones share one
 * launch (pararnn_set_fused_tail) or are launches of their own. */
int pararnn_solve_plan(float tol, int max_iter, int *block_sizes, int capacity);

/*
 * Forward: solve Eq. (2) by Newton iterations (Alg. 1a).
 *   initial guess   h^0_l = f(h0, u_l) for every l (App. A; f(0, x_l) when h0 = 0)
 *   iteration k     r_l = f(h^{k-1}_{l-1}, u_l) - h^{k-1}_l,
 *                   J_l = df/dh at (h^{k-1}_{l-1}, u_l)        (Eq. (3))
 *                   delta_l = J_l delta_{l-1} + r_l, delta_0 = 0 (Eq. (4), as a
 *                   prefix scan over affine maps (A2,b2)o(A1,b1) = (A2A1, A2b1+b2))
 *                   h^k = h^{k-1} + delta;  m_k = max |delta| over the whole batch
 *   stop            when m_k <= tol (checked on the device after the update;
 *                   no host synchronisation per iteration) or k = max_iter.
 *
 *   params, u, h0   inputs; h0 may be NULL (= zeros, the paper's h_0 = 0)
 *   B, L, H         batch, timesteps, channels; H <= 4 194 304 (INVALID_ARG beyond: row
 *                   offsets inside the kernels are 32-bit)
 *   tol             absolute tolerance on max|delta h|; tol < 0 runs exactly
 *                   max_iter iterations (the paper's fixed N_its) with status OK
 *   max_iter        >= 0; 0 returns the initial guess
 *   h               out [B][L][S][H]; on NOT_CONVERGED the last iterate; on OK an
 *                   iterate at or after the one that met the tolerance (see
 *                   pararnn_set_fused_head)
 *   iters           out, DEVICE int32[2] = {iterations performed (number of
 *                   linear solves), device status (OK / NOT_CONVERGED /
 *                   NONFINITE / INTERNAL)}
 *   delta_trace     optional DEVICE float[max_iter]: m_k of each performed
 *                   iteration (entries past iters are left untouched); or NULL
 *   workspace       DEVICE scratch of at least pararnn_workspace_bytes(.., 0)
 * Returns PARARNN_OK when everything was enqueued, else the host-detectable
 * error (INVALID_ARG, WORKSPACE_TOO_SMALL, UNSUPPORTED, HIP_ERROR); on error
 * nothing useful has been written.
 */
int pararnn_forward(int cell, int dtype, const float *params, const void *u, const void *h0,
                    int B, int L, int H, float tol, int max_iter, void *h, int *iters,
                    float *delta_trace, void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * pararnn_forward with per-call choices instead of the process-wide switches
 * (two threads with different choices do not interfere; nothing is written to
 * the library's settings).
 *   first_block  Newton iterations the first launch of a solve to a tolerance
 *                runs on registers (u read once): -1 the library's setting
 *                (default 5), 0 one launch per iteration, 1..8.  The paper's
 *                regime of three iterations (Sec. 2.1, App. A) is first_block = 3:
 *                the returned h is then the iterate of the third iteration when
 *                the tolerance is met there, and a solve that needs more goes on
 *                in further launches.
 *   fused        -1 the library's setting, 0 never run more than one iteration
 *                per launch (as pararnn_set_fused(0)), 1 allow it.
 * options = NULL means all defaults: the call is then pararnn_forward.  Fields
 * out of range give PARARNN_INVALID_ARG.  The workspace must have
 * pararnn_workspace_bytes_ex bytes for the same options (0 on invalid
 * arguments); pararnn_solve_plan_ex is pararnn_solve_plan for given options.
 */
typedef struct pararnn_solve_options {
    int first_block;
    int fused;
} pararnn_solve_options_t;
size_t pararnn_workspace_bytes_ex(int cell, int dtype, int B, int L, int H, const pararnn_solve_options_t *options);
int pararnn_solve_plan_ex(float tol, int max_iter, const pararnn_solve_options_t *options, int *block_sizes,
                          int capacity);
int pararnn_forward_ex(int cell, int dtype, const float *params, const void *u, const void *h0,
                       int B, int L, int H, float tol, int max_iter, void *h, int *iters,
                       float *delta_trace, void *workspace, size_t workspace_bytes, void *hip_stream,
                       const pararnn_solve_options_t *options);

/*
 * pararnn_forward for callers that cannot allocate device memory or hand over
 * a workspace: code under HIP graph capture, tight serving loops, harnesses
 * that forbid hipMalloc.  Same arguments, results and status codes as
 * pararnn_forward without the workspace pair: the scratch memory (control
 * block, carry records, tile-boundary rows, the fp32 iterate of bf16 storage;
 * the dense cell's factors and chunk products) is a static device array of
 * PARARNN_NOALLOC_SCRATCH_BYTES inside the library, one copy per GPU the
 * library runs on, held until the process ends.  The call allocates and frees
 * nothing; what must start at zero is cleared by a kernel on the stream at the
 * start of every call.  A problem whose workspace does not fit the array
 * returns PARARNN_WORKSPACE_TOO_SMALL and enqueues nothing (a solve to a
 * tolerance first gives up the carry-record slots of its multi-iteration first
 * launch and runs one launch per iteration; pararnn_workspace_bytes(.., 0) with
 * pararnn_set_fused(0) is the smallest size that still fits).  All calls on one
 * GPU share that GPU's array: calls that overlap on one GPU (two streams, two
 * threads) race, exactly as two pararnn_forward calls that share a workspace.
 */
#define PARARNN_NOALLOC_SCRATCH_BYTES (32u << 20)
int pararnn_forward_noalloc(int cell, int dtype, const float *params, const void *u, const void *h0,
                            int B, int L, int H, float tol, int max_iter, void *h, int *iters,
                            float *delta_trace, void *hip_stream);

/*
 * Backward: the adjoint recurrence of Eq. (6) at the forward result h,
 *   lam_L = g_L,  lam_{l-1} = J_l^T lam_l + g_{l-1},  J_l = df/dh at (h_{l-1}, u_l),
 * evaluated as one reverse prefix scan, plus the step-local gradients
 *   dL_du_l = (df/du_l)^T lam_l,  dL_dparams = sum_{b,l} (df/dparams)^T lam_l,
 *   dL_dh0 = J_1^T lam_1.
 *
 *   h               the converged forward output (same layout/dtype as forward's h)
 *   dL_dh           g, [B][L][S][H]; for the LSTM it covers both c and h
 *   dL_du           out [B][L][G][H]
 *   dL_dparams      out fp32, same shape as params; overwritten, not accumulated
 *   dL_dh0          out [B][S][H], or NULL
 *   workspace       DEVICE scratch of at least pararnn_workspace_bytes(.., 1)
 * Dense cell (H = 64, fp32): with mu_l = (1 - F_l^2) * lam_l the recurrence reads
 * mu_l = diag(1 - F_l^2) W^T mu_{l+1} + (1 - F_l^2) * g_l, which the forward scan
 * kernels run with W^T and the time axis reversed; dL_du = mu, dL_dparams =
 * dL/dW = sum_{b,l} mu_l h_{l-1}^T, dL_dh0 = W^T mu_1.
 * Same return convention as pararnn_forward.
 */
int pararnn_backward(int cell, int dtype, const float *params, const void *u, const void *h0,
                     const void *h, const void *dL_dh, int B, int L, int H, void *dL_du,
                     float *dL_dparams, void *dL_dh0, void *workspace, size_t workspace_bytes,
                     void *hip_stream);

/*
 * How far given states are from solving the stacked system of Sec. 2, Eq. (2),
 * in max-norm: the quantity App. A's convergence figure plots per Newton
 * iteration,
 *     max over b, l, state value, channel of | h_l - f(h_{l-1}, u_l) |,  h_0 = h0.
 * Evaluate it on the iterates of fixed-count solves (tol < 0, max_iter = k) to
 * obtain that curve; pararnn_forward's own stopping test uses the size of the
 * update instead.
 *   params, u, h0  as for pararnn_forward (h0 may be NULL = zeros)
 *   h              device [B][L][S][H], the states to test, in the storage type
 *   out            device float[1]; overwritten.  A NaN among the inputs gives NaN.
 * One pass over u and h (each read once), no workspace, asynchronous on the
 * stream, nothing allocated.  Returns PARARNN_OK or a host-detected error as
 * pararnn_forward does; the dense cell has pararnn_forward's restrictions
 * (fp32, H = 64, 16-byte aligned pointers, else PARARNN_UNSUPPORTED).
 */
int pararnn_residual_norm(int cell, int dtype, const float *params, const void *u, const void *h0,
                          const void *h, int B, int L, int H, float *out, void *hip_stream);

/*
 * The linear solve on its own (the operation Alg. 1b performs), for testing
 * and profiling the scan without a cell: delta_l = J_l delta_{l-1} + r_l,
 * delta_0 = 0 (reverse = 0), or the adjoint
 * lam_l = J_{l+1}^T lam_{l+1} + r_l, lam_{L+1} = 0 (reverse = 1).
 *   kind   0: diagonal, J [B][L][H];  1, 2, 3: blocks of S x S with S = 2, 3, 4
 *          (the block-diagonal Jacobians of Sec. 3 for cells with S state
 *          values per channel), J [B][L][S][S][H] with J[p][q] =
 *          d(out_p)/d(in_q);  r, delta [B][L][S][H], fp32
 *   workspace of at least pararnn_affine_scan_workspace_bytes(kind, reverse, ..)
 */
size_t pararnn_affine_scan_workspace_bytes(int kind, int reverse, int B, int L, int H);
int pararnn_affine_scan(int kind, int reverse, const float *J, const float *r, int B, int L, int H,
                        float *delta, void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * The input projection in front of the recurrence and its derivatives, on the
 * matrix cores.  Sec. 3, Eq. (7a) / (7b): every gate reads the input through
 * B_g x_l + b_g; App. C: with n_heads heads the channels are split into n_heads
 * groups of dh = H / n_heads and B_g is block diagonal, head k's dh outputs
 * reading only head k's dh inputs (n_heads = 1: a full H x H matrix).
 *
 *   forward:   u[b][l][g][h] = sum_j Wx[g][h][j] * x[b][l][head(h)*dh + j] + bias[g][h]
 *   backward:  dx[b][l][k*dh + j] = sum_g sum_i du[b][l][g][k*dh + i] * Wx[g][k*dh + i][j]
 *              dWx[g][h][j]       = sum_{b,l} du[b][l][g][h] * x[b][l][head(h)*dh + j]
 *              dbias[g][h]        = sum_{b,l} du[b][l][g][h]
 *
 * x, dx [B][L][H]; u, du [B][L][G][H] (the layout pararnn_forward reads and
 * pararnn_backward writes), all of type dtype; Wx, dWx fp32 [G][H][dh]; bias,
 * dbias fp32 [G][H].  bias may be NULL (no bias); in the backward call dx, dWx
 * and dbias may each be NULL (not wanted), dbias only together with dWx.
 * Arithmetic: operands rounded to bf16, products accumulated in fp32 (the
 * paper's mixed-precision set-up); dWx / dbias partial sums are added in a fixed
 * order, so results are bit-reproducible.  Device pointers, 16-byte aligned
 * (else UNSUPPORTED); dh must be a multiple of 64 (else UNSUPPORTED), G <= 8.
 * workspace: pararnn_input_projection_workspace_bytes() bytes (0 for invalid
 * arguments), 256-byte aligned, needs no initialisation, may be shared with the
 * other calls on the same stream.  Kernels are enqueued on hip_stream; nothing
 * is allocated or synchronised.  Status codes as above.
 */
size_t pararnn_input_projection_workspace_bytes(int dtype, int B, int L, int H, int G, int n_heads, int backward);
int pararnn_input_projection(int dtype, const void *x, const float *Wx, const float *bias, int B, int L, int H,
                             int G, int n_heads, void *u, void *workspace, size_t workspace_bytes,
                             void *hip_stream);
int pararnn_input_projection_backward(int dtype, const void *x, const float *Wx, const void *du, int B, int L,
                                      int H, int G, int n_heads, void *dx, float *dWx, float *dbias,
                                      void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * The composition kernel of the dense scan on its own (testing / profiling):
 * the products of Jacobians J_l = diag(d_l) W that Alg. 1b's update of A
 * performs, taken over chunks of pararnn_dense_chunk() consecutive timesteps,
 *     A[b][c] = J_e ... J_{s+1} J_s,   s = c*chunk, e = min(L, s+chunk) - 1,
 * on the matrix cores.  W [H][H] row-major, d [B][L][H], A out
 * [B][ceil(L/chunk)][H][H] row-major; only the chunks c = 1 .. n_c-2 that the
 * scan uses are written.  fp32, H = 64 (else UNSUPPORTED).  workspace: 256
 * bytes of device memory, 256-byte aligned.  pararnn_dense_chunk() is the
 * number of timesteps per chunk.
 */
int pararnn_dense_chunk(void);
int pararnn_dense_chunk_products(const float *W, const float *d, int B, int L, int H, float *A,
                                 void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * Inexact-Newton switch of the dense path (host, process-wide; default 0).
 * The Jacobian products of the scan are what makes dense Jacobians expensive
 * (Sec. 2.1: cubic in the state size); mode selects their arithmetic in
 * FORWARD solves (pararnn_forward, pararnn_dense_chunk_products):
 *   0  fp32 on the matrix cores: Newton's method proper;
 *   1  every operand split into two bf16 terms, three bf16 products per fp32
 *      product (relative error about 2^-16 per product);
 *   2  one bf16 product (about 2^-8).
 * In modes 1 and 2 the linear solve of an iteration is approximate while the
 * residual stays fp32, so a solve to a tolerance converges to the same states
 * (same stopping test) and may take more iterations; with tol < 0 the iterate
 * after max_iter iterations differs from Newton's.  pararnn_backward is one
 * linear solve, not an iteration, and always uses fp32 products.
 * Returns PARARNN_INVALID_ARG for any other mode.
 */
int pararnn_set_dense_products(int mode);

/*
 * Quasi-Newton switch of the dense path (host, process-wide; default 0): the
 * variant of prior work that Sec. 1 and Sec. 2.1 describe, in which the
 * Jacobian of the linear solve is replaced by its diagonal.
 *   0  the full Jacobian J_l = diag(1 - F_l^2) W: Newton's method;
 *   1  its diagonal (1 - F_l^2) * W_ii: the linear solve of an iteration is a
 *      diagonal scan over the H channels, no matrix products at all.  The
 *      residual is still the exact one, so the iteration has the same fixed
 *      point (the recurrence's states) and the same stopping test; it
 *      converges linearly instead of quadratically, i.e. it needs more (and
 *      much cheaper) iterations, and when it stops the error of h is of the
 *      order of tol rather than far below it.  Iteration k makes timestep
 *      k + 1 exact, so at most L - 1 iterations are needed in any case.
 * Affects pararnn_forward of PARARNN_TANH_DENSE only; pararnn_set_dense_products
 * is irrelevant in mode 1; pararnn_backward always solves with the full
 * transposed Jacobian.  Returns PARARNN_INVALID_ARG for any other mode.
 */
int pararnn_set_dense_jacobian(int mode);

/*
 * Launch structure of the dense path's forward solves (host, process-wide, not
 * thread-safe; default 1).  An iteration has four phases (residual; chunk
 * products and chunk-local sweeps; carry; final sweep).
 *   1  the first six iterations are enqueued as one launch per phase; whatever is
 *      left of max_iter runs in ONE persistent launch whose phases are separated
 *      by grid-wide barriers and which returns at once when the solve has already
 *      ended.  A solve that converges early (the usual case: Newton needs 3-5
 *      iterations) costs one idle launch instead of four per iteration up to
 *      max_iter;
 *   0  one launch per phase for every iteration up to max_iter (those after
 *      convergence return at once);
 *   2  the persistent launch from the first iteration (slower per iteration:
 *      every phase then runs at the occupancy of the largest one).
 * Same arithmetic in all three: bit-identical results.  Other values give
 * PARARNN_INVALID_ARG.
 */
int pararnn_set_dense_tail(int mode);

#ifdef __cplusplus
}
#endif
#endif /* PARARNN_H */
