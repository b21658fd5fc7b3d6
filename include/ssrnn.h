/* ssrnn -- single-stream, multi-time-step inference of stacked SRU and QRNN
 * layers on one MI355X (gfx950).  C ABI of libssrnn.so.
 *
 * Method: arXiv 1803.11389.  A block of T consecutive time steps is processed
 * per pass over a layer's weights (Section 3, Eq. 4): the gate pre-activations
 * of the T steps are one skinny matrix product U = W * X, X = [x_0 ... x_{T-1}],
 * so that each weight fetched from memory is used T times; the element-wise
 * recurrence of Eq. 2 (SRU) / Eq. 3 (QRNN) then ripples over the T steps.
 * Every layer's weights are read once per block.  A (block, layer) pair is a
 * stage; stage (b, l) depends on (b, l-1) for its input and on (b-1, l) for its
 * state, so the stages with equal b + l are independent.  By default a call
 * that holds more than one block runs those together, one launch per value of
 * b + l (the wavefront schedule: block b+1 enters the first layer while block b
 * is in the second); a call of one block, or SSRNN_SCHED_STAGES, takes the
 * stages one by one in streaming order (block b through every layer before
 * block b+1 starts).  The two schedules give the same results up to fp32
 * re-association, and the same bits where one kernel instance with one launch
 * geometry serves both (the geometry may depend on how many stages a launch
 * holds: see the SSRNN_OPT_* flags).
 *
 * Conventions
 *   - Every pointer is a DEVICE pointer unless it says "host".  W[] and bias[]
 *     are HOST arrays (n_layers entries) of device pointers.
 *   - The caller owns every buffer.  *_forward never allocates or frees device
 *     memory and never synchronises with the host: all work is queued on
 *     `stream` (a hipStream_t passed as void*; NULL = the default stream).
 *     Buffers must stay valid until that work has finished.  The work is
 *     kernel launches only, so a call on a capturing stream records into a HIP
 *     graph.
 *   - x, h: time-major [L x d] fp32, row t = time step t.  State c: fp32.
 *   - Weights: row-major, fp32 (SSRNN_F32), bfloat16 bit patterns (SSRNN_BF16)
 *     or 8-bit floats with one fp32 scale per row (SSRNN_FP8, see
 *     ssrnn_weight_bytes); products accumulate in fp32, state stays fp32.  The
 *     paper's point is that the bytes of weights fetched per time step decide
 *     the speed (Sections 1 and 3); narrower weights cut those bytes the same
 *     way a larger T does, and the two multiply.
 *   - Return value: an ssrnn_status.  On failure nothing (EINVAL, EUNSUPPORTED,
 *     EWORKSPACE) or an unspecified part (EDEVICE) of the work was queued, and
 *     ssrnn_last_error() describes the cause.  No exception crosses the ABI.
 *   - L == 0 is valid: c_final (and xhist_final) receive the initial state.
 *     T > L is valid (one short block); L need not be a multiple of T.
 *   - Results do not depend on T, nor on `flags`, beyond fp32 re-association.
 */
#ifndef SSRNN_H
#define SSRNN_H

#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  SSRNN_OK = 0,
  SSRNN_EINVAL = 1,       /* NULL required pointer, size out of range              */
  SSRNN_EUNSUPPORTED = 2, /* shape or option no kernel here can take               */
  SSRNN_EWORKSPACE = 3,   /* workspace NULL, misaligned or too small               */
  SSRNN_EDEVICE = 4       /* a HIP call failed                                     */
} ssrnn_status;

typedef enum { SSRNN_F32 = 0, SSRNN_BF16 = 1, SSRNN_FP8 = 2 } ssrnn_wdtype;

/* `flags` of *_forward: 0 picks the schedule and kernel by shape.  The other
 * values force one (tests and measurements use them); a forced choice that the
 * shape does not allow returns SSRNN_EUNSUPPORTED. */
enum {
  SSRNN_SCHED_AUTO = 0,
  SSRNN_SCHED_STAGES = 1,     /* one kernel launch per (block, layer) stage, streaming order */
  SSRNN_SCHED_WAVEFRONT = 3,  /* one launch per anti-diagonal b + l of the (block, layer)
                                 grid: up to n_layers independent stages side by side       */
  SSRNN_SCHED_MASK = 3,
  SSRNN_KERNEL_AUTO = 0,
  SSRNN_KERNEL_GENERIC = 1 << 4, /* any d, k, T: one wavefront per output feature            */
  SSRNN_KERNEL_VALU = 2 << 4,    /* bandwidth kernel, FMA on the vector ALU (short blocks)   */
  SSRNN_KERNEL_MFMA = 3 << 4,    /* matrix-core kernel                                       */
  SSRNN_KERNEL_MASK = 7 << 4,
  SSRNN_WEIGHTS_PACKED = 1 << 8, /* every W[l] was written by ssrnn_pack_weights                */
  /* Per-call limits on the launch geometry (tests and measurements; results change by fp32
     re-association at most).  By default the matrix-core kernels adapt to the number of
     stages a launch holds: a narrow layer's columns are split over several workgroups when
     the launch would not fill the chip otherwise, and a workgroup owns 32 or 64 features
     instead of 16 when the launch is wide enough. */
  SSRNN_OPT_NO_SPLIT = 1 << 9,   /* never split a layer's columns over workgroups               */
  SSRNN_OPT_ONE_TILE = 1 << 10,  /* always 16 features per workgroup                            */
  SSRNN_OPT_MASK = 3 << 9,
  /* Direction (Section 2.1: a bidirectional network is two independent passes, one in each
     direction; joining their outputs is the caller's).  Every layer walks the sequence from
     its last step to its first: c_{t+1} takes the place of c_{t-1}, the QRNN window of step t
     holds x_t, x_{t+1}, ..., c_init is the state before time L-1 is taken in, c_final the state
     after time 0, xhist_init entry (l, j) layer l's input j+1 steps beyond time L-1, xhist_final
     its inputs at times j.  x and h stay indexed by time.  The result equals the forward pass
     over the time-reversed x, read backwards. */
  SSRNN_REVERSE = 1 << 11
};

/* Library version, major*10000 + minor*100 + patch.  Host; never fails. */
int ssrnn_version(void);

/* Description of the last failure on the calling thread (host, static storage,
 * valid until the next failing call on that thread); "" if none. */
const char* ssrnn_last_error(void);

/* Bytes of device scratch *_forward needs for this shape (inter-layer
 * activations for two blocks in flight, their operand copies for the
 * matrix-core kernels, partial sums of split stages).  Host.  Returns 0 for arguments *_forward would
 * reject.  The workspace must be 256-byte aligned; its contents need not be
 * initialised and are not preserved.  Calls that share a workspace must not
 * overlap in time (queue them on one stream, or order the streams). */
size_t ssrnn_workspace_bytes(int n_layers, int d, int k, int T, int wdtype);

/* Bytes of one layer's weight buffer W[l] for a [3d x k*d] matrix.  Host; 0 for
 * sizes out of range.  SSRNN_F32: 12*d*k*d.  SSRNN_BF16: 6*d*k*d.  SSRNN_FP8:
 * the 3*d*k*d OCP FP8 E4M3 codes (1 sign, 4 exponent bits with bias 7, 3
 * mantissa bits, subnormals, no infinities, largest finite value 448),
 * row-major, zero padding up to the next multiple of 256 bytes, then 3*d fp32
 * scales, one per matrix row: W[row][col] = scale[row] * value(code[row][col]).
 * NaN codes (0x7F, 0xFF) are the caller's to avoid.  The kernels widen the
 * codes exactly (to fp32 on the vector ALU, to bf16 on the matrix cores) and
 * apply the scale to the finished fp32 sum of a row. */
size_t ssrnn_weight_bytes(int d, int k, int wdtype);

/* Stacked SRU forward, Eq. 2 per layer, T steps per weight pass (Section 3).
 *   xh = W x_t;  f = sigma(W_f x_t + b_f);  r = sigma(W_r x_t + b_r);
 *   c_t = f*c_{t-1} + (1-f)*xh;  h_t = r*tanh(c_t) + (1-r)*x_t.
 * W[l]     [3d x d] rows [0,d) = W, [d,2d) = W_f, [2d,3d) = W_r.
 * bias     NULL (all zero), or host array whose entry l is NULL or [2d] = b_f | b_r.
 * x        [L x d] input of layer 0.
 * c_init   [n_layers x d], or NULL for zeros.
 * h        out [L x d]: the top layer's output.
 * c_final  out [n_layers x d]: state after the last step; may alias c_init.
 * d >= 1, n_layers >= 1, L >= 0, T >= 1. */
int sru_forward(const void* const* W, const float* const* bias, const float* x,
                const float* c_init, float* h, float* c_final, int n_layers,
                int d, long L, int T, int wdtype, int flags, void* workspace,
                size_t workspace_bytes, void* stream);

/* sru_forward for callers that cannot allocate device memory and so have no
 * workspace to pass: code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc.  Same arguments, kernels and results as
 * sru_forward; the scratch is
 * a static array of SSRNN_NOALLOC_SCRATCH_BYTES in device memory that is part
 * of the library's code object: every GPU the library runs on holds its own copy
 * from the first call there until the process ends.  The call allocates and
 * frees nothing.  The first call on a device looks the array's address up
 * (make it outside any stream capture); later calls only launch kernels.
 * A shape whose ssrnn_workspace_bytes(n_layers, d, 1, min(T, L), wdtype)
 * exceeds SSRNN_NOALLOC_SCRATCH_BYTES fails with SSRNN_EWORKSPACE before any
 * work is queued.  All calls on one GPU share that GPU's array, whatever their
 * stream or thread: calls that overlap in time there race; queue them on one
 * stream or order the streams.  Nothing in the array needs to start at zero
 * and nothing is kept in it between calls. */
#define SSRNN_NOALLOC_SCRATCH_BYTES (32u << 20)
int sru_forward_noalloc(const void* const* W, const float* const* bias,
                        const float* x, const float* c_init, float* h,
                        float* c_final, int n_layers, int d, long L, int T,
                        int wdtype, int flags, void* stream);

/* Stacked QRNN forward with fo-pooling, Eq. 3 per layer generalised from the
 * printed window of 2 to a causal window of k inputs:
 *   u_g = sum_{j<k} W_g^j x_{t-j} (+ b_g);  xh = tanh(u_0); f = sigma(u_1); o = sigma(u_2);
 *   c_t = f*c_{t-1} + (1-f)*xh;  h_t = o*tanh(c_t).
 * W[l]        [3d x k*d]; columns [j*d,(j+1)*d) multiply x_{t-j}; rows xh | f | o.
 * bias        NULL, or host array whose entry l is NULL or [3d] (Eq. 3 has none).
 * xhist_init  [n_layers x (k-1) x d]: entry (l, j) is layer l's input at lag
 *             j+1 before step 0; NULL for zeros (causal zero padding).
 * xhist_final out, same shape, or NULL: the last k-1 inputs of every layer.
 *             May alias xhist_init.  Ignored when k == 1.
 * Other arguments as for sru_forward.  k >= 1. */
int qrnn_forward(const void* const* W, const float* const* bias, const float* x,
                 const float* c_init, const float* xhist_init, float* h,
                 float* c_final, float* xhist_final, int n_layers, int d,
                 long L, int T, int k, int wdtype, int flags, void* workspace,
                 size_t workspace_bytes, void* stream);

/* Stacked LSTM forward, Eq. 1 per layer: the network the paper compares SRU and
 * QRNN with, run as its Section 3.1 describes.
 *   f = sigma(W_f x_t + U_f h_{t-1} + b_f);  i, o likewise;
 *   chat = tanh(W_c x_t + U_c h_{t-1} + b_c);
 *   c_t = f*c_{t-1} + i*chat;  h_t = o*tanh(c_t).
 * The products with the input are formed for min(T, 16) steps in one pass over
 * W; the products with h_{t-1} take one pass over U per time step, whatever T
 * is -- which is the paper's point: blocking can at best halve an LSTM's weight
 * traffic.  fp32 only.
 * W[l], U[l] [4d x d] row-major, rows [0,d) = f, [d,2d) = i, [2d,3d) = o,
 *            [3d,4d) = chat (the order of Eq. 1).
 * bias       NULL (all zero), or host array whose entry l is NULL or [4d].
 * x          [L x d] input of layer 0;  h  out [L x d], the top layer's output
 *            (must not overlap x).
 * h_init, c_init  [n_layers x d], or NULL for zeros.
 * h_final, c_final  out [n_layers x d]: every layer's h and c after the last
 *            step; may alias h_init / c_init.
 * flags      0.  workspace: lstm_workspace_bytes(n_layers, d, T) bytes, 256-byte
 *            aligned, contents neither expected nor preserved.
 * d >= 1 (any width; rows that are a multiple of 4 values in 16-byte aligned
 * buffers take the fast path), n_layers >= 1, L >= 0, T >= 1.  Errors as for
 * sru_forward.  Asynchronous on `stream`; kernel launches only. */
size_t lstm_workspace_bytes(int n_layers, int d, int T);
int lstm_forward(const float* const* W, const float* const* U,
                 const float* const* bias, const float* x, const float* h_init,
                 const float* c_init, float* h, float* h_final, float* c_final,
                 int n_layers, int d, long L, int T, int flags, void* workspace,
                 size_t workspace_bytes, void* stream);

/* y[L x d_out] = feat[L x d_in] * P^T, P row-major [d_out x d_in]; no bias, no
 * activation.  The input projection of the ASR-shaped benchmark workload
 * (40-dim features -> d); not part of the paper's method. */
int ssrnn_linear_forward(const float* P, const float* feat, float* y, int d_out,
                         int d_in, long L, void* stream);

/* Weight pre-pack (model-load time, once per layer): re-tiles a row-major
 * [3d x k*d] matrix into the order the matrix-core kernel consumes it, so that
 * each of that kernel's load instructions reads one contiguous KiB of whole
 * cache lines.  It is the row-blocking of Section 3 (fetch a piece of a row
 * once, use it for all T steps) applied to 16-row MFMA tiles.  The values are
 * only permuted (the row scales of SSRNN_FP8 stay where they are, behind the
 * matrix).  ssrnn_packed_weight_bytes: host; bytes of the packed buffer
 * (equal to ssrnn_weight_bytes), or 0 if the shape cannot be packed (needs
 * d % 16 == 0 and d*sizeof(weight) % 128 == 0).  ssrnn_pack_weights: W and
 * W_packed are distinct 16-byte aligned device buffers of that size; the copy
 * is enqueued on stream.  Pass the packed buffers as W[l] together with
 * SSRNN_WEIGHTS_PACKED in flags; shapes the matrix-core kernel cannot take
 * then fail with SSRNN_EUNSUPPORTED.  SSRNN_FP8 weights reach the matrix
 * cores in packed form only: row-major, they run on the vector ALU
 * (d % 1024 == 0; blocks longer than 8 steps are processed 8 steps per weight
 * pass) and on the generic kernel otherwise. */
size_t ssrnn_packed_weight_bytes(int d, int k, int wdtype);
int ssrnn_pack_weights(const void* W, void* W_packed, int d, int k, int wdtype,
                       void* stream);

#ifdef __cplusplus
}
#endif
#endif /* SSRNN_H */
