/*
 * mpcpipe - two-party semi-honest online phase of MPC-Pipe's secure layer on
 * one AMD MI355X (gfx950): Beaver-triple matmul / conv over the ring Z_2^64
 * with fixed-point truncation, and secure ReLU through A2B conversion.
 *
 * Both parties are simulated on one device.  Party i's work is enqueued on
 * party i's stream and touches only party i's buffers plus opened ("public")
 * values; the exchange of masked shares - the protocol's communication - is
 * a device-to-device copy on a third, "wire" stream ordered by events.
 *
 * General rules for every entry point
 *   - all tensor pointers are DEVICE pointers to dense row-major arrays of
 *     uint64_t ring elements unless a parameter says otherwise;
 *   - the caller owns every buffer it passes in, including the workspace; the
 *     library never allocates or frees device memory in these calls (the
 *     context owns only streams and events);
 *   - calls enqueue work and return; party i's outputs are ordered on party
 *     i's stream (mpc_ctx_sync waits for all three streams);
 *   - return value 0 = success, negative = error (see mpc_strerror); on an
 *     argument error nothing has been enqueued and no output is written;
 *   - build party 0 is the paper's "Party #1": the one whose share receives
 *     the Delta*epsilon term (Alg. 1; Alg. 4);
 *   - a context is one execution lane: two calls on the same context are
 *     serialised by its streams and share its workspace; use one context per
 *     micro-batch to overlap them (inter-batch pipeline, Sec. 4.3).
 */
#ifndef MPCPIPE_H
#define MPCPIPE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct mpc_ctx mpc_ctx;

/* One pointer per simulated party. */
typedef struct { const uint64_t* p[2]; } mpc_cshare;
typedef struct { uint64_t* p[2]; } mpc_share;

enum {
    MPC_OK = 0,
    MPC_EINVAL = -1,   /* null pointer, non-positive size, unsupported shape   */
    MPC_ENOMEM = -2,   /* workspace missing or smaller than mpc_*_workspace()  */
    MPC_EHIP = -3,     /* a HIP call failed; mpc_last_hip_error() has the code */
    MPC_ERANGE = -4    /* contraction too long for exact int32 digit sums, or
                          n beyond a fixed-size entry point's maximum          */
};

/* flags for mpc_beaver_matmul / mpc_conv2d and the gradient products */
enum {
    MPC_TRUNCATE = 1,     /* rescale the product by 2^-frac_bits (local truncation)       */
    MPC_TWO_PHASE = 2,    /* Alg. 3 ordering: [a_i]*f first, while e is still "in flight" */
    MPC_TRANS_X = 4,      /* mpc_beaver_matmul: x, a are stored [K][M] (left operand = their transpose)  */
    MPC_TRANS_Y = 8,      /* mpc_beaver_matmul: y, b, f_public are stored [N][K]                          */
    MPC_FOLDED = 16       /* mpc_*_prepared: c.p[0] is the folded addend c_0 - a_0*b_0 of mpc_*_fold      */
};

#define MPC_N_AND_TRIPLES 12
/* Longest contraction (K, or KH*KW*Cin padded to 16 per filter tap) one
 * workgroup sums exactly in int32 digit sums.  Longer contractions, up to
 * MPC_MAX_K_TOTAL, are cut into slices whose 64-bit partial products are added
 * by a finishing kernel (workspace grows accordingly); beyond that MPC_ERANGE. */
#define MPC_MAX_K 16368
#define MPC_MAX_K_TOTAL 4194304

/* ------------------------------------------------------------------ context */

/* A context ("lane") is used by one host thread at a time; different lanes
 * may be driven from different threads.  Calls only enqueue work: outputs are
 * valid after mpc_ctx_sync (or after waiting on the lane's streams), and no
 * buffer passed to a call may be freed or rewritten before that.
 *
 * Creates a lane on `device` with its own three non-blocking streams (default
 * priority).  frac_bits in [0, 62] is the fixed-point scale used by
 * MPC_TRUNCATE.  Host-side allocation only. */
int mpc_ctx_create(mpc_ctx** out, int device, int frac_bits);
/* The same lane with one in-order stream for both parties and the wire (what mpc_ctx_set_streams(s0, s0, s0)
 * turns a lane into).  The stream comes from a fixed set of four per device that the library creates once and
 * keeps until the process ends; a lane takes the least used of them and gives it back when it is destroyed.  The
 * runtime multiplexes streams onto a small number of hardware queues (four by default), and lanes that are meant
 * to overlap (Sec. 4.3: one lane per micro-batch; Alg. 3: chunks of a layer) were measured to lose half of their
 * overlap once the process had used more streams than that: with the fixed set the overlap does not depend on
 * what ran before.  A fifth concurrent single-queue lane shares a stream with another one: the two are then
 * ordered with each other (never a wrong result); mpc_ctx_capture_begin refuses such a lane (MPC_EINVAL), since a
 * graph recorded on a shared stream would also record what the other lane issues meanwhile. */
int mpc_ctx_create_single_queue(mpc_ctx** out, int device, int frac_bits);
int mpc_ctx_destroy(mpc_ctx* ctx);

/* Replace the lane's streams by caller-owned hipStream_t handles (e.g. from
 * torch.cuda.Stream); NULL keeps the current one. */
int mpc_ctx_set_streams(mpc_ctx* ctx, void* s_party0, void* s_party1, void* s_wire);
/* stream handle: which = 0, 1 (party) or 2 (wire) */
void* mpc_ctx_stream(mpc_ctx* ctx, int which);

/* Caller-allocated device scratch, 256-byte aligned.  Contents are undefined
 * between calls.  The lane must be idle when the workspace is replaced. */
int mpc_ctx_set_workspace(mpc_ctx* ctx, void* dev_ptr, size_t bytes);

/* Blocks the host until all three streams of the lane are idle. */
int mpc_ctx_sync(mpc_ctx* ctx);

/* Make party streams of `ctx` wait (device side) for everything enqueued so
 * far on the party streams of `after`; used to chain layers across lanes. */
int mpc_ctx_wait(mpc_ctx* ctx, mpc_ctx* after);

/* Optional timing for benchmarks.  While enabled, the lane brackets three
 * kinds of region with timing-enabled HIP events on the stream that executes
 * them: which = 0 the digit-plane GEMM kernel alone, 1 a whole secure linear
 * call (mask, exchange, recode, GEMM), 2 a whole secure ReLU call.
 * mpc_ctx_profile synchronises the lane, returns the summed duration and the
 * number of regions recorded since the last mpc_ctx_profile_reset. */
enum { MPC_PROF_GEMM_KERNEL = 0, MPC_PROF_LINEAR = 1, MPC_PROF_RELU = 2 };
int mpc_ctx_set_profiling(mpc_ctx* ctx, int enable);
int mpc_ctx_profile(mpc_ctx* ctx, int which, double* total_ms, int* count);
/* The individual region durations (host array ms_out of `capacity` doubles, in
 * recording order; *count = number recorded, which may exceed capacity). */
int mpc_ctx_profile_samples(mpc_ctx* ctx, int which, double* ms_out, int capacity, int* count);
int mpc_ctx_profile_reset(mpc_ctx* ctx);

/* Carry network of the whole-word secure ReLU (mpc_relu, mpc_maxpool2x2):
 * MPC_ADDER_KOGGE_STONE (default), or MPC_ADDER_TREE, the divide-and-conquer
 * prefix tree of the listing in Sec. 4.2 (level i joins blocks of 2^i bits:
 * the upper half of each 2^(i+1)-bit block is combined with the top bit of
 * its lower half, copied over the upper half by an integer multiply).  Same
 * rounds, triples (1 + 6 + 5 word ANDs) and exchanged words; the sign-bit
 * shares differ between the two, every output after the B2A opening does not.
 * mpc_relu_msb always evaluates the pruned Kogge-Stone chain. */
enum { MPC_ADDER_KOGGE_STONE = 0, MPC_ADDER_TREE = 1 };
int mpc_ctx_set_adder(mpc_ctx* ctx, int adder);

/* Graph capture.  On a lane whose three streams are one queue, the calls made
 * between mpc_ctx_capture_begin and mpc_ctx_capture_end are recorded into a HIP
 * graph instead of being executed; mpc_graph_launch enqueues one replay on the
 * given lane (any single-queue or three-stream lane of the same device).  A
 * replay reads and writes the very buffers (and workspace) the recorded calls
 * were given: keep them allocated and in place, refill the inputs, replay.
 * Run the sequence once eagerly first (kernel attributes, workspace size).
 * While a capture is open mpc_ctx_sync, mpc_ctx_set_workspace,
 * mpc_ctx_set_streams and profiling return MPC_EINVAL; profiling must be off.
 * The library records kernel launches only (no memset or copy nodes). */
typedef struct mpc_graph mpc_graph;
int mpc_ctx_capture_begin(mpc_ctx* ctx);
int mpc_ctx_capture_end(mpc_ctx* ctx, mpc_graph** out);
int mpc_graph_launch(mpc_graph* graph, mpc_ctx* ctx);
int mpc_graph_destroy(mpc_graph* graph);

/* How masked words are exchanged (the rounds of the secure ReLU, and the masked
 * operands of the Beaver products).
 * MPC_EXCHANGE_COPY (default): a copy kernel on the wire stream moves every
 *   party's send buffer into the other party's receive buffer after each round.
 * MPC_EXCHANGE_PUT: the kernel that forms the masked words also stores them
 *   into the peer's receive buffer (what a peer-to-peer store would be between
 *   two devices); the next round starts when that kernel has ended.  One launch
 *   per round instead of two and one traversal less per exchanged word.  Takes
 *   effect on lanes whose three streams are one queue; elsewhere the copy
 *   kernels are used.  Results are identical.  The three-party ReLU and
 *   max-pool calls honour it on every lane (they use one stream): each stage
 *   kernel stores its masked words into both peers' receive buffers. */
enum { MPC_EXCHANGE_COPY = 0, MPC_EXCHANGE_PUT = 1 };
int mpc_ctx_set_exchange(mpc_ctx* ctx, int mode);

int mpc_last_hip_error(const mpc_ctx* ctx);
const char* mpc_strerror(int code);

/* Bytes of workspace the calls below need for the given problem. */
size_t mpc_matmul_workspace_bytes(int M, int K, int N, int batch);
size_t mpc_conv2d_workspace_bytes(int B, int H, int W, int Cin, int Cout,
                                  int KH, int KW, int pad, int stride);
size_t mpc_relu_workspace_bytes(size_t n);
size_t mpc_maxpool_workspace_bytes(int B, int H, int W, int C);
size_t mpc_relu_msb_workspace_bytes(size_t n);
size_t mpc_maxpool_msb_workspace_bytes(int B, int H, int W, int C);

/* ------------------------------------------------------------------ opening */

/* Reconstruct an additive sharing (Sec. 3.1; Alg. 1's Delta = sum of the
 * broadcast differences): out[k] = s.p[0][k] + s.p[1][k] mod 2^64.  Each
 * party's share crosses the wire stream once; the sum is written by party
 * 0's stream.  Needs 16*n bytes of workspace. */
int mpc_open(mpc_ctx* ctx, mpc_cshare s, uint64_t* out_public, size_t n);

/* Share-wise difference out_i = x_i - a_i (shares are linear, Eq. 1); with x a
 * weight and a the B part of its layer's triple this is the masked weight
 * that Alg. 3 broadcasts one layer ahead: follow it with mpc_open
 * to obtain f_public. */
int mpc_sub(mpc_ctx* ctx, mpc_cshare x, mpc_cshare a, mpc_share out, size_t n);

/* out_i = x_i + y_i: the local sum of two sharings (residual connections,
 * shared biases; addition of secret-shared values needs no communication,
 * Sec. 3.1).  out may alias x or y. */
int mpc_add(mpc_ctx* ctx, mpc_cshare x, mpc_cshare y, mpc_share out, size_t n);

/* --------------------------------------------------- Beaver matmul (Alg. 1) */

/* z = x * y on additive shares with the triple (a, b, c), C = A*B:
 *   e = open(x - a), f = open(y - b)
 *   z_0 = c_0 + e*b_0 + a_0*f + e*f,   z_1 = c_1 + e*b_1 + a_1*f
 * x, a: [batch][M][K];  y, b: [batch][K][N];  c, z: [batch][M][N].
 * f_public: NULL, or a device array [batch][K][N] holding y - b already
 *   opened ahead of time (Alg. 3: the weight mask is input independent); y
 *   may then be {NULL, NULL}.
 * n_chunks >= 1 splits the opening of e by rows into that many pieces whose
 *   mask kernels and wire copies are issued back to back (Alg. 4's tiling
 *   applied to the linear layer's exchange); results do not depend on it.
 * flags: MPC_TRUNCATE, MPC_TWO_PHASE; MPC_TRANS_X / MPC_TRANS_Y read the left
 *   / right operand from transposed storage (x, a as [batch][K][M]; y, b,
 *   f_public as [batch][N][K]).  These give the two gradient products of a
 *   dense layer without moving data (Sec. 5.3: x^T * grad and grad * w^T):
 *   grad_w = matmul(x, grad) with M' = K, K' = M and MPC_TRANS_X;
 *   grad_x = matmul(grad, w) with K' = N, N' = K and MPC_TRANS_Y, where
 *   f_public may be the forward pass's opened w - b.
 * Errors: MPC_EINVAL (null / non-positive), MPC_ERANGE (K > MPC_MAX_K_TOTAL),
 *   MPC_ENOMEM (workspace < mpc_matmul_workspace_bytes). */
int mpc_beaver_matmul(mpc_ctx* ctx, mpc_cshare x, mpc_cshare y,
                      mpc_cshare a, mpc_cshare b, mpc_cshare c, mpc_share z,
                      int M, int K, int N, int batch,
                      const uint64_t* f_public, int n_chunks, int flags);

/* The same with Conv as the product (Eq. 3).  x, a: [B][H][W][Cin] (NHWC);
 * w, b: [KH][KW][Cin][Cout];  c, z: [B][Ho][Wo][Cout] with
 * Ho = (H + 2*pad - KH)/stride + 1.  Padding pads shares with zero words.
 * The im2col matrix is never materialised as ring words: the GEMM's tile
 * loader gathers filter taps from the NHWC digit planes. */
int mpc_conv2d(mpc_ctx* ctx, mpc_cshare x, mpc_cshare w,
               mpc_cshare a, mpc_cshare b, mpc_cshare c, mpc_share z,
               int B, int H, int W, int Cin, int Cout, int KH, int KW,
               int pad, int stride,
               const uint64_t* f_public, int n_chunks, int flags);

/* Tuning of the ring GEMM's tile choice, process-wide; results never depend on it.  A launch whose longest
 * contraction has at most max_steps K steps (32 terms each; default 16) and whose output has at least min_tiles
 * tiles of 64 x 64 (default 512) runs with 64 x 64 workgroup tiles of four half-width waves, two workgroups per
 * compute unit: short contractions spend most of a workgroup's life in pipeline fill and epilogue, which a second
 * resident wave per SIMD hides.  Launches whose parties contract different lengths (the folded calls) also take
 * that tile at any contraction length once the output has 768 such tiles.  max_steps = 0 switches the small tile off.  MPC_EINVAL for max_steps < 0 or
 * min_tiles < 1. */
int mpc_set_gemm_small_tile(int max_steps, int min_tiles);

/* Measurement aid for the roofline of the ring GEMM (no step of the protocol): the int8 matrix-core rate the
 * device sustains on register-resident operands, in the instruction order of the GEMM's K step, one workgroup of
 * four waves per compute unit, no memory traffic.  random_operands = 0: all-zero operands; 1: every operand
 * byte a uniform pseudo-random digit, which is what the digit planes of secret shares look like.  Runs
 * `launches` launches of `iters` K steps (72 MFMA instructions each per wave) back to back on the lane's first
 * stream, waits for them (the call blocks) and returns the rate in int8 operations per second (a
 * multiply-accumulate counts as two).  Needs 4 bytes of workspace per thread launched (compute units x 256 x 4
 * bytes; MPC_ENOMEM otherwise); MPC_EINVAL for iters outside [1, 2^20] or launches outside [1, 1024]. */
int mpc_mfma_rate(mpc_ctx* ctx, int random_operands, int iters, int launches, double* int8_ops_per_s);

/* Prepared layers.  The GEMM consumes digit planes; those of the operands that
 * do not depend on the input - the triple's [a_i] on the left, and on the right
 * the opened weight mask f = w - b (Alg. 3 sends it ahead of time), b_0 + f and
 * b_1 - can be recoded once, when the offline material and the weights are in
 * place, and kept resident: a call then only masks and exchanges x, recodes the
 * opened e and runs the GEMM.  Results are the same words as from
 * mpc_beaver_matmul / mpc_conv2d with f_public.
 *   mpc_*_prepared_bytes: sizes of the two caller-owned device buffers
 *     (right: three plane tensors; left: two); either pointer may be NULL.
 *   mpc_*_prepare: fill them.  right_planes needs b and f_public (with f_public = NULL only the
 *     slot of b_1 is filled: see the folded product of two activations below), left_planes
 *     needs a; pass NULL for the one not wanted.  Buffers 16-byte aligned.
 *     flags: MPC_TRANS_X / MPC_TRANS_Y as for mpc_beaver_matmul (storage of a / of b, f).
 *   mpc_beaver_matmul_prepared / mpc_conv2d_prepared: the online call.
 *     right_planes is required; left_planes may be NULL (then [a_i] is recoded
 *     in the call).  Other arguments, workspace and errors as for the plain calls.
 *   Folded triple (flag MPC_FOLDED on the online call; needs both plane buffers).  Alg. 1's
 *     z_0 = c_0 + e*b_0 + a_0*f + e*f equals (c_0 - a_0*b_0) + (a_0 + e)*(b_0 + f) in the ring, and
 *     a_0 + e = x_0 + e_1, party 0's own share plus the masked word it receives.  With the
 *     input-independent local product folded into the addend ahead of time (mpc_*_fold:
 *     c0_folded = c_0 - a_0*b_0, M x N words, all pointers party 0's), party 0 contracts one product
 *     online instead of two (party 1 keeps [e | a_1] x [b_1 ; f]): three ring products per call, the
 *     same output words.  The online call then takes c.p[0] = c0_folded; a.p[0] is still needed for
 *     the mask x_0 - a_0, a_0's planes in left_planes are not read.  Not with MPC_TWO_PHASE.
 *   Folded product of two activations (mpc_beaver_matmul_folded; Sec. 5.3's attention products Q*K^T and
 *     A*V, where y is a share like x and f = y - b opens in the call).  The triple is still input-independent:
 *     c.p[0] = c0_folded from mpc_matmul_fold, left_planes from mpc_matmul_prepare (a_1's planes are read),
 *     right_planes from mpc_matmul_prepare with f_public = NULL, which fills only the slot of b_1 (the two
 *     others are workspace-side in this call and are not read).  Online, party 0 contracts
 *     (x_0 + e_1) * (y_0 + f_1), since b_0 + f = y_0 + f_1, and party 1 [e | a_1] x [b_1 ; f]: three ring
 *     products, the same output words as mpc_beaver_matmul.  x, y, a, b: both parties' shares (all four
 *     needed for the masks); flags: MPC_TRUNCATE, MPC_TRANS_X, MPC_TRANS_Y (MPC_FOLDED is implied);
 *     MPC_EINVAL for a NULL plane buffer or share. */
int mpc_matmul_fold(mpc_ctx* ctx, const uint64_t* a0, const uint64_t* b0, const uint64_t* c0,
                    uint64_t* c0_folded, int M, int K, int N, int batch, int flags);
int mpc_conv2d_fold(mpc_ctx* ctx, const uint64_t* a0, const uint64_t* b0, const uint64_t* c0,
                    uint64_t* c0_folded, int B, int H, int W, int Cin, int Cout, int KH, int KW,
                    int pad, int stride);
int mpc_matmul_prepared_bytes(int M, int K, int N, int batch, size_t* right, size_t* left);
int mpc_conv2d_prepared_bytes(int B, int H, int W, int Cin, int Cout, int KH, int KW,
                              int pad, int stride, size_t* right, size_t* left);
int mpc_matmul_prepare(mpc_ctx* ctx, mpc_cshare a, mpc_cshare b, const uint64_t* f_public,
                       void* right_planes, void* left_planes,
                       int M, int K, int N, int batch, int flags);
int mpc_conv2d_prepare(mpc_ctx* ctx, mpc_cshare a, mpc_cshare b, const uint64_t* f_public,
                       void* right_planes, void* left_planes,
                       int B, int H, int W, int Cin, int Cout, int KH, int KW,
                       int pad, int stride);
int mpc_beaver_matmul_prepared(mpc_ctx* ctx, mpc_cshare x, mpc_cshare a, mpc_cshare c, mpc_share z,
                               const void* right_planes, const void* left_planes,
                               int M, int K, int N, int batch, int n_chunks, int flags);
int mpc_conv2d_prepared(mpc_ctx* ctx, mpc_cshare x, mpc_cshare a, mpc_cshare c, mpc_share z,
                        const void* right_planes, const void* left_planes,
                        int B, int H, int W, int Cin, int Cout, int KH, int KW,
                        int pad, int stride, int n_chunks, int flags);
int mpc_beaver_matmul_folded(mpc_ctx* ctx, mpc_cshare x, mpc_cshare y, mpc_cshare a, mpc_cshare b, mpc_cshare c,
                             mpc_share z, const void* right_planes, const void* left_planes,
                             int M, int K, int N, int batch, int n_chunks, int flags);

/* Backward pass of mpc_conv2d (Sec. 4.1 "Application to the backward pass",
 * Sec. 5.3): both gradients are Alg. 1 / Eq. 3 with another bilinear product
 * in place of Conv, on operands that are available before the backward pass
 * starts, so their masks can be opened ahead of time.
 *
 * mpc_conv2d_grad_x: gradient w.r.t. the input,
 *     gx[b][hi][wi][ci] = sum g[b][ho][wo][co] * w[kh][kw][ci][co]
 *   over all (ho, wo, kh, kw, co) with hi = ho*s + kh - pad, wi = wo*s + kw - pad.
 *   g, a: [B][Ho][Wo][Cout] (output gradient and its mask); w, b: the forward
 *   filter layout [KH][KW][Cin][Cout]; c, gx: [B][H][W][Cin].  f_public: NULL
 *   or w - b as opened for the forward pass (same layout as w).  KH == KW is
 *   required (else MPC_EINVAL).  Runs as a stride-1 convolution of g with the
 *   filter read in reverse tap order, padding KH - 1 - pad; for a strided
 *   layer g and its mask are first scattered into a zero-filled grid with
 *   stride-1 gaps (workspace grows by four such tensors).
 * mpc_conv2d_grad_w: gradient w.r.t. the filter,
 *     gw[kh][kw][ci][co] = sum_{b,ho,wo} x[b][ho*s+kh-pad][wo*s+kw-pad][ci] * g[b][ho][wo][co].
 *   x, a: [B][H][W][Cin] (the stored activation and the mask it was opened
 *   with); g, b: [B][Ho][Wo][Cout]; c, gw: [KH][KW][Cin][Cout].  e_public:
 *   NULL, or x - a as opened in the forward pass; x may then be {NULL, NULL}.
 *   The contraction runs over the B*Ho*Wo output pixels.
 * n_chunks, MPC_TRUNCATE as for mpc_conv2d; errors likewise. */
size_t mpc_conv2d_grad_x_workspace_bytes(int B, int H, int W, int Cin, int Cout,
                                         int KH, int KW, int pad, int stride);
size_t mpc_conv2d_grad_w_workspace_bytes(int B, int H, int W, int Cin, int Cout,
                                         int KH, int KW, int pad, int stride);
int mpc_conv2d_grad_x(mpc_ctx* ctx, mpc_cshare g, mpc_cshare w,
                      mpc_cshare a, mpc_cshare b, mpc_cshare c, mpc_share gx,
                      int B, int H, int W, int Cin, int Cout, int KH, int KW,
                      int pad, int stride,
                      const uint64_t* f_public, int n_chunks, int flags);
int mpc_conv2d_grad_w(mpc_ctx* ctx, mpc_cshare x, mpc_cshare g,
                      mpc_cshare a, mpc_cshare b, mpc_cshare c, mpc_share gw,
                      int B, int H, int W, int Cin, int Cout, int KH, int KW,
                      int pad, int stride,
                      const uint64_t* e_public, int n_chunks, int flags);

/* Element-wise Alg. 1 on n words: z = x * y with the triple (a, b, c),
 * c = a * b element by element; flags: 0 or MPC_TRUNCATE.  Workspace:
 * mpc_mul_workspace_bytes(n).
 * mpc_relu_backward: the backward pass of ReLU (Sec. 4.2, Sec. 5.3): output
 * gradient times the input mask 1 - s, where s_arith are the additive sign
 * shares mpc_relu / mpc_relu_msb returned in the forward pass; the mask shares
 * are [1 - s]_0 = 1 - [s]_0, [1 - s]_1 = -[s]_1, b masks them.  No rescale. */
size_t mpc_mul_workspace_bytes(size_t n);
int mpc_mul(mpc_ctx* ctx, mpc_cshare x, mpc_cshare y,
            mpc_cshare a, mpc_cshare b, mpc_cshare c, mpc_share z,
            size_t n, int flags);
int mpc_relu_backward(mpc_ctx* ctx, mpc_cshare g, mpc_cshare s_arith,
                      mpc_cshare a, mpc_cshare b, mpc_cshare c, mpc_share gx,
                      size_t n);

/* Local fixed-point rescale of a two-party sharing, in place (the paper only
 * requires fixed-point operands, Sec. 1.1; this is the usual local protocol):
 *   z_0 <- z_0 >> bits (logical),   z_1 <- -((-z_1) >> bits). */
int mpc_truncate(mpc_ctx* ctx, mpc_share z, size_t n, int bits);

/* --------------------------------------------- secure ReLU (Alg. 2, Sec. 4.2) */

/* Offline material for n elements, one pointer per party (device memory):
 *   r            n words      A2B masks: party i keeps x_i ^ r_i, sends r_i
 *   and_a/b/c    [12][n]      XOR-shared AND triples, triple-major; triple 0
 *                             for G = U & V, 1+2l / 2+2l for prefix level l
 *   rb, ra       n bytes / n words: XOR-shared random bit and additive shares
 *                             of the same bit (B2A of the sign)
 *   ma, mb, mc   n words      element-wise multiplication triple (select) */
typedef struct {
    mpc_cshare r;
    mpc_cshare and_a, and_b, and_c;
    const uint8_t* rb[2];
    mpc_cshare ra;
    mpc_cshare ma, mb, mc;
} mpc_relu_material;

/* y = ReLU(x) = x * (1 - MSB(x)) on additive shares:
 *   A2B distribution (Alg. 2) -> 64-bit Kogge-Stone carry network whose AND
 *   gates are Beaver ANDs (Eq. 4 / Alg. 4; 7 opening rounds, 12 word ANDs)
 *   -> sign share = bit 63 of the sum -> B2A with a shared random bit
 *   -> y = x * (1 - s) by element-wise Alg. 1 (no rescale).
 * n_chunks >= 1 tiles every round's exchange as in Alg. 4: all chunks' mask
 *   kernels and wire copies are issued back to back, then each chunk's gate
 *   evaluation waits only for its own copy.  On a lane whose three streams
 *   are one queue the chunks run one after the other through all rounds
 *   instead (same element ranges, same results).  n_chunks = 0 lets the
 *   library choose.  Results do not depend on it.
 * s_bit[i] (n bytes) / s_arith[i] (n words): optional per-party outputs of
 *   the sign's XOR share and additive share; NULL to skip. */
int mpc_relu(mpc_ctx* ctx, mpc_cshare x, const mpc_relu_material* mat, mpc_share y,
             size_t n, int n_chunks,
             uint8_t* const s_bit[2], uint64_t* const s_arith[2]);

/* Chunk size that n_chunks = 0 picks on this lane (results never depend on it): elements per chunk for mpc_relu /
 * mpc_maxpool2x2 and for the packed chain of mpc_relu_msb; 0 = the library's default (2^20 / 2^22).  A chunk's
 * exchanged words and carried state should still be in the last-level cache when the next round reads them; with
 * several lanes converting at once (Sec. 4.3: one lane per micro-batch) each lane has a share of that cache only, and
 * a runner gives its lanes the default divided by their number.  MPC_EINVAL below 1024 elements (other than 0). */
int mpc_ctx_set_relu_chunk(mpc_ctx* ctx, size_t whole_word_elems, size_t packed_elems);

/* mpc_relu for callers that cannot allocate device memory or own a workspace
 * (code under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc): same arguments, same shares, but the rounds' exchange buffers
 * and carried state live in a fixed array inside the library's code object
 * instead of the context's workspace.  The call performs no device or pinned
 * allocation and opens no timing region (mpc_ctx_profile never counts it).
 *   n <= mpc_relu_static_max_n() (65536), else MPC_ERANGE; the array takes
 *   about 14.4 MiB on every device the library runs on, until the process ends.
 *   The context must come from mpc_ctx_create or mpc_ctx_create_single_queue
 *   (which resolve the array's device address for the context's device), else
 *   MPC_EINVAL.
 *   All calls on one device share the array, which keeps the previous call's
 *   contents (every word read is first written by the same call, so nothing
 *   needs clearing): calls that overlap on a device, on any lane, race.
 *   Calls on one lane are ordered as usual. */
size_t mpc_relu_static_max_n(void);
int mpc_relu_static(mpc_ctx* ctx, mpc_cshare x, const mpc_relu_material* mat, mpc_share y,
                    size_t n, int n_chunks,
                    uint8_t* const s_bit[2], uint64_t* const s_arith[2]);

/* 2x2 / stride-2 max-pool on NHWC shares by max(p, q) = q + ReLU(p - q): two
 * tournament levels, i.e. two conversions per window (Sec. 4.2).  mat1 holds
 * material for 2*n_out elements (level 1: pairs (p00,p01), (p10,p11) per
 * output, interleaved), mat2 for n_out = B*(H/2)*(W/2)*C elements.  H, W even. */
int mpc_maxpool2x2(mpc_ctx* ctx, mpc_cshare x, const mpc_relu_material* mat1,
                   const mpc_relu_material* mat2, mpc_share y,
                   int B, int H, int W, int C, int n_chunks);

/* ------------------- secure ReLU on the sign's carry chain only (Sec. 4.2) */

/* The sign needs one output of the adder circuit of Sec. 4.2: the carry into
 * bit 63.  Of the Kogge-Stone network that mpc_relu evaluates on whole words,
 * prefix level l (shift 2^l) then contributes only the bit positions
 * p = 2^(l+1) - 2 (mod 2^(l+1)), p <= 62: 32, 16, 8, 4, 2, 1 positions for
 * l = 0..5.  mpc_relu_msb evaluates exactly those gates, with the same triple
 * bit at every gate as mpc_relu, so all outputs (y, s_bit, s_arith) are the
 * same words bit for bit; what changes is the layout: 2^(l+1) consecutive
 * elements share one word at level l, so the triples of a level, its masked
 * operands and its exchange are 2^(l+1) times smaller.
 *
 * Packed word j of level l holds elements j*2^(l+1) + k, k = 0..2^(l+1)-1,
 * as OR_k rotl(w_k & mask_l, k), mask_l = the positions above.
 *
 * Material: an mpc_relu_material whose and_a / and_b / and_c each point to
 * mpc_relu_packed_words(n) words (16-byte aligned) instead of [12][n]:
 *   triple 0 (G = U & V): n plain words, padded to a multiple of 4;
 *   triple t = 1..11 (level l = (t-1)/2): ceil64(n) / 2^(l+1) packed words,
 *   padded to a multiple of 4; segments follow one another in triple order.
 * mpc_relu_pack_triples converts one [12][n] array pair into this layout on
 * the device (an offline-phase helper: runs on the party streams, allocates
 * nothing).  All other material fields are as for mpc_relu.
 *
 * Opening rounds, chunking (chunk boundaries fall on multiples of 256
 * elements) and optional outputs are as for mpc_relu.  Errors: MPC_EINVAL for
 * null pointers, n == 0 or misaligned packed triples; MPC_ENOMEM if the
 * workspace is smaller than mpc_relu_msb_workspace_bytes(n). */
size_t mpc_relu_packed_words(size_t n);
int mpc_relu_pack_triples(mpc_ctx* ctx, mpc_cshare words, mpc_share packed, size_t n);
int mpc_relu_msb(mpc_ctx* ctx, mpc_cshare x, const mpc_relu_material* mat, mpc_share y,
                 size_t n, int n_chunks,
                 uint8_t* const s_bit[2], uint64_t* const s_arith[2]);

/* mpc_maxpool2x2 with both conversions on the pruned chain; mat1 / mat2 carry
 * packed triples for 2*n_out and n_out elements. */
int mpc_maxpool2x2_msb(mpc_ctx* ctx, mpc_cshare x, const mpc_relu_material* mat1,
                       const mpc_relu_material* mat2, mpc_share y,
                       int B, int H, int W, int C, int n_chunks);

/* Max-pool for training.  mpc_maxpool2x2_signs is mpc_maxpool2x2 (packed = 0)
 * or mpc_maxpool2x2_msb (packed != 0) that also returns the additive sign
 * shares of its two conversions: s1[i] 2*n_out words (pairs interleaved as in
 * mat1), s2[i] n_out words.  mpc_maxpool2x2_backward routes the output
 * gradient g [B][H/2][W/2][C] to the window maxima (Sec. 5.3: element-wise
 * products with the stored masks): with m = 1 - s,
 *   grad_u = g * m2, grad_v = g - grad_u                       (triple a2, b2, c2 on n_out words)
 *   grad_p00 = grad_u * m1, grad_p01 = grad_u - grad_p00, and the same for
 *   (grad_v; p10, p11)                                         (triple a1, b1, c1 on 2*n_out words)
 * gx: [B][H][W][C].  Workspace: mpc_maxpool_backward_workspace_bytes. */
int mpc_maxpool2x2_signs(mpc_ctx* ctx, mpc_cshare x, const mpc_relu_material* mat1,
                         const mpc_relu_material* mat2, mpc_share y,
                         uint64_t* const s1[2], uint64_t* const s2[2],
                         int B, int H, int W, int C, int n_chunks, int packed);
size_t mpc_maxpool_backward_workspace_bytes(int B, int H, int W, int C);
int mpc_maxpool2x2_backward(mpc_ctx* ctx, mpc_cshare g, mpc_cshare s1, mpc_cshare s2,
                            mpc_cshare a1, mpc_cshare b1, mpc_cshare c1,
                            mpc_cshare a2, mpc_cshare b2, mpc_cshare c2,
                            mpc_share gx, int B, int H, int W, int C);

/* ------------------------------------------ three parties (Sec. 3.3, Sec. 5.6) */

/* Alg. 1 and Alg. 2 are stated for N parties.  The calls below run them for
 * three simulated parties: an additive sharing is x = x_0 + x_1 + x_2, a
 * masked value is opened by summing what the three parties broadcast, and
 * party 0 (the paper's "Party #1") adds the Delta*epsilon term.  All work is
 * issued on the lane's first stream (the other two streams of the lane wait
 * for it on return), one launch per step for all parties, every exchange a
 * copy kernel; outputs are valid after any stream of the lane, or
 * mpc_ctx_sync.  Pointers are device memory, one per party; nothing is
 * allocated.  Errors as for the two-party calls. */
typedef struct { const uint64_t* p[3]; } mpc_cshare3;
typedef struct { uint64_t* p[3]; } mpc_share3;

/* out[k] = s_0[k] + s_1[k] + s_2[k].  Needs 24*n bytes of workspace. */
int mpc_open3(mpc_ctx* ctx, mpc_cshare3 s, uint64_t* out_public, size_t n);

/* Alg. 1 / Eq. 3 with three parties: z_i = c_i + e*b_i + a_i*f (+ e*f for
 * i = 0), e and f the sums of the three broadcast differences.  Shapes,
 * layouts and f_public as for mpc_beaver_matmul / mpc_conv2d; flags:
 * MPC_TRANS_X, MPC_TRANS_Y only (the rescale needs an exchange with three
 * parties: follow with mpc_truncate3).  Six ring products on the matrix
 * cores: parties 0 and 1 in one launch, party 2 in a second one. */
size_t mpc_matmul3_workspace_bytes(int M, int K, int N, int batch);
int mpc_beaver_matmul3(mpc_ctx* ctx, mpc_cshare3 x, mpc_cshare3 y,
                       mpc_cshare3 a, mpc_cshare3 b, mpc_cshare3 c, mpc_share3 z,
                       int M, int K, int N, int batch,
                       const uint64_t* f_public, int flags);
size_t mpc_conv2d3_workspace_bytes(int B, int H, int W, int Cin, int Cout,
                                   int KH, int KW, int pad, int stride);
int mpc_conv2d3(mpc_ctx* ctx, mpc_cshare3 x, mpc_cshare3 w,
                mpc_cshare3 a, mpc_cshare3 b, mpc_cshare3 c, mpc_share3 z,
                int B, int H, int W, int Cin, int Cout, int KH, int KW,
                int pad, int stride, const uint64_t* f_public);

/* Fixed-point rescale with three parties, in place.  Shifting every share
 * locally is sound for two parties only, and the paper states no rescale
 * (Sec. 1.1 names fixed point, nothing more); this is the usual masked one
 * with an offline pair: r uniform in [0, 2^63) shared as r, its shift
 * r >> bits shared as rt.  Parties 1 and 2 send z_i + r_i to party 0, which
 * forms m = z + r + 2^62 (no wrap for z in [-2^62, 2^62)) and
 *   z_0 <- (m >> bits) - 2^(62-bits) - rt_0,   z_i <- -rt_i  (i = 1, 2).
 * The result reconstructs to floor(z / 2^bits) + {0, 1}.  0 <= bits <= 62. */
size_t mpc_truncate3_workspace_bytes(size_t n);
int mpc_truncate3(mpc_ctx* ctx, mpc_share3 z, mpc_cshare3 r, mpc_cshare3 rt,
                  size_t n, int bits);

/* Offline material of the three-party ReLU for n elements:
 *   r0, r1       n words each  A2B masks: party j keeps x_j ^ r0_j ^ r1_j,
 *                              sends r0_j to party j+1 and r1_j to party j+2 (mod 3)
 *   and_a/b/c    [13][n]       XOR-shared AND triples: 0 the majority of the
 *                              carry-save step, 1 for G = S & K, 2+2l / 3+2l
 *                              for prefix level l
 *   rb, ra, ma, mb, mc         as in mpc_relu_material */
typedef struct {
    mpc_cshare3 r0, r1;
    mpc_cshare3 and_a, and_b, and_c;
    const uint8_t* rb[3];
    mpc_cshare3 ra;
    mpc_cshare3 ma, mb, mc;
} mpc_relu3_material;

/* y = ReLU(x) with three parties.  Alg. 2's last step has to add three
 * binary-shared words; the paper names no circuit for that, and the one used
 * is a carry-save step S = U ^ V ^ W, C = ((U ^ W) & (V ^ W)) ^ W (one Beaver
 * AND) followed by the Kogge-Stone network of mpc_relu on S and C << 1:
 * 13 word ANDs, 10 word exchanges and one byte exchange, each to both peers.
 * Sign, B2A and select as in mpc_relu.  s_bit / s_arith: optional outputs
 * (n bytes / n words per party), NULL to skip.  Whole-word chain, no chunking. */
size_t mpc_relu3_workspace_bytes(size_t n);
int mpc_relu3(mpc_ctx* ctx, mpc_cshare3 x, const mpc_relu3_material* mat, mpc_share3 y,
              size_t n, uint8_t* const s_bit[3], uint64_t* const s_arith[3]);

/* 2x2 / stride-2 max-pool with three parties by max(p, q) = q + ReLU(p - q),
 * as mpc_maxpool2x2: mat1 holds material for 2*n_out elements (pairs
 * interleaved), mat2 for n_out = B*(H/2)*(W/2)*C.  H, W even. */
size_t mpc_maxpool3_workspace_bytes(int B, int H, int W, int C);
int mpc_maxpool3(mpc_ctx* ctx, mpc_cshare3 x, const mpc_relu3_material* mat1,
                 const mpc_relu3_material* mat2, mpc_share3 y,
                 int B, int H, int W, int C);

/* The three-party ReLU on the sign's carry chain only (Sec. 4.2), as
 * mpc_relu_msb is to mpc_relu: the carry-save step and G = S & K stay on whole
 * words, the six prefix levels keep the positions bit 63 depends on, packed
 * 2^(l+1) elements to a word at level l (the layout mpc_relu_msb documents).
 * Every output (y, s_bit, s_arith) is the same word as mpc_relu3 returns for
 * the same material.  and_a / and_b / and_c of the material each point to
 * mpc_relu3_packed_words(n) words, 16-byte aligned:
 *   triples 0 and 1: n plain words each, padded to a multiple of 4;
 *   triple t = 2..12 (level l = (t-2)/2): ceil64(n) / 2^(l+1) packed words,
 *   padded to a multiple of 4; segments follow one another in triple order.
 * mpc_relu3_pack_triples converts one [13][n] array per party into this
 * layout on the device (offline helper, no workspace).  One pass, no chunks.
 * Errors: MPC_EINVAL for null or misaligned packed arrays, MPC_ENOMEM for a
 * workspace below mpc_relu3_msb_workspace_bytes(n). */
size_t mpc_relu3_packed_words(size_t n);
int mpc_relu3_pack_triples(mpc_ctx* ctx, mpc_cshare3 words, mpc_share3 packed, size_t n);
size_t mpc_relu3_msb_workspace_bytes(size_t n);
int mpc_relu3_msb(mpc_ctx* ctx, mpc_cshare3 x, const mpc_relu3_material* mat, mpc_share3 y,
                  size_t n, uint8_t* const s_bit[3], uint64_t* const s_arith[3]);
/* mpc_maxpool3 with both conversions on the packed chain (packed material). */
size_t mpc_maxpool3_msb_workspace_bytes(int B, int H, int W, int C);
int mpc_maxpool3_msb(mpc_ctx* ctx, mpc_cshare3 x, const mpc_relu3_material* mat1,
                     const mpc_relu3_material* mat2, mpc_share3 y,
                     int B, int H, int W, int C);

/* Prepared layers with three parties, as mpc_*_prepared for two: right_planes
 * holds the planes of f, b_0 + f, b_1, b_2 (needs b and the opened f_public),
 * left_planes those of a_0, a_1, a_2; sizes from mpc_*3_prepared_bytes, buffers
 * caller-owned and 16-byte aligned, either may be NULL in the prepare call;
 * the online calls need right_planes, left_planes may be NULL.  Same words as
 * mpc_beaver_matmul3 / mpc_conv2d3 with f_public; no rescale inside. */
int mpc_matmul3_prepared_bytes(int M, int K, int N, int batch, size_t* right, size_t* left);
int mpc_conv2d3_prepared_bytes(int B, int H, int W, int Cin, int Cout, int KH, int KW,
                               int pad, int stride, size_t* right, size_t* left);
int mpc_matmul3_prepare(mpc_ctx* ctx, mpc_cshare3 a, mpc_cshare3 b, const uint64_t* f_public,
                        void* right_planes, void* left_planes,
                        int M, int K, int N, int batch, int flags);
int mpc_conv2d3_prepare(mpc_ctx* ctx, mpc_cshare3 a, mpc_cshare3 b, const uint64_t* f_public,
                        void* right_planes, void* left_planes,
                        int B, int H, int W, int Cin, int Cout, int KH, int KW,
                        int pad, int stride);
int mpc_beaver_matmul3_prepared(mpc_ctx* ctx, mpc_cshare3 x, mpc_cshare3 a, mpc_cshare3 c, mpc_share3 z,
                                const void* right_planes, const void* left_planes,
                                int M, int K, int N, int batch, int flags);
int mpc_conv2d3_prepared(mpc_ctx* ctx, mpc_cshare3 x, mpc_cshare3 a, mpc_cshare3 c, mpc_share3 z,
                         const void* right_planes, const void* left_planes,
                         int B, int H, int W, int Cin, int Cout, int KH, int KW,
                         int pad, int stride);

/* Backward pass with three parties (Sec. 4.1 and Sec. 5.3 for N = 3): the
 * gradient products are Alg. 1 with another bilinear map, as for two parties.
 * Dense layers: mpc_beaver_matmul3 with MPC_TRANS_X / MPC_TRANS_Y.
 * mpc_conv2d3_grad_x: g, a [B][Ho][Wo][Cout]; w, b the forward filter layout
 * [KH][KW][Cin][Cout]; c and gx [B][H][W][Cin]; square filters, pad <= KH-1;
 * f_public: the opened w - b of the forward pass, or NULL.
 * mpc_conv2d3_grad_w: x, a [B][H][W][Cin]; g, b [B][Ho][Wo][Cout]; c and gw
 * [KH][KW][Cin][Cout].  No rescale inside (mpc_truncate3 follows).
 * Errors as for mpc_conv2d3. */
size_t mpc_conv2d3_grad_x_workspace_bytes(int B, int H, int W, int Cin, int Cout,
                                          int KH, int KW, int pad, int stride);
size_t mpc_conv2d3_grad_w_workspace_bytes(int B, int H, int W, int Cin, int Cout,
                                          int KH, int KW, int pad, int stride);
int mpc_conv2d3_grad_x(mpc_ctx* ctx, mpc_cshare3 g, mpc_cshare3 w,
                       mpc_cshare3 a, mpc_cshare3 b, mpc_cshare3 c, mpc_share3 gx,
                       int B, int H, int W, int Cin, int Cout, int KH, int KW,
                       int pad, int stride, const uint64_t* f_public);
int mpc_conv2d3_grad_w(mpc_ctx* ctx, mpc_cshare3 x, mpc_cshare3 g,
                       mpc_cshare3 a, mpc_cshare3 b, mpc_cshare3 c, mpc_share3 gw,
                       int B, int H, int W, int Cin, int Cout, int KH, int KW,
                       int pad, int stride);

/* Element-wise Alg. 1 on n words with three parties: z = x * y with the
 * triple (a, b, c), c = a * b element by element, no rescale.
 * mpc_relu3_backward: output gradient times the input mask 1 - s; s_arith are
 * the additive sign shares mpc_relu3 / mpc_relu3_msb returned, the mask
 * shares are [1 - s]_0 = 1 - [s]_0, [1 - s]_i = -[s]_i.
 * mpc_maxpool3_signs: mpc_maxpool3 (packed = 0) or mpc_maxpool3_msb that also
 * returns the sign shares of its two conversions (s1[i]: 2*n_out words, pairs
 * interleaved as in mat1; s2[i]: n_out words).  mpc_maxpool3_backward routes
 * the output gradient to the window maxima exactly as
 * mpc_maxpool2x2_backward does (triples a2, b2, c2 on n_out words, a1, b1, c1
 * on 2*n_out words).  Workspace: the matching *_workspace_bytes query. */
/* Local linear steps on three shares (Sec. 3.1: additions need no
 * communication): out_i = x_i + y_i / x_i - y_i; out may alias x or y. */
int mpc_add3(mpc_ctx* ctx, mpc_cshare3 x, mpc_cshare3 y, mpc_share3 out, size_t n);
int mpc_sub3(mpc_ctx* ctx, mpc_cshare3 x, mpc_cshare3 y, mpc_share3 out, size_t n);
size_t mpc_mul3_workspace_bytes(size_t n);
int mpc_mul3(mpc_ctx* ctx, mpc_cshare3 x, mpc_cshare3 y,
             mpc_cshare3 a, mpc_cshare3 b, mpc_cshare3 c, mpc_share3 z, size_t n);
int mpc_relu3_backward(mpc_ctx* ctx, mpc_cshare3 g, mpc_cshare3 s_arith,
                       mpc_cshare3 a, mpc_cshare3 b, mpc_cshare3 c, mpc_share3 gx,
                       size_t n);
int mpc_maxpool3_signs(mpc_ctx* ctx, mpc_cshare3 x, const mpc_relu3_material* mat1,
                       const mpc_relu3_material* mat2, mpc_share3 y,
                       uint64_t* const s1[3], uint64_t* const s2[3],
                       int B, int H, int W, int C, int packed);
size_t mpc_maxpool3_backward_workspace_bytes(int B, int H, int W, int C);
int mpc_maxpool3_backward(mpc_ctx* ctx, mpc_cshare3 g, mpc_cshare3 s1, mpc_cshare3 s2,
                          mpc_cshare3 a1, mpc_cshare3 b1, mpc_cshare3 c1,
                          mpc_cshare3 a2, mpc_cshare3 b2, mpc_cshare3 c2,
                          mpc_share3 gx, int B, int H, int W, int C);

/* -------------------------------------------------- dealer helper (offline) */

/* Plain ring product Z = L*R mod 2^64 on public device arrays, computed with
 * the same digit-plane MFMA kernel: lets a synthetic dealer form C = A*B for
 * a triple without leaving the device.  Not part of the online phase.
 * Runs on party 0's stream; workspace as for mpc_beaver_matmul. */
int mpc_ring_matmul(mpc_ctx* ctx, const uint64_t* L, const uint64_t* R, uint64_t* Z,
                    int M, int K, int N, int batch);
int mpc_ring_conv2d(mpc_ctx* ctx, const uint64_t* x, const uint64_t* w, uint64_t* z,
                    int B, int H, int W, int Cin, int Cout, int KH, int KW,
                    int pad, int stride);
/* The two gradient products of a convolution on public arrays (layouts as for
 * mpc_conv2d_grad_x / mpc_conv2d_grad_w): C = F(A, B) of their triples. */
int mpc_ring_conv2d_grad_x(mpc_ctx* ctx, const uint64_t* g, const uint64_t* w, uint64_t* gx,
                           int B, int H, int W, int Cin, int Cout, int KH, int KW,
                           int pad, int stride);
int mpc_ring_conv2d_grad_w(mpc_ctx* ctx, const uint64_t* x, const uint64_t* g, uint64_t* gw,
                           int B, int H, int W, int Cin, int Cout, int KH, int KW,
                           int pad, int stride);

#ifdef __cplusplus
}
#endif
#endif /* MPCPIPE_H */
