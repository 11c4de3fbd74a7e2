/*
 * rodimus.h -- C ABI of the MI355X (gfx950) library for the Rodimus DDTS
 * gated linear-attention recurrence.
 *
 * The operation (paper Sec. 3.1.3, state recurrence of the Rodimus block, with the
 * general gated transition of Sec. 3.1.1 in its factored form and the value-side
 * transition gate fixed to one), for every (batch, head) pair independently:
 *
 *     S_t = diag(exp(log_alpha_t)) S_{t-1} + k_t^T (beta_t .* v_t),    o_t = q_t S_t
 *
 * S is dk x dv.  log_alpha_t (1 x dk) is the log of the decay gate
 * alpha_t = exp(-g_t .* tau_t) of Sec. 3.1.2, i.e. log_alpha = -g .* tau <= 0.
 * beta_t (1 x dv) is the input gate on the value.  The key-side input gate
 * g_t^tau_t, the normalisation of k and the 1/sqrt(dk) on q are folded into k and
 * q by the caller (second form of the transition in Sec. 3.1.1); the library
 * applies no scaling.  The output uses the state AFTER the update.  The block's
 * feed-through term is added by the caller.
 *
 * General conventions
 *   - Every pointer is a DEVICE pointer owned by the caller.  The library never
 *     allocates or frees device memory, never synchronises and keeps no global
 *     state (one exception: rodimus_chunk_scan_fwd_noalloc and its built-in scratch
 *     buffer); all work is enqueued on `stream` (a hipStream_t, NULL = default).
 *   - Innermost index contiguous, no strides:
 *         q, k, log_alpha : [B, T, H, dk]     v, beta, o : [B, T, H, dv]
 *         S0, S_T, S      : [B, H, dk, dv]    (decode: B -> N, T dropped)
 *   - q, k, v, o have element type `io_dtype` (RODIMUS_F32 or RODIMUS_BF16,
 *     bf16 = upper 16 bits of an IEEE float, round-to-nearest-even on output).
 *     log_alpha, beta and every state are fp32; all accumulation is fp32.
 *   - Base pointers must be 16-byte aligned.
 *   - Every function validates its arguments on the host BEFORE any launch and
 *     returns a rodimus_status; nothing is written on error.  No exceptions,
 *     no aborts.
 *   - log_alpha = -inf (alpha = 0) is legal.  log_alpha > 0 is not rejected but
 *     products of gates may then overflow.
 */
#ifndef RODIMUS_H
#define RODIMUS_H

#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    RODIMUS_OK = 0,
    RODIMUS_ERR_NULL = 1,        /* a required pointer is NULL                           */
    RODIMUS_ERR_SHAPE = 2,       /* a size is negative/zero or out of the supported range */
    RODIMUS_ERR_DTYPE = 3,       /* io_dtype is not a rodimus_dtype                       */
    RODIMUS_ERR_ALIGN = 4,       /* a base pointer is not 16-byte aligned                 */
    RODIMUS_ERR_WORKSPACE = 5,   /* workspace missing or smaller than required            */
    RODIMUS_ERR_LAUNCH = 6,      /* the HIP runtime refused the launch                    */
    RODIMUS_ERR_ALIAS = 7,       /* an output overlaps an input it must not overlap       */
    RODIMUS_ERR_SCRATCH = 8      /* rodimus_chunk_scan_fwd_noalloc: the shape needs more than the built-in scratch */
} rodimus_status;

typedef enum { RODIMUS_F32 = 0, RODIMUS_BF16 = 1 } rodimus_dtype;

/* Which kernel family a chunk-scan call of this shape runs (for tests and reports). */
typedef enum {
    RODIMUS_PATH_NONE = 0,       /* shape not supported                                  */
    RODIMUS_PATH_GENERIC = 1,    /* fp32 ALU chunkwise kernel, any supported shape        */
    RODIMUS_PATH_MFMA = 2        /* bf16 MFMA chunkwise kernel (dk = 64, chunk = 64, ...) */
} rodimus_path;

/* Human-readable name of a status code (static storage, never NULL). */
const char *rodimus_status_string(int status);

/*
 * Chunkwise-parallel forward scan over T tokens (prefill / training forward).
 * Appendix "Chunkwise Parallel Representation of the Rodimus Block": inside each chunk the
 * masked, decayed scores (Q .* A)(K / A)^T and their product with beta .* V give the
 * intra-chunk output; the state entering the chunk gives the inter-chunk output; the
 * state is carried from chunk to chunk in fp32.  The result does not depend on `chunk`
 * beyond rounding.
 *
 *   q, k        [B,T,H,dk] io_dtype      in
 *   v           [B,T,H,dv] io_dtype      in
 *   log_alpha   [B,T,H,dk] fp32          in
 *   beta        [B,T,H,dv] fp32          in, or NULL = all ones
 *   S0          [B,H,dk,dv] fp32         in, or NULL = zero state
 *   o           [B,T,H,dv] io_dtype      out; must not overlap any input
 *   S_T         [B,H,dk,dv] fp32         out, or NULL if not wanted; MAY be the same buffer as S0
 *   chunk       1..64.  T need not be a multiple of it (the last chunk is shorter).
 *   workspace   device scratch of at least rodimus_chunk_scan_workspace_bytes(...) bytes,
 *               16-byte aligned; may be NULL when that size is 0.  Contents are undefined
 *               afterwards; concurrent calls need distinct workspaces.
 *
 * Supported shapes: 1 <= dk <= 128, dv >= 1, 1 <= chunk <= 64, chunk * dk <= 4096 (generic fp32-ALU path);
 * the MFMA path is taken for io_dtype = BF16, dk = 64, chunk = 64, dv % 128 == 0 (it carries the state every
 * 16 tokens internally and, when B * H * dv / 128 < 192, cuts the sequence into segments that run concurrently;
 * only then is a workspace needed).  B, T or H equal to 0 is a successful no-op (T = 0 copies S0 to S_T).
 */
int rodimus_chunk_scan_fwd(const void *q, const void *k, const void *v,
                           const float *log_alpha, const float *beta, const float *S0,
                           void *o, float *S_T,
                           int B, int T, int H, int dk, int dv, int chunk, int io_dtype,
                           void *workspace, size_t workspace_bytes, void *stream);

/* Scratch bytes the call above needs for this shape (0 if none, or if the shape is invalid). */
size_t rodimus_chunk_scan_workspace_bytes(int B, int T, int H, int dk, int dv, int chunk, int io_dtype);

/* Kernel family (rodimus_path) the call above would run for this shape. */
int rodimus_chunk_scan_path(int B, int T, int H, int dk, int dv, int chunk, int io_dtype);

/*
 * Measurement aid (no part of the paper's method): a plain streaming kernel, against which the bandwidth of the calls in
 * this header can be judged on the GPU at hand.  Writes `units` 16-byte units to dst; unit i is a constant plus the sum of
 * unit i of each of `reads_per_write` (0, 1, 2 or 4) input streams laid end to end in src (src holds reads_per_write *
 * units units; ignored and may be NULL for 0).  Coalesced, streaming accesses, `workgroups` workgroups of 256 lanes in a
 * grid-stride loop.  Device pointers, 16-byte aligned, dst must not overlap src.  No workspace, no synchronisation.
 * RODIMUS_ERR_SHAPE for another reads_per_write or workgroups outside 1 .. 2^20.
 */
int rodimus_hbm_stream_probe(const void *src, void *dst, size_t units, int reads_per_write, int workgroups, void *stream);

/*
 * rodimus_chunk_scan_fwd for callers that cannot allocate device memory: code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc.  Same arguments, same kernels and bit-identical results, but no
 * workspace argument: a call that is cut along the sequence keeps its segment summaries and entering states in a
 * buffer of RODIMUS_NOALLOC_SCRATCH_BYTES that is part of the library's device image (every GPU the library runs
 * on holds its own copy until the process ends).  The call allocates and frees nothing.
 *   - A shape whose workspace (rodimus_chunk_scan_workspace_bytes) exceeds the buffer returns RODIMUS_ERR_SCRATCH
 *     before anything is launched; so does a failure to locate the buffer on the current device.
 *   - Every call on a GPU shares that GPU's buffer, which keeps the last call's contents (nothing in it has to start
 *     at zero).  Calls that overlap in time on one GPU, on different streams, race on it: order them on one stream
 *     or with events.
 *   - The first call on each device looks the buffer's address up (hipGetSymbolAddress, once per device, under a
 *     lock); make that first call outside stream capture.
 */
#define RODIMUS_NOALLOC_SCRATCH_BYTES (10u << 20)
int rodimus_chunk_scan_fwd_noalloc(const void *q, const void *k, const void *v,
                                   const float *log_alpha, const float *beta, const float *S0,
                                   void *o, float *S_T,
                                   int B, int T, int H, int dk, int dv, int chunk, int io_dtype, void *stream);

/* Size of that built-in buffer (RODIMUS_NOALLOC_SCRATCH_BYTES of the library that is loaded). */
size_t rodimus_chunk_scan_fwd_noalloc_scratch_bytes(void);

/*
 * One recurrent decode step for N independent sequences (paper Sec. 3.1.3: at inference the
 * block keeps only the fixed-size state, O(1) work per token):
 *     S' = diag(exp(log_alpha)) S + k^T (beta .* v),   o = q S'
 *
 *   q, k        [N,H,dk] io_dtype        in
 *   v           [N,H,dv] io_dtype        in
 *   log_alpha   [N,H,dk] fp32            in
 *   beta        [N,H,dv] fp32            in, or NULL = all ones
 *   S           [N,H,dk,dv] fp32         in/out, updated IN PLACE to S'
 *   o           [N,H,dv] io_dtype        out
 *
 * Supported shapes: 1 <= dk <= 256, dv >= 4, dv % 4 == 0.  N or H equal to 0 is a no-op.
 */
int rodimus_decode_step(const void *q, const void *k, const void *v,
                        const float *log_alpha, const float *beta,
                        float *S, void *o,
                        int N, int H, int dk, int dv, int io_dtype, void *stream);

/*
 * DDTS gate front-end (paper Sec. 3.1.2 "Design of alpha, alpha-hat and beta-hat"; pre-processing of q and k in
 * Sec. 3.1.3): turns the pre-activations of the gates and the raw q, k into the arguments of the two calls above.
 * A row is one token of one head (rows = B*T*H for a scan, N*H for a decode step).
 *     g = softplus(z_g), tau = sigmoid(z_tau)
 *     log_alpha = -g .* tau                               (alpha = exp(-g .* tau))
 *     k_out     = g^tau .* k / max(||k||_2, 1e-12)        (alpha-hat folded into the L2-normalised key)
 *     q_out     = q / sqrt(dk)
 *     beta      = sigmoid(z_beta)
 *
 *   z_g, z_tau  [rows, dk] io_dtype      in
 *   z_beta      [rows, dv] io_dtype      in, or NULL (then beta must be NULL too and dv is ignored)
 *   q, k        [rows, dk] io_dtype      in
 *   log_alpha   [rows, dk] fp32          out
 *   beta        [rows, dv] fp32          out
 *   q_out,k_out [rows, dk] io_dtype      out; q_out may be the same buffer as q, k_out the same buffer as k;
 *                                        no other overlap between an output and any other argument is allowed
 *
 * Supported shapes: dk a power of two in 8..512, dv % 8 == 0.  rows = 0 is a no-op.
 */
int rodimus_ddts_gates(const void *z_g, const void *z_tau, const void *z_beta,
                       const void *q, const void *k,
                       float *log_alpha, float *beta, void *q_out, void *k_out,
                       long long rows, int dk, int dv, int io_dtype, void *stream);

/*
 * The two recurrence calls with the value gate fused in (paper Sec. 3.1.2: the input gate on the value side is
 * beta-hat = sigmoid of a projection of the token): identical to rodimus_chunk_scan_fwd / rodimus_decode_step in
 * every respect except that the gate arrives as its pre-activation
 *
 *   z_beta      [B,T,H,dv] (scan) / [N,H,dv] (decode step), io_dtype, in, required (NULL only for an empty call)
 *
 * and beta = sigmoid(z_beta) is evaluated inside the kernel in fp32.  With bf16 I/O this halves the bytes of the
 * largest input stream of the scan (1024 -> 512 per token-head at dv = 256) and makes the value half of
 * rodimus_ddts_gates unnecessary (call that with z_beta = NULL for the key side).  Same shapes, workspace, aliasing
 * rules, status codes and kernel families as the calls they mirror; -inf / +inf give the gate 0 / 1 exactly.
 */
int rodimus_chunk_scan_fwd_zbeta(const void *q, const void *k, const void *v,
                                 const float *log_alpha, const void *z_beta, const float *S0,
                                 void *o, float *S_T,
                                 int B, int T, int H, int dk, int dv, int chunk, int io_dtype,
                                 void *workspace, size_t workspace_bytes, void *stream);

int rodimus_decode_step_zbeta(const void *q, const void *k, const void *v,
                              const float *log_alpha, const void *z_beta,
                              float *S, void *o,
                              int N, int H, int dk, int dv, int io_dtype, void *stream);

/* How the value gate is passed to rodimus_chunk_scan_varlen_fwd. */
typedef enum {
    RODIMUS_BETA_VALUES = 0,          /* fp32 gate values (or NULL = all ones)              */
    RODIMUS_BETA_PREACTIVATION = 1    /* pre-activations in io_dtype, beta = sigmoid(.)     */
} rodimus_beta_kind;

/*
 * Chunkwise forward scan over a PACKED batch of N sequences of different lengths (serving prefill): the same
 * recurrence as rodimus_chunk_scan_fwd (paper Sec. 3.1.3 and the appendix on the chunkwise form), run independently on
 * every sequence; a sequence need not be a multiple of `chunk` long (the appendix assumes it is; a shorter last chunk
 * behaves as if padded with alpha = 1, q = k = v = 0).
 *
 *   q, k        [total_tokens,H,dk] io_dtype   in    sequence b owns the rows cu_seqlens[b] .. cu_seqlens[b+1]-1
 *   v           [total_tokens,H,dv] io_dtype   in
 *   log_alpha   [total_tokens,H,dk] fp32       in
 *   beta        [total_tokens,H,dv]            in    fp32 values or NULL (beta_kind = RODIMUS_BETA_VALUES), or
 *                                                    io_dtype pre-activations (RODIMUS_BETA_PREACTIVATION, required)
 *   S0          [N,H,dk,dv] fp32               in, or NULL = zero states
 *   o           [total_tokens,H,dv] io_dtype   out
 *   S_T         [N,H,dk,dv] fp32               out, or NULL; MAY be the same buffer as S0 (a state cache updated in
 *                                                    place); it is the state rodimus_decode_step continues from
 *   cu_seqlens  [N+1] int32, DEVICE memory     in    non-decreasing, cu_seqlens[0] = 0, cu_seqlens[N] = total_tokens.
 *                                                    The library cannot read it on the host: the kernels clamp every
 *                                                    entry to [0, total_tokens], so a corrupt table gives wrong
 *                                                    results but no access outside the tensors.  Empty sequences are
 *                                                    allowed (S_T = S0, no output rows).
 *
 * One workgroup set per (sequence, head): no workspace, no sequence split (a batch of few long sequences is better
 * served by rodimus_chunk_scan_varlen_fwd_cut).  With up to 64 sequences the workgroups take the sequences longest
 * first, whatever their order in the batch.  Shapes, kernel families, alignment (16 bytes, cu_seqlens included),
 * aliasing rules and status codes as for rodimus_chunk_scan_fwd; an unknown beta_kind gives RODIMUS_ERR_DTYPE.
 */
int rodimus_chunk_scan_varlen_fwd(const void *q, const void *k, const void *v,
                                  const float *log_alpha, const void *beta, int beta_kind, const float *S0,
                                  void *o, float *S_T,
                                  const int *cu_seqlens, int N, int total_tokens,
                                  int H, int dk, int dv, int chunk, int io_dtype, void *stream);

/*
 * rodimus_chunk_scan_varlen_fwd for a packed batch dominated by FEW LONG sequences (a handful of long prompts, or one
 * long prompt among short ones): one workgroup set per (sequence, head) lasts as long as the longest sequence and leaves
 * most of the chip idle meanwhile.  Here every sequence is cut into segments of a fixed length chosen from total_tokens
 * alone (the lengths stay on the device: every workgroup finds its sequence and segment from cu_seqlens), and the
 * segments run side by side: the state increment and decay of every segment (one pass over k, v and the gates), the
 * chain of entering states along each sequence, then the scan proper of every segment from its entering state -- the
 * split of the recurrence across chunks that the appendix on the chunkwise form states, applied at segment level.
 * Same results as rodimus_chunk_scan_varlen_fwd to rounding (the state passes through one more fp32 sum per segment).
 * The cut reads k, v and the gates of all but each sequence's last segment twice, so its duration depends on
 * total_tokens and hardly on the lengths; which call is faster is the caller's decision (it built cu_seqlens).  A
 * segment has total_tokens * H * (dv / 128) / 256 tokens (the share of one of the 256 compute units), rounded up to a
 * multiple of 64 and at least 512; as a rule this call wins when the longest sequence is longer than about 2.5
 * segments (measured at H = 16, dv = 256, 32768 tokens, segments of 4096: 390 us whatever the lengths, against 330 us
 * uncut when the longest sequence has 8192 tokens, 640 us at 16311 and 1000 us at 25045).
 *
 *   workspace   rodimus_chunk_scan_varlen_workspace_bytes(...) bytes of device memory, 16-byte aligned, contents
 *               undefined before and after; must not overlap any other argument.  The size depends on N and
 *               total_tokens only (the largest number of segments the batch can have); 0 = this batch is not cut
 *               (under 1024 tokens in all, more than 256 sequences, or a shape the matrix-core kernels do not take)
 *               and the call is then exactly rodimus_chunk_scan_varlen_fwd; workspace may be NULL.
 *
 * Every other argument, layout, aliasing rule and status code as for rodimus_chunk_scan_varlen_fwd (S_T may be S0);
 * RODIMUS_ERR_WORKSPACE if the workspace is missing or too small, RODIMUS_ERR_ALIAS if it overlaps another argument.
 */
int rodimus_chunk_scan_varlen_fwd_cut(const void *q, const void *k, const void *v,
                                      const float *log_alpha, const void *beta, int beta_kind, const float *S0,
                                      void *o, float *S_T,
                                      const int *cu_seqlens, int N, int total_tokens,
                                      int H, int dk, int dv, int chunk, int io_dtype,
                                      void *workspace, size_t workspace_bytes, void *stream);

size_t rodimus_chunk_scan_varlen_workspace_bytes(int N, int total_tokens, int H, int dk, int dv, int chunk, int io_dtype);

/* Activation of the output gate in the *_block calls. */
typedef enum {
    RODIMUS_GATE_SIGMOID = 0,         /* act(z) = sigmoid(z): the gated linear unit as cited by the paper   */
    RODIMUS_GATE_SILU = 1             /* act(z) = z * sigmoid(z): the gate of the Mamba-style blocks        */
} rodimus_gate_act;

/*
 * The two recurrence calls with the output stage of the block fused into the store of o (paper Sec. 3.1.3: the block's
 * state-space form ends with the feed-through o_t = q_t S_t + d .* x'_t, and the block is merged into a gated linear unit
 * whose output gate multiplies o).  Identical to rodimus_chunk_scan_fwd / rodimus_decode_step except:
 *
 *   beta, beta_kind   the value gate as in rodimus_chunk_scan_varlen_fwd (values, pre-activations, or NULL)
 *   x_prime     [B,T,H,dv] / [N,H,dv] io_dtype   in, or NULL = no feed-through
 *   d           [H,dv] fp32                      in, required with x_prime
 *   z_gate      [B,T,H,dv] / [N,H,dv] io_dtype   in, or NULL = no output gate
 *   gate_act    rodimus_gate_act (the paper does not print the activation; both common readings are offered)
 *   o           = (q S + d .* x') .* act(z_gate), evaluated in fp32 and rounded once
 *
 * The decode kernel and the generic scan kernel apply the stage where they store o (no extra pass over o); the MFMA scan
 * kernel has no registers left for two more input streams, so on that path the stage is a second, bandwidth-bound kernel
 * of the same call that rewrites o in place.  S_T / S are unaffected.  An unknown gate_act or beta_kind gives
 * RODIMUS_ERR_DTYPE; x_prime without d gives RODIMUS_ERR_NULL.
 */
int rodimus_chunk_scan_fwd_block(const void *q, const void *k, const void *v,
                                 const float *log_alpha, const void *beta, int beta_kind, const float *S0,
                                 const void *x_prime, const float *d, const void *z_gate, int gate_act,
                                 void *o, float *S_T,
                                 int B, int T, int H, int dk, int dv, int chunk, int io_dtype,
                                 void *workspace, size_t workspace_bytes, void *stream);

int rodimus_decode_step_block(const void *q, const void *k, const void *v,
                              const float *log_alpha, const void *beta, int beta_kind,
                              const void *x_prime, const float *d, const void *z_gate, int gate_act,
                              float *S, void *o,
                              int N, int H, int dk, int dv, int io_dtype, void *stream);

/*
 * Backward pass of rodimus_chunk_scan_fwd (training; paper Sec. 3.1.3 trains the block through its chunkwise form):
 * reverse-mode differentiation of the recurrence.  Given the cotangents d_o of the outputs and dS_T of the final
 * state, with u_t = beta_t .* v_t, a_t = exp(log_alpha_t) and G_t = q_t^T do_t + diag(a_{t+1}) G_{t+1} the total
 * cotangent of S_t:
 *     dq_t = do_t S_t^T,  dk_t = u_t G_t^T,  dv_t = beta_t .* (k_t G_t),  dbeta_t = v_t .* (k_t G_t),
 *     dlog_alpha_t = a_t .* rowsum(G_t .* S_{t-1}),  dS0 = diag(a_1) G_1.
 *
 *   q, k, v, log_alpha, beta, S0    as for rodimus_chunk_scan_fwd                      in
 *   d_o         [B,T,H,dv] io_dtype      in
 *   dS_T        [B,H,dk,dv] fp32         in, or NULL = zero
 *   dq, dk      [B,T,H,dk] io_dtype      out
 *   dv          [B,T,H,dv] io_dtype      out
 *   dlog_alpha  [B,T,H,dk] fp32          out   (0 where log_alpha <= -128: such a gate is treated as closed)
 *   dbeta       [B,T,H,dv] fp32          out, or NULL if not wanted (v .* (k G) is written even when beta is NULL)
 *   dS0         [B,H,dk,dv] fp32         out, or NULL if not wanted
 *   workspace   rodimus_chunk_scan_bwd_workspace_bytes(...) bytes of device scratch (q .* dq, and on the MFMA path k .* dk,
 *               in fp32), 16-byte aligned
 *
 * No output may overlap an input, another output or the workspace.  Two kernel families:
 *   io_dtype = BF16, dk = 64, dv = 128 or 256, any T: bf16 MFMA operands, fp32 accumulation and fp32 gate arithmetic, a
 *     16-token tile as the internal chunk; a forward sweep for dq and a reverse sweep for dk, dv, dbeta, dS0 run side by
 *     side in one launch (one workgroup per (batch, head) each), a second launch forms dlog_alpha; when B * H is small
 *     (2 * B * H < 192) and T >= 512 the sequences are cut into segments of at least 256 tokens that run as workgroups of
 *     their own, the states and state cotangents at the cuts coming from two summary passes (larger workspace);
 *   any other shape with dk <= 128 and dk * (dv + 1) <= 32768, either io_dtype: token by token in fp32 with the state in
 *     LDS (one workgroup per (batch, head), a forward launch then a reverse launch) -- complete, not fast.
 * Anything else returns RODIMUS_ERR_SHAPE (also T * H >= 2^31).
 */
int rodimus_chunk_scan_bwd(const void *q, const void *k, const void *v,
                           const float *log_alpha, const float *beta, const float *S0,
                           const void *d_o, const float *dS_T,
                           void *dq, void *dk, void *dv_out, float *dlog_alpha, float *dbeta, float *dS0,
                           int B, int T, int H, int dk_width, int dv, int io_dtype,
                           void *workspace, size_t workspace_bytes, void *stream);

/* Scratch bytes the call above needs (0 if the shape is not supported). */
size_t rodimus_chunk_scan_bwd_workspace_bytes(int B, int T, int H, int dk, int dv, int io_dtype);

/*
 * The backward pass of rodimus_chunk_scan_fwd_zbeta: the value gate arrives as its pre-activation (paper Sec. 3.1.2,
 * beta_hat = sigmoid(z_beta)) and its cotangent leaves as that of the pre-activation, so that no fp32 gate tensor is
 * read or written (18 % fewer bytes than rodimus_chunk_scan_bwd on the layer shapes):
 *
 *   z_beta      [B,T,H,dv] io_dtype      in    required
 *   dz_beta     [B,T,H,dv] io_dtype      out, or NULL if not wanted:  (v .* (k G)) .* beta_hat (1 - beta_hat)
 *   everything else as in rodimus_chunk_scan_bwd (same workspace size).
 *
 * Matrix-core shapes only (io_dtype = BF16, dk = 64, dv = 128 or 256); any other shape returns RODIMUS_ERR_SHAPE (evaluate
 * the gate with rodimus_ddts_gates and call rodimus_chunk_scan_bwd there).
 */
int rodimus_chunk_scan_bwd_zbeta(const void *q, const void *k, const void *v,
                                 const float *log_alpha, const void *z_beta, const float *S0,
                                 const void *d_o, const float *dS_T,
                                 void *dq, void *dk, void *dv_out, float *dlog_alpha, void *dz_beta, float *dS0,
                                 int B, int T, int H, int dk_width, int dv, int io_dtype,
                                 void *workspace, size_t workspace_bytes, void *stream);

/*
 * The backward pass of rodimus_chunk_scan_fwd_gated: training through the whole DDTS gate front-end (paper Sec. 3.1.2,
 * definitions of alpha, alpha-hat and beta-hat; pre-processing of q and k in Sec. 3.1.3).  With g = softplus(z_g),
 * tau = sigmoid(z_tau), w = g^tau, n = max(||k||_2, 1e-12) the forward call scans with log_alpha = -g .* tau,
 * k_hat = w .* k / n, q_hat = q / sqrt(dk), beta_hat = sigmoid(z_beta); this call returns the cotangents of the RAW q, k, v
 * and of the three pre-activations:
 *
 *   q, k, z_g, z_tau   [B,T,H,dk] io_dtype     in
 *   v, d_o             [B,T,H,dv] io_dtype     in
 *   z_beta             [B,T,H,dv] io_dtype     in, or NULL = no value gate (then dz_beta must be NULL)
 *   S0, dS_T           [B,H,dk,dv] fp32        in, or NULL = zero
 *   dq, dk, dz_g, dz_tau [B,T,H,dk] io_dtype   out
 *   dv, dz_beta        [B,T,H,dv] io_dtype     out (dz_beta may be NULL)
 *   dS0                [B,H,dk,dv] fp32        out, or NULL
 *
 *     dq   = dq_hat / sqrt(dk)
 *     dk   = dk_hat .* w / n - k (sum_r dk_hat_r w_r k_r) / n^3     (second term only while ||k|| is above the guard)
 *     dz_g   = (-dlog_alpha .* tau + dw .* tau .* w ./ g) .* sigmoid(z_g),        dw = dk_hat .* k / n
 *     dz_tau = (-dlog_alpha .* g   + dw .* w .* ln g) .* tau .* (1 - tau)
 *
 * where dq_hat, dk_hat, dlog_alpha, dv, dz_beta, dS0 are what rodimus_chunk_scan_bwd_zbeta returns for the scan on
 * (q_hat, k_hat, log_alpha, z_beta).  Three steps on `stream`: the key-side gate pass into the workspace, the backward of
 * the scan, the backward of the gate pass (dq_hat and dk_hat pass through the dq and dk buffers, in the I/O dtype).
 * Matrix-core shapes only (io_dtype = BF16, dk = 64, dv = 128 or 256), others return RODIMUS_ERR_SHAPE.  On an argument
 * error no output is written (the workspace may have been).
 */
int rodimus_chunk_scan_bwd_gated(const void *q, const void *k, const void *v,
                                 const void *z_g, const void *z_tau, const void *z_beta,
                                 const float *S0, const void *d_o, const float *dS_T,
                                 void *dq, void *dk, void *dv_out, void *dz_g, void *dz_tau, void *dz_beta, float *dS0,
                                 int B, int T, int H, int dk_width, int dv, int io_dtype,
                                 void *workspace, size_t workspace_bytes, void *stream);

/* Scratch bytes the call above needs (0 if the shape is not supported). */
size_t rodimus_chunk_scan_bwd_gated_workspace_bytes(int B, int T, int H, int dk, int dv, int io_dtype);

/*
 * rodimus_chunk_scan_bwd_gated over a PACKED batch of N sequences of different lengths (training on packed batches straight
 * from the projections; the backward of rodimus_chunk_scan_varlen_fwd_gated_block without its output stage): the same
 * chain rule and the same three steps, with the layouts and the length table of rodimus_chunk_scan_varlen_bwd:
 *
 *   token tensors [total_tokens,H,.], S0, dS_T, dS0 [N,H,dk,dv], cu_seqlens [N+1] int32 in DEVICE memory (clamped by the
 *   kernels); cut != 0: the scan backward in the middle lets the kernels cut the sequences into segments, as
 *   rodimus_chunk_scan_varlen_bwd_cut (for batches dominated by few long sequences);
 *   workspace: rodimus_chunk_scan_varlen_bwd_gated_workspace_bytes(..., cut) bytes.
 *
 * Shapes, alignment, aliasing rules and status codes as for rodimus_chunk_scan_bwd_gated.
 */
int rodimus_chunk_scan_varlen_bwd_gated(const void *q, const void *k, const void *v,
                                        const void *z_g, const void *z_tau, const void *z_beta,
                                        const float *S0, const void *d_o, const float *dS_T,
                                        void *dq, void *dk, void *dv_out, void *dz_g, void *dz_tau, void *dz_beta, float *dS0,
                                        const int *cu_seqlens, int N, int total_tokens,
                                        int H, int dk_width, int dv, int io_dtype, int cut,
                                        void *workspace, size_t workspace_bytes, void *stream);

size_t rodimus_chunk_scan_varlen_bwd_gated_workspace_bytes(int N, int total_tokens, int H, int dk, int dv, int io_dtype, int cut);

/*
 * Backward pass over a packed batch of sequences of different lengths (training on packed sequences; the backward of
 * rodimus_chunk_scan_varlen_fwd with the value gate given as values): exactly rodimus_chunk_scan_bwd applied to every
 * sequence, with the layouts of rodimus_chunk_scan_varlen_fwd:
 *
 *   q, k, log_alpha, dq, dk, dlog_alpha   [total_tokens,H,dk]          v, beta, d_o, dv, dbeta   [total_tokens,H,dv]
 *   S0, dS_T, dS0                         [N,H,dk,dv] fp32             cu_seqlens   [N+1] int32, device (clamped as there)
 *   workspace   rodimus_chunk_scan_varlen_bwd_workspace_bytes(...) bytes
 *
 * Same kernel families, NULL conventions, alignment, aliasing rules and status codes as rodimus_chunk_scan_bwd; an empty
 * sequence gets dS0 = dS_T.
 */
int rodimus_chunk_scan_varlen_bwd(const void *q, const void *k, const void *v,
                                  const float *log_alpha, const float *beta, const float *S0,
                                  const void *d_o, const float *dS_T,
                                  void *dq, void *dk, void *dv_out, float *dlog_alpha, float *dbeta, float *dS0,
                                  const int *cu_seqlens, int N, int total_tokens,
                                  int H, int dk_width, int dv, int io_dtype,
                                  void *workspace, size_t workspace_bytes, void *stream);

size_t rodimus_chunk_scan_varlen_bwd_workspace_bytes(int N, int total_tokens, int H, int dk, int dv, int io_dtype);

/*
 * rodimus_chunk_scan_varlen_bwd for a packed batch dominated by FEW LONG sequences (the backward counterpart of
 * rodimus_chunk_scan_varlen_fwd_cut, with the same reasoning): the kernels cut every sequence into segments of a fixed
 * length chosen from total_tokens alone -- total_tokens * H / 256 tokens, rounded up to a multiple of 64, at least 256 --
 * find each segment's sequence from cu_seqlens on the device, and run the segments side by side: the state entering and
 * the state cotangent leaving every segment come from two summary passes and two chains along each sequence, then both
 * sweeps and the gate pass run per segment.  Same results as rodimus_chunk_scan_varlen_bwd to rounding.  The summary
 * passes read k, v, the gates, q and d_o once more, so the call pays when the longest sequence would otherwise keep most
 * of the chip waiting (as a rule: longer than about three segments).
 *
 *   workspace   rodimus_chunk_scan_varlen_bwd_cut_workspace_bytes(...) bytes; the size depends on N and total_tokens only.
 *               Batches under 512 tokens or of more than 256 sequences and shapes outside the matrix-core kernels (bf16,
 *               dk = 64, dv = 128 or 256) are not cut: the call is then exactly rodimus_chunk_scan_varlen_bwd and the size function returns that
 *               call's size.
 *
 * Every other argument, layout, aliasing rule and status code as for rodimus_chunk_scan_varlen_bwd.
 */
int rodimus_chunk_scan_varlen_bwd_cut(const void *q, const void *k, const void *v,
                                      const float *log_alpha, const float *beta, const float *S0,
                                      const void *d_o, const float *dS_T,
                                      void *dq, void *dk, void *dv,
                                      float *dlog_alpha, float *dbeta, float *dS0,
                                      const int *cu_seqlens, int N, int total_tokens,
                                      int H, int dk_width, int dv_width, int io_dtype,
                                      void *workspace, size_t workspace_bytes, void *stream);

size_t rodimus_chunk_scan_varlen_bwd_cut_workspace_bytes(int N, int total_tokens, int H, int dk, int dv, int io_dtype);

/*
 * The two recurrence calls with the whole DDTS gate front-end fused in (paper Sec. 3.1.2 and the pre-processing of q and k
 * in Sec. 3.1.3; the block's state-space form of Sec. 3.1.3 evaluated straight from the projections): every gate arrives
 * as its pre-activation and q, k arrive raw.  Per token and head, inside the kernels, in fp32:
 *     g = softplus(z_g), tau = sigmoid(z_tau)
 *     S_t = diag(exp(-g .* tau)) S_{t-1} + (g^tau .* k_t / max(||k_t||_2, 1e-12))^T (sigmoid(z_beta_t) .* v_t)
 *     o_t = (q_t / sqrt(dk)) S_t
 * i.e. rodimus_ddts_gates followed by rodimus_chunk_scan_fwd / rodimus_decode_step without the pass over HBM in between
 * (no log_alpha, beta, scaled q or folded k is ever stored).
 *
 *   q, k        [B,T,H,dk] / [N,H,dk] io_dtype   in, raw projections
 *   z_g, z_tau  same shape as q, io_dtype        in
 *   z_beta      [B,T,H,dv] / [N,H,dv] io_dtype   in, or NULL = value gate of all ones
 *   everything else as in rodimus_chunk_scan_fwd / rodimus_decode_step (shapes, kernel families, workspace, alignment,
 *   aliasing, status codes).
 */
int rodimus_chunk_scan_fwd_gated(const void *q, const void *k, const void *v,
                                 const void *z_g, const void *z_tau, const void *z_beta, const float *S0,
                                 void *o, float *S_T,
                                 int B, int T, int H, int dk, int dv, int chunk, int io_dtype,
                                 void *workspace, size_t workspace_bytes, void *stream);

int rodimus_decode_step_gated(const void *q, const void *k, const void *v,
                              const void *z_g, const void *z_tau, const void *z_beta,
                              float *S, void *o,
                              int N, int H, int dk, int dv, int io_dtype, void *stream);

/*
 * The whole block of Sec. 3.1.3 around the recurrence in one call: the gates and the pre-processing of q and k as in
 * rodimus_chunk_scan_fwd_gated / rodimus_decode_step_gated (Sec. 3.1.2) AND the output stage of rodimus_chunk_scan_fwd_block /
 * rodimus_decode_step_block (feed-through d .* x' and output gate act(z_gate)), all inside the kernel that runs the
 * recurrence:
 *     y_t = (q_t / sqrt(dk) S_t + d .* x'_t) .* act(z_gate_t)
 * Arguments as in those calls (x_prime, z_gate may each be NULL; d is required with x_prime; z_beta may be NULL).
 */
int rodimus_chunk_scan_fwd_gated_block(const void *q, const void *k, const void *v,
                                       const void *z_g, const void *z_tau, const void *z_beta, const float *S0,
                                       const void *x_prime, const float *d, const void *z_gate, int gate_act,
                                       void *o, float *S_T,
                                       int B, int T, int H, int dk, int dv, int chunk, int io_dtype,
                                       void *workspace, size_t workspace_bytes, void *stream);
int rodimus_decode_step_gated_block(const void *q, const void *k, const void *v,
                                    const void *z_g, const void *z_tau, const void *z_beta,
                                    const void *x_prime, const float *d, const void *z_gate, int gate_act,
                                    float *S, void *o,
                                    int N, int H, int dk, int dv, int io_dtype, void *stream);

/*
 * rodimus_chunk_scan_fwd_gated_block over a PACKED batch of N sequences of different lengths (serving prefill of the whole
 * block in one launch; paper Sec. 3.1.2 and 3.1.3 as for the calls it combines): the layouts and the length table of
 * rodimus_chunk_scan_varlen_fwd, the gates and the output stage of rodimus_chunk_scan_fwd_gated_block.
 *
 *   q, k, z_g, z_tau          [total_tokens,H,dk] io_dtype   in
 *   v, z_beta, x_prime, z_gate [total_tokens,H,dv] io_dtype  in   z_beta, x_prime (with d [H,dv] fp32) and z_gate may each be
 *                                                                 NULL: no value gate / no feed-through / no output gate
 *   S0, S_T                   [N,H,dk,dv] fp32               S_T may be S0 (a state cache updated in place)
 *   cu_seqlens                [N+1] int32, DEVICE memory     as in rodimus_chunk_scan_varlen_fwd (clamped by the kernels)
 *   workspace                 NULL: one workgroup set per (sequence, head), as rodimus_chunk_scan_varlen_fwd;
 *                             otherwise rodimus_chunk_scan_varlen_workspace_bytes(...) bytes: the kernels cut the sequences
 *                             into segments that run side by side, as rodimus_chunk_scan_varlen_fwd_cut (same rule of thumb)
 *
 * Shapes, kernel families, alignment, aliasing rules and status codes as for the calls it combines.
 */
int rodimus_chunk_scan_varlen_fwd_gated_block(const void *q, const void *k, const void *v,
                                              const void *z_g, const void *z_tau, const void *z_beta, const float *S0,
                                              const void *x_prime, const float *d, const void *z_gate, int gate_act,
                                              void *o, float *S_T,
                                              const int *cu_seqlens, int N, int total_tokens,
                                              int H, int dk, int dv, int chunk, int io_dtype,
                                              void *workspace, size_t workspace_bytes, void *stream);

/*
 * The two recurrence calls with the general transition of paper Sec. 3.1.1 (first equation of the section), which gates
 * the state along the value dimension as well:
 *     S_t = (alpha_t^T beta_t) .* S_{t-1} + k_t^T (beta_hat_t .* v_t),   o_t = q_t S_t
 * The paper fixes beta_t = 1 for the block after an ablation (the other calls); this variant is for the models of its
 * comparison table that use such a gate.
 *
 *   log_beta_t  [B,T,H,dv] / [N,H,dv] fp32     in, required: log of the transition gate beta_t, <= 0 (-inf allowed)
 *   beta        the input gate beta_hat on the value, fp32 values or NULL = all ones (as in rodimus_chunk_scan_fwd)
 *   everything else as in rodimus_chunk_scan_fwd / rodimus_decode_step.
 *
 * The scan always runs on the any-shape fp32 kernel (no workspace): the pair (write i, read t) carries
 * exp(sum_{j=i+1..t} log_beta_j) per value column, which is evaluated per pair (never as a quotient of running
 * products), so this form is several times slower than the block's own recurrence.  The decode step costs the same as
 * rodimus_decode_step.
 */
int rodimus_chunk_scan_fwd_general(const void *q, const void *k, const void *v,
                                   const float *log_alpha, const float *log_beta_t, const float *beta, const float *S0,
                                   void *o, float *S_T,
                                   int B, int T, int H, int dk, int dv, int chunk, int io_dtype, void *stream);

int rodimus_decode_step_general(const void *q, const void *k, const void *v,
                                const float *log_alpha, const float *log_beta_t, const float *beta,
                                float *S, void *o,
                                int N, int H, int dk, int dv, int io_dtype, void *stream);

/* Activation after the short convolution. */
typedef enum {
    RODIMUS_CONV_NONE = 0,            /* the convolution alone                                              */
    RODIMUS_CONV_SILU = 1             /* z * sigmoid(z), as in the recurrent models the paper points to     */
} rodimus_conv_act;

/*
 * ShortConv of the block (paper Sec. 3.1.3: the block's input x_t passes through a short convolution to give x'_t,
 * which feeds the gates and the feed-through term).  The paper names the operator without printing it; the reading
 * taken is a causal depthwise convolution over time of width W with a bias, then the activation:
 *     x'_t[c] = act( bias[c] + sum_{j=0..W-1} w[c][j] * x_{t-(W-1)+j}[c] )
 * (w[c][W-1] multiplies the current token).  Inputs before the call's first token come from state_in or are zero.
 *
 *   x           [B,T,C] io_dtype         in
 *   w           [C,W] fp32               in
 *   bias        [C] fp32                 in, or NULL = zero
 *   state_in    [B,W-1,C] io_dtype       in, or NULL = zero history; the last W-1 inputs of the previous call, oldest first
 *   y           [B,T,C] io_dtype         out
 *   state_out   [B,W-1,C] io_dtype       out, or NULL if not wanted: the last W-1 inputs seen so far
 *   act         rodimus_conv_act
 *
 * fp32 arithmetic, one rounding at the store.  Supported: 1 <= W <= 8, C % 8 == 0; B, T or C equal to 0 is a no-op
 * (T = 0 still copies state_in to state_out).  No output may overlap an input or the other output.  An unknown act
 * gives RODIMUS_ERR_DTYPE.
 */
int rodimus_short_conv_fwd(const void *x, const float *w, const float *bias, const void *state_in,
                           void *y, void *state_out,
                           int B, int T, int C, int W, int act, int io_dtype, void *stream);

/*
 * One decode step of the same operator for N sequences (paper Sec. 3.1.3: at inference only fixed-size state is kept;
 * for ShortConv that state is the last W-1 inputs):
 *
 *   x           [N,C] io_dtype           in
 *   state       [N,W-1,C] io_dtype       in/out, updated IN PLACE (shifted by one token, x appended); NULL only if W = 1
 *   y           [N,C] io_dtype           out
 */
int rodimus_short_conv_step(const void *x, const float *w, const float *bias, void *state, void *y,
                            int N, int C, int W, int act, int io_dtype, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* RODIMUS_H */
