// C-ABI entry points of librodimus_hip: argument validation on the host, then dispatch to a kernel
// family.  Nothing here allocates, synchronises or keeps state.  See include/rodimus.h for the contract.
#include "internal.h"

#include <mutex>

namespace {

using namespace rodimus;

inline bool misaligned(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) != 0; }

inline bool overlaps(const void *a, size_t a_bytes, const void *b, size_t b_bytes)
{
    if (a == nullptr || b == nullptr || a_bytes == 0 || b_bytes == 0) return false;
    const uintptr_t a0 = reinterpret_cast<uintptr_t>(a), b0 = reinterpret_cast<uintptr_t>(b);
    return a0 < b0 + b_bytes && b0 < a0 + a_bytes;
}

inline size_t elem_bytes(int io_dtype) { return io_dtype == RODIMUS_BF16 ? 2 : 4; }

constexpr int kMaxScanDk = 128;
constexpr int kMaxChunk = 64;
constexpr int kMaxChunkTimesDk = 4096;
constexpr int kMaxDecodeDk = 256;
constexpr long long kMaxGridX = 2147483647LL;

// Shape rules shared by the scan entry point and its two query functions.
int scan_shape_status(int B, int T, int H, int dk, int dv, int chunk, int io_dtype)
{
    if (io_dtype != RODIMUS_F32 && io_dtype != RODIMUS_BF16) return RODIMUS_ERR_DTYPE;
    if (B < 0 || T < 0 || H < 0) return RODIMUS_ERR_SHAPE;
    if (dk < 1 || dk > kMaxScanDk || dv < 1) return RODIMUS_ERR_SHAPE;
    if (chunk < 1 || chunk > kMaxChunk || chunk * dk > kMaxChunkTimesDk) return RODIMUS_ERR_SHAPE;
    if ((long long)B * H > kMaxGridX || (dv + 63) / 64 > 65535) return RODIMUS_ERR_SHAPE;
    return RODIMUS_OK;
}

// The value gate `beta` is either fp32 gate values or (beta_preact) pre-activations in the I/O dtype.
// Dense layout: B sequences of T tokens.  Packed layout (`packed`): B sequences, T tokens in total, sequence b owning
// the rows [cu_seqlens[b], cu_seqlens[b+1]) (device memory, so its contents cannot be checked here; the kernels
// clamp them to the tensor).
int scan_entry(const void *q, const void *k, const void *v, const float *log_alpha, const void *beta, bool beta_preact,
               const float *S0, void *o, float *S_T, int B, int T, int H, int dk, int dv, int chunk, int io_dtype,
               void *workspace, size_t workspace_bytes, void *stream, bool packed = false, const int *cu_seqlens = nullptr,
               OutputStage stage = OutputStage{nullptr, nullptr, nullptr, 0}, bool gated = false, const void *z_g = nullptr,
               const void *z_tau = nullptr, bool general = false, const float *log_beta_t = nullptr, bool packed_cut = false)
{
    const int shape = scan_shape_status(B, T, H, dk, dv, chunk, io_dtype);
    if (shape != RODIMUS_OK) return shape;
    if (packed && B > 0 && cu_seqlens == nullptr) return RODIMUS_ERR_NULL;
    if (packed && misaligned(cu_seqlens)) return RODIMUS_ERR_ALIGN;
    if (packed && ((long long)B * H + 8) * ((dv + 127) / 128) > kMaxGridX) return RODIMUS_ERR_SHAPE;      // the packed scan runs on a flat grid, rounded up to whole runs of eight
    const size_t tokens = packed ? (size_t)T * H : (size_t)B * T * H;
    // the key-side gates: log_alpha (fp32), or in the gated form the two pre-activations (I/O dtype)
    const void *gate_a = gated ? z_g : static_cast<const void *>(log_alpha);
    const void *gate_b = gated ? z_tau : nullptr;
    if (tokens > 0 && (!q || !k || !v || !gate_a || !o)) return RODIMUS_ERR_NULL;   // empty tensors may be NULL
    if (tokens > 0 && gated && !gate_b) return RODIMUS_ERR_NULL;
    if (tokens > 0 && beta_preact && !beta && !gated) return RODIMUS_ERR_NULL;
    if (tokens > 0 && general && !log_beta_t) return RODIMUS_ERR_NULL;
    if (misaligned(q) || misaligned(k) || misaligned(v) || misaligned(gate_a) || misaligned(gate_b) || misaligned(beta) ||
        misaligned(S0) || misaligned(o) || misaligned(S_T) || misaligned(workspace) || misaligned(log_beta_t))
        return RODIMUS_ERR_ALIGN;

    const size_t eb = elem_bytes(io_dtype);
    const size_t qk_bytes = tokens * dk * eb, v_bytes = tokens * dv * eb;
    const size_t la_bytes = tokens * dk * (gated ? eb : 4), beta_bytes = tokens * dv * (beta_preact ? eb : 4);
    const size_t state_bytes = (size_t)B * H * dk * dv * 4;
    if (overlaps(o, v_bytes, q, qk_bytes) || overlaps(o, v_bytes, k, qk_bytes) || overlaps(o, v_bytes, v, v_bytes) ||
        overlaps(o, v_bytes, gate_a, la_bytes) || overlaps(o, v_bytes, gate_b, la_bytes) ||
        overlaps(o, v_bytes, beta, beta_bytes) || overlaps(o, v_bytes, S0, state_bytes) || overlaps(o, v_bytes, S_T, state_bytes))
        return RODIMUS_ERR_ALIAS;
    if (S_T != nullptr && S_T != S0 && overlaps(S_T, state_bytes, S0, state_bytes)) return RODIMUS_ERR_ALIAS;
    if (overlaps(S_T, state_bytes, q, qk_bytes) || overlaps(S_T, state_bytes, k, qk_bytes) ||
        overlaps(S_T, state_bytes, v, v_bytes) || overlaps(S_T, state_bytes, gate_a, la_bytes) ||
        overlaps(S_T, state_bytes, gate_b, la_bytes) || overlaps(S_T, state_bytes, beta, beta_bytes))
        return RODIMUS_ERR_ALIAS;
    if (stage.x_prime != nullptr && stage.d == nullptr) return RODIMUS_ERR_NULL;
    if (misaligned(stage.x_prime) || misaligned(stage.d) || misaligned(stage.z_gate)) return RODIMUS_ERR_ALIGN;
    if (overlaps(o, v_bytes, stage.x_prime, v_bytes) || overlaps(o, v_bytes, stage.z_gate, v_bytes) ||
        overlaps(o, v_bytes, stage.d, (size_t)H * dv * 4) || overlaps(S_T, state_bytes, stage.x_prime, v_bytes) ||
        overlaps(S_T, state_bytes, stage.z_gate, v_bytes) || overlaps(S_T, state_bytes, stage.d, (size_t)H * dv * 4))
        return RODIMUS_ERR_ALIAS;
    if (overlaps(o, v_bytes, log_beta_t, tokens * dv * 4) || overlaps(S_T, state_bytes, log_beta_t, tokens * dv * 4))
        return RODIMUS_ERR_ALIAS;
    const size_t cu_bytes = packed ? ((size_t)B + 1) * sizeof(int) : 0;
    if (overlaps(o, v_bytes, cu_seqlens, cu_bytes) || overlaps(S_T, state_bytes, cu_seqlens, cu_bytes)) return RODIMUS_ERR_ALIAS;

    // the general transition runs on the any-shape kernel only
    const bool mfma = !general && scan_mfma_supports(dk, dv, chunk, io_dtype);
    // a packed batch is cut along its sequences only through the entry point that brings a workspace for it
    const size_t need = !mfma ? 0 : !packed ? scan_mfma_workspace_bytes(B, T, H, dv)
                                : packed_cut ? scan_mfma_packed_workspace_bytes(B, T, H, dv) : 0;
    if (need > 0 && (workspace == nullptr || workspace_bytes < need)) return RODIMUS_ERR_WORKSPACE;
    if (need > 0) {
        // the kernels write the first `need` bytes of the workspace while they read the inputs and write the outputs
        const void *others[13] = {q, k, v, gate_a, gate_b, beta, S0, o, S_T, stage.x_prime, stage.d, stage.z_gate, log_beta_t};
        const size_t other_bytes[13] = {qk_bytes, qk_bytes, v_bytes, la_bytes, la_bytes, beta_bytes, state_bytes, v_bytes, state_bytes,
                                        v_bytes, (size_t)H * dv * 4, v_bytes, tokens * dv * 4};
        for (int i = 0; i < 13; ++i)
            if (overlaps(workspace, need, others[i], other_bytes[i])) return RODIMUS_ERR_ALIAS;
    }

    ScanArgs a{q, k, v, log_alpha, beta, beta_preact, S0, o, S_T, B, T, H, dk, dv, chunk, io_dtype,
               packed ? cu_seqlens : nullptr, stage, need > 0 ? workspace : nullptr, workspace_bytes, static_cast<hipStream_t>(stream)};
    if (gated) { a.log_alpha = nullptr; a.z_g = z_g; a.z_tau = z_tau; }
    if (general) a.log_beta_t = log_beta_t;
    const hipError_t err = mfma ? launch_scan_mfma(a) : launch_scan_generic(a);
    return err == hipSuccess ? RODIMUS_OK : RODIMUS_ERR_LAUNCH;
}

int decode_entry(const void *q, const void *k, const void *v, const float *log_alpha, const void *beta, bool beta_preact,
                 float *S, void *o, int N, int H, int dk, int dv, int io_dtype, void *stream,
                 OutputStage stage = OutputStage{nullptr, nullptr, nullptr, 0}, bool gated = false, const void *z_g = nullptr,
                 const void *z_tau = nullptr, bool general = false, const float *log_beta_t = nullptr)
{
    if (io_dtype != RODIMUS_F32 && io_dtype != RODIMUS_BF16) return RODIMUS_ERR_DTYPE;
    if (N < 0 || H < 0 || dk < 1 || dk > kMaxDecodeDk || dv < 4 || (dv & 3) != 0) return RODIMUS_ERR_SHAPE;
    if ((long long)N * H > kMaxGridX || (dv + 255) / 256 > 65535) return RODIMUS_ERR_SHAPE;
    const size_t states = (size_t)N * H;
    const void *gate_a = gated ? z_g : static_cast<const void *>(log_alpha);
    const void *gate_b = gated ? z_tau : nullptr;
    if (states > 0 && (!q || !k || !v || !gate_a || !S || !o)) return RODIMUS_ERR_NULL;
    if (states > 0 && gated && !gate_b) return RODIMUS_ERR_NULL;
    if (states > 0 && beta_preact && !beta && !gated) return RODIMUS_ERR_NULL;
    if (states > 0 && general && !log_beta_t) return RODIMUS_ERR_NULL;
    if (misaligned(q) || misaligned(k) || misaligned(v) || misaligned(gate_a) || misaligned(gate_b) || misaligned(beta) ||
        misaligned(S) || misaligned(o) || misaligned(log_beta_t))
        return RODIMUS_ERR_ALIGN;

    const size_t eb = elem_bytes(io_dtype);
    const size_t o_bytes = states * dv * eb, s_bytes = states * dk * dv * 4;
    const size_t beta_bytes = states * dv * (beta_preact ? eb : 4), la_bytes = states * dk * (gated ? eb : 4);
    if (overlaps(o, o_bytes, q, states * dk * eb) || overlaps(o, o_bytes, k, states * dk * eb) ||
        overlaps(o, o_bytes, v, o_bytes) || overlaps(o, o_bytes, gate_a, la_bytes) || overlaps(o, o_bytes, gate_b, la_bytes) ||
        overlaps(o, o_bytes, beta, beta_bytes) || overlaps(o, o_bytes, S, s_bytes))
        return RODIMUS_ERR_ALIAS;
    if (overlaps(S, s_bytes, q, states * dk * eb) || overlaps(S, s_bytes, k, states * dk * eb) ||
        overlaps(S, s_bytes, v, o_bytes) || overlaps(S, s_bytes, gate_a, la_bytes) || overlaps(S, s_bytes, gate_b, la_bytes) ||
        overlaps(S, s_bytes, beta, beta_bytes))
        return RODIMUS_ERR_ALIAS;

    if (overlaps(o, o_bytes, log_beta_t, states * dv * 4) || overlaps(S, s_bytes, log_beta_t, states * dv * 4))
        return RODIMUS_ERR_ALIAS;
    if (stage.x_prime != nullptr && stage.d == nullptr) return RODIMUS_ERR_NULL;
    if (misaligned(stage.x_prime) || misaligned(stage.d) || misaligned(stage.z_gate)) return RODIMUS_ERR_ALIGN;
    if (overlaps(o, o_bytes, stage.x_prime, o_bytes) || overlaps(o, o_bytes, stage.z_gate, o_bytes) ||
        overlaps(o, o_bytes, stage.d, (size_t)H * dv * 4) || overlaps(S, s_bytes, stage.x_prime, o_bytes) ||
        overlaps(S, s_bytes, stage.z_gate, o_bytes) || overlaps(S, s_bytes, stage.d, (size_t)H * dv * 4))
        return RODIMUS_ERR_ALIAS;
    DecodeArgs a{q, k, v, log_alpha, beta, beta_preact, stage, S, o, N, H, dk, dv, io_dtype, static_cast<hipStream_t>(stream)};
    if (gated) { a.log_alpha = nullptr; a.z_g = z_g; a.z_tau = z_tau; }
    if (general) a.log_beta_t = log_beta_t;
    const hipError_t err = launch_decode_step(a);
    return err == hipSuccess ? RODIMUS_OK : RODIMUS_ERR_LAUNCH;
}

}  // namespace

extern "C" {

const char *rodimus_status_string(int status)
{
    switch (status) {
    case RODIMUS_OK: return "ok";
    case RODIMUS_ERR_NULL: return "a required pointer is NULL";
    case RODIMUS_ERR_SHAPE: return "a size is invalid or outside the supported range";
    case RODIMUS_ERR_DTYPE: return "io_dtype is not RODIMUS_F32 or RODIMUS_BF16";
    case RODIMUS_ERR_ALIGN: return "a base pointer is not 16-byte aligned";
    case RODIMUS_ERR_WORKSPACE: return "workspace is missing or too small";
    case RODIMUS_ERR_LAUNCH: return "the HIP runtime refused the launch";
    case RODIMUS_ERR_ALIAS: return "an output overlaps an input it must not overlap";
    case RODIMUS_ERR_SCRATCH: return "the call needs more scratch than the library's built-in buffer holds (or the buffer could not be located)";
    default: return "unknown status";
    }
}

int rodimus_hbm_stream_probe(const void *src, void *dst, size_t units, int reads_per_write, int workgroups, void *stream)
{
    if (reads_per_write != 0 && reads_per_write != 1 && reads_per_write != 2 && reads_per_write != 4) return RODIMUS_ERR_SHAPE;
    if (workgroups < 1 || workgroups > 1 << 20) return RODIMUS_ERR_SHAPE;
    if (units > 0 && (!dst || (reads_per_write > 0 && !src))) return RODIMUS_ERR_NULL;
    if (misaligned(src) || misaligned(dst)) return RODIMUS_ERR_ALIGN;
    if (overlaps(dst, units * 16, src, units * 16 * (size_t)reads_per_write)) return RODIMUS_ERR_ALIAS;
    const hipError_t err = launch_hbm_stream_probe(src, dst, units, reads_per_write, workgroups, static_cast<hipStream_t>(stream));
    return err == hipSuccess ? RODIMUS_OK : RODIMUS_ERR_LAUNCH;
}

int rodimus_chunk_scan_path(int B, int T, int H, int dk, int dv, int chunk, int io_dtype)
{
    if (scan_shape_status(B, T, H, dk, dv, chunk, io_dtype) != RODIMUS_OK) return RODIMUS_PATH_NONE;
    return scan_mfma_supports(dk, dv, chunk, io_dtype) ? RODIMUS_PATH_MFMA : RODIMUS_PATH_GENERIC;
}

size_t rodimus_chunk_scan_workspace_bytes(int B, int T, int H, int dk, int dv, int chunk, int io_dtype)
{
    if (scan_shape_status(B, T, H, dk, dv, chunk, io_dtype) != RODIMUS_OK) return 0;
    return scan_mfma_supports(dk, dv, chunk, io_dtype) ? scan_mfma_workspace_bytes(B, T, H, dv) : 0;
}

int rodimus_chunk_scan_fwd(const void *q, const void *k, const void *v, const float *log_alpha, const float *beta,
                           const float *S0, void *o, float *S_T, int B, int T, int H, int dk, int dv, int chunk,
                           int io_dtype, void *workspace, size_t workspace_bytes, void *stream)
{
    return scan_entry(q, k, v, log_alpha, beta, false, S0, o, S_T, B, T, H, dk, dv, chunk, io_dtype, workspace,
                      workspace_bytes, stream);
}

int rodimus_chunk_scan_fwd_zbeta(const void *q, const void *k, const void *v, const float *log_alpha, const void *z_beta,
                                 const float *S0, void *o, float *S_T, int B, int T, int H, int dk, int dv, int chunk,
                                 int io_dtype, void *workspace, size_t workspace_bytes, void *stream)
{
    return scan_entry(q, k, v, log_alpha, z_beta, true, S0, o, S_T, B, T, H, dk, dv, chunk, io_dtype, workspace,
                      workspace_bytes, stream);
}

int rodimus_chunk_scan_varlen_fwd(const void *q, const void *k, const void *v, const float *log_alpha, const void *beta,
                                  int beta_kind, const float *S0, void *o, float *S_T, const int *cu_seqlens, int N,
                                  int total_tokens, int H, int dk, int dv, int chunk, int io_dtype, void *stream)
{
    if (beta_kind != RODIMUS_BETA_VALUES && beta_kind != RODIMUS_BETA_PREACTIVATION) return RODIMUS_ERR_DTYPE;
    return scan_entry(q, k, v, log_alpha, beta, beta_kind == RODIMUS_BETA_PREACTIVATION, S0, o, S_T, N, total_tokens, H,
                      dk, dv, chunk, io_dtype, nullptr, 0, stream, true, cu_seqlens);
}

size_t rodimus_chunk_scan_varlen_workspace_bytes(int N, int total_tokens, int H, int dk, int dv, int chunk, int io_dtype)
{
    if (scan_shape_status(N, total_tokens, H, dk, dv, chunk, io_dtype) != RODIMUS_OK) return 0;
    return scan_mfma_supports(dk, dv, chunk, io_dtype) ? scan_mfma_packed_workspace_bytes(N, total_tokens, H, dv) : 0;
}

int rodimus_chunk_scan_varlen_fwd_cut(const void *q, const void *k, const void *v, const float *log_alpha, const void *beta,
                                      int beta_kind, const float *S0, void *o, float *S_T, const int *cu_seqlens, int N,
                                      int total_tokens, int H, int dk, int dv, int chunk, int io_dtype, void *workspace,
                                      size_t workspace_bytes, void *stream)
{
    if (beta_kind != RODIMUS_BETA_VALUES && beta_kind != RODIMUS_BETA_PREACTIVATION) return RODIMUS_ERR_DTYPE;
    return scan_entry(q, k, v, log_alpha, beta, beta_kind == RODIMUS_BETA_PREACTIVATION, S0, o, S_T, N, total_tokens, H,
                      dk, dv, chunk, io_dtype, workspace, workspace_bytes, stream, true, cu_seqlens,
                      OutputStage{nullptr, nullptr, nullptr, 0}, false, nullptr, nullptr, false, nullptr, true);
}

int rodimus_chunk_scan_fwd_block(const void *q, const void *k, const void *v, const float *log_alpha, const void *beta,
                                 int beta_kind, const float *S0, const void *x_prime, const float *d, const void *z_gate,
                                 int gate_act, void *o, float *S_T, int B, int T, int H, int dk, int dv, int chunk,
                                 int io_dtype, void *workspace, size_t workspace_bytes, void *stream)
{
    if (beta_kind != RODIMUS_BETA_VALUES && beta_kind != RODIMUS_BETA_PREACTIVATION) return RODIMUS_ERR_DTYPE;
    if (gate_act != RODIMUS_GATE_SIGMOID && gate_act != RODIMUS_GATE_SILU) return RODIMUS_ERR_DTYPE;
    return scan_entry(q, k, v, log_alpha, beta, beta_kind == RODIMUS_BETA_PREACTIVATION, S0, o, S_T, B, T, H, dk, dv, chunk,
                      io_dtype, workspace, workspace_bytes, stream, false, nullptr, OutputStage{x_prime, d, z_gate, gate_act});
}

int rodimus_decode_step_block(const void *q, const void *k, const void *v, const float *log_alpha, const void *beta,
                              int beta_kind, const void *x_prime, const float *d, const void *z_gate, int gate_act,
                              float *S, void *o, int N, int H, int dk, int dv, int io_dtype, void *stream)
{
    if (beta_kind != RODIMUS_BETA_VALUES && beta_kind != RODIMUS_BETA_PREACTIVATION) return RODIMUS_ERR_DTYPE;
    if (gate_act != RODIMUS_GATE_SIGMOID && gate_act != RODIMUS_GATE_SILU) return RODIMUS_ERR_DTYPE;
    return decode_entry(q, k, v, log_alpha, beta, beta_kind == RODIMUS_BETA_PREACTIVATION, S, o, N, H, dk, dv, io_dtype, stream,
                        OutputStage{x_prime, d, z_gate, gate_act});
}

int rodimus_decode_step(const void *q, const void *k, const void *v, const float *log_alpha, const float *beta,
                        float *S, void *o, int N, int H, int dk, int dv, int io_dtype, void *stream)
{
    return decode_entry(q, k, v, log_alpha, beta, false, S, o, N, H, dk, dv, io_dtype, stream);
}

int rodimus_decode_step_zbeta(const void *q, const void *k, const void *v, const float *log_alpha, const void *z_beta,
                              float *S, void *o, int N, int H, int dk, int dv, int io_dtype, void *stream)
{
    return decode_entry(q, k, v, log_alpha, z_beta, true, S, o, N, H, dk, dv, io_dtype, stream);
}

int rodimus_chunk_scan_fwd_gated(const void *q, const void *k, const void *v, const void *z_g, const void *z_tau,
                                 const void *z_beta, const float *S0, void *o, float *S_T, int B, int T, int H, int dk, int dv,
                                 int chunk, int io_dtype, void *workspace, size_t workspace_bytes, void *stream)
{
    return scan_entry(q, k, v, nullptr, z_beta, true, S0, o, S_T, B, T, H, dk, dv, chunk, io_dtype, workspace, workspace_bytes,
                      stream, false, nullptr, OutputStage{nullptr, nullptr, nullptr, 0}, true, z_g, z_tau);
}

int rodimus_decode_step_gated(const void *q, const void *k, const void *v, const void *z_g, const void *z_tau,
                              const void *z_beta, float *S, void *o, int N, int H, int dk, int dv, int io_dtype, void *stream)
{
    return decode_entry(q, k, v, nullptr, z_beta, true, S, o, N, H, dk, dv, io_dtype, stream,
                        OutputStage{nullptr, nullptr, nullptr, 0}, true, z_g, z_tau);
}

int rodimus_chunk_scan_fwd_gated_block(const void *q, const void *k, const void *v, const void *z_g, const void *z_tau,
                                       const void *z_beta, const float *S0, const void *x_prime, const float *d, const void *z_gate,
                                       int gate_act, void *o, float *S_T, int B, int T, int H, int dk, int dv, int chunk, int io_dtype,
                                       void *workspace, size_t workspace_bytes, void *stream)
{
    if (gate_act != RODIMUS_GATE_SIGMOID && gate_act != RODIMUS_GATE_SILU) return RODIMUS_ERR_DTYPE;
    return scan_entry(q, k, v, nullptr, z_beta, true, S0, o, S_T, B, T, H, dk, dv, chunk, io_dtype, workspace, workspace_bytes,
                      stream, false, nullptr, OutputStage{x_prime, d, z_gate, gate_act}, true, z_g, z_tau);
}

int rodimus_decode_step_gated_block(const void *q, const void *k, const void *v, const void *z_g, const void *z_tau,
                                    const void *z_beta, const void *x_prime, const float *d, const void *z_gate, int gate_act,
                                    float *S, void *o, int N, int H, int dk, int dv, int io_dtype, void *stream)
{
    if (gate_act != RODIMUS_GATE_SIGMOID && gate_act != RODIMUS_GATE_SILU) return RODIMUS_ERR_DTYPE;
    return decode_entry(q, k, v, nullptr, z_beta, true, S, o, N, H, dk, dv, io_dtype, stream, OutputStage{x_prime, d, z_gate, gate_act},
                        true, z_g, z_tau);
}

int rodimus_chunk_scan_varlen_fwd_gated_block(const void *q, const void *k, const void *v, const void *z_g, const void *z_tau,
                                              const void *z_beta, const float *S0, const void *x_prime, const float *d,
                                              const void *z_gate, int gate_act, void *o, float *S_T, const int *cu_seqlens, int N,
                                              int total_tokens, int H, int dk, int dv, int chunk, int io_dtype, void *workspace,
                                              size_t workspace_bytes, void *stream)
{
    if (gate_act != RODIMUS_GATE_SIGMOID && gate_act != RODIMUS_GATE_SILU) return RODIMUS_ERR_DTYPE;
    // without a workspace the batch is never cut along its sequences
    return scan_entry(q, k, v, nullptr, z_beta, true, S0, o, S_T, N, total_tokens, H, dk, dv, chunk, io_dtype, workspace,
                      workspace_bytes, stream, true, cu_seqlens, OutputStage{x_prime, d, z_gate, gate_act}, true, z_g, z_tau, false,
                      nullptr, workspace != nullptr);
}

int rodimus_chunk_scan_fwd_general(const void *q, const void *k, const void *v, const float *log_alpha,
                                   const float *log_beta_t, const float *beta, const float *S0, void *o, float *S_T, int B, int T,
                                   int H, int dk, int dv, int chunk, int io_dtype, void *stream)
{
    return scan_entry(q, k, v, log_alpha, beta, false, S0, o, S_T, B, T, H, dk, dv, chunk, io_dtype, nullptr, 0, stream, false,
                      nullptr, OutputStage{nullptr, nullptr, nullptr, 0}, false, nullptr, nullptr, true, log_beta_t);
}

int rodimus_decode_step_general(const void *q, const void *k, const void *v, const float *log_alpha, const float *log_beta_t,
                                const float *beta, float *S, void *o, int N, int H, int dk, int dv, int io_dtype, void *stream)
{
    return decode_entry(q, k, v, log_alpha, beta, false, S, o, N, H, dk, dv, io_dtype, stream,
                        OutputStage{nullptr, nullptr, nullptr, 0}, false, nullptr, nullptr, true, log_beta_t);
}

}  // extern "C"

namespace {

size_t bwd_workspace(size_t token_rows, int B, int T, int H, int dk, int dv, int io_dtype, bool packed)
{
    if (io_dtype != RODIMUS_F32 && io_dtype != RODIMUS_BF16) return 0;
    if (scan_bwd_supports(dk, dv, io_dtype)) return scan_bwd_workspace_bytes(token_rows, B, T, H, dv, packed);
    return scan_bwd_generic_supports(dk, dv) ? scan_bwd_generic_workspace_bytes(token_rows, B, H, dk) : 0;
}

// Dense layout: B sequences of T tokens.  Packed (`packed`): B sequences, T tokens in total, lengths in cu_seqlens (device).
// beta_preact: `beta` holds the pre-activations of the value gate in the I/O dtype (required then) and `dbeta` receives their
// cotangent in the I/O dtype; matrix-core shapes only.
int bwd_entry(const void *q, const void *k, const void *v, const float *log_alpha, const void *beta, const float *S0,
              const void *d_o, const float *dS_T, void *dq, void *dk, void *dv_out, float *dlog_alpha, void *dbeta, float *dS0,
              int B, int T, int H, int dk_width, int dv, int io_dtype, void *workspace, size_t workspace_bytes, void *stream,
              bool packed, const int *cu_seqlens, bool beta_preact = false, bool packed_cut = false)
{
    if (io_dtype != RODIMUS_F32 && io_dtype != RODIMUS_BF16) return RODIMUS_ERR_DTYPE;
    if (B < 0 || T < 0 || H < 0 || (long long)B * H > kMaxGridX) return RODIMUS_ERR_SHAPE;
    if ((long long)T * H > kMaxGridX) return RODIMUS_ERR_SHAPE;          // the kernels index a sequence's rows in 32 bits
    const bool mfma = scan_bwd_supports(dk_width, dv, io_dtype);
    if (!mfma && (beta_preact || !scan_bwd_generic_supports(dk_width, dv))) return RODIMUS_ERR_SHAPE;
    if (packed && B > 0 && cu_seqlens == nullptr) return RODIMUS_ERR_NULL;
    if (packed && misaligned(cu_seqlens)) return RODIMUS_ERR_ALIGN;
    const size_t token_rows = packed ? (size_t)T : (size_t)B * T;
    const size_t tokens = token_rows * H, states = (size_t)B * H;
    if (tokens > 0 && (!q || !k || !v || !log_alpha || !d_o || !dq || !dk || !dv_out || !dlog_alpha)) return RODIMUS_ERR_NULL;
    if (tokens > 0 && beta_preact && !beta) return RODIMUS_ERR_NULL;
    const size_t eb = elem_bytes(io_dtype);
    const size_t gate_bytes = beta_preact ? eb : 4;                      // bytes per element of beta and of dbeta
    const void *ins[9] = {q, k, v, log_alpha, beta, S0, d_o, dS_T, packed ? cu_seqlens : nullptr};
    const size_t in_bytes[9] = {tokens * dk_width * eb, tokens * dk_width * eb, tokens * dv * eb, tokens * dk_width * 4,
                                tokens * dv * gate_bytes, states * dk_width * dv * 4, tokens * dv * eb, states * dk_width * dv * 4,
                                packed ? ((size_t)B + 1) * sizeof(int) : 0};
    void *outs[7] = {dq, dk, dv_out, dlog_alpha, dbeta, dS0, workspace};
    size_t need = bwd_workspace(token_rows, B, T, H, dk_width, dv, io_dtype, packed);
    // a packed batch is cut along its sequences only on request, by the matrix-core kernels, and if it is long enough
    const size_t need_cut = (packed && packed_cut && mfma) ? scan_bwd_packed_cut_workspace_bytes(B, T, H, dv) : 0;
    packed_cut = need_cut > 0;
    if (packed_cut) need = need_cut;
    const size_t out_bytes[7] = {tokens * dk_width * eb, tokens * dk_width * eb, tokens * dv * eb, tokens * dk_width * 4,
                                 tokens * dv * gate_bytes, states * dk_width * dv * 4, need};
    for (int i = 0; i < 9; ++i)
        if (misaligned(ins[i])) return RODIMUS_ERR_ALIGN;
    for (int o = 0; o < 7; ++o)
        if (misaligned(outs[o])) return RODIMUS_ERR_ALIGN;
    for (int o = 0; o < 7; ++o) {
        for (int i = 0; i < 9; ++i)
            if (overlaps(outs[o], out_bytes[o], ins[i], in_bytes[i])) return RODIMUS_ERR_ALIAS;
        for (int p = o + 1; p < 7; ++p)
            if (overlaps(outs[o], out_bytes[o], outs[p], out_bytes[p])) return RODIMUS_ERR_ALIAS;
    }
    if (states > 0 && need > 0 && (workspace == nullptr || workspace_bytes < need)) return RODIMUS_ERR_WORKSPACE;

    ScanBwdArgs a{q, k, v, log_alpha, beta, S0, d_o, dS_T, dq, dk, dv_out, dlog_alpha, dbeta, dS0, B, T, H, dk_width, dv,
                  io_dtype, workspace, workspace_bytes, static_cast<hipStream_t>(stream)};
    if (packed) a.cu_seqlens = cu_seqlens;
    a.beta_preact = beta_preact;
    a.packed_cut = packed_cut;
    return (mfma ? launch_scan_bwd(a) : launch_scan_bwd_generic(a)) == hipSuccess ? RODIMUS_OK : RODIMUS_ERR_LAUNCH;
}

}  // namespace

extern "C" {

size_t rodimus_chunk_scan_bwd_workspace_bytes(int B, int T, int H, int dk, int dv, int io_dtype)
{
    if (B < 0 || T < 0 || H < 0) return 0;
    return bwd_workspace((size_t)B * T, B, T, H, dk, dv, io_dtype, false);
}

size_t rodimus_chunk_scan_varlen_bwd_workspace_bytes(int N, int total_tokens, int H, int dk, int dv, int io_dtype)
{
    if (N < 0 || total_tokens < 0 || H < 0) return 0;
    return bwd_workspace((size_t)total_tokens, N, total_tokens, H, dk, dv, io_dtype, true);
}

int rodimus_chunk_scan_bwd(const void *q, const void *k, const void *v, const float *log_alpha, const float *beta,
                           const float *S0, const void *d_o, const float *dS_T, void *dq, void *dk, void *dv_out,
                           float *dlog_alpha, float *dbeta, float *dS0, int B, int T, int H, int dk_width, int dv,
                           int io_dtype, void *workspace, size_t workspace_bytes, void *stream)
{
    return bwd_entry(q, k, v, log_alpha, beta, S0, d_o, dS_T, dq, dk, dv_out, dlog_alpha, dbeta, dS0, B, T, H, dk_width, dv,
                     io_dtype, workspace, workspace_bytes, stream, false, nullptr);
}

int rodimus_chunk_scan_bwd_zbeta(const void *q, const void *k, const void *v, const float *log_alpha, const void *z_beta,
                                 const float *S0, const void *d_o, const float *dS_T, void *dq, void *dk, void *dv_out,
                                 float *dlog_alpha, void *dz_beta, float *dS0, int B, int T, int H, int dk_width, int dv,
                                 int io_dtype, void *workspace, size_t workspace_bytes, void *stream)
{
    return bwd_entry(q, k, v, log_alpha, z_beta, S0, d_o, dS_T, dq, dk, dv_out, dlog_alpha, dz_beta, dS0, B, T, H, dk_width, dv,
                     io_dtype, workspace, workspace_bytes, stream, false, nullptr, true);
}

// Backward of the gated scan: key-side gate pass into the workspace, backward of the scan on its outputs (value gate as
// its pre-activation), then the backward of the gate pass.  Workspace: log_alpha fp32, scaled q and folded k in the I/O
// dtype, dlog_alpha fp32 (each [B,T,H,dk]), then the scan backward's own workspace.  The cotangents of the scaled q and the
// folded k pass through the caller's dq and dk buffers, which the last kernel updates in place.
static size_t gated_bwd_front_bytes(size_t tokens, int dk, int io_dtype) { return tokens * dk * (4 + 2 * elem_bytes(io_dtype) + 4); }

// workspace of the scan backward inside the gated backward: dense, packed, or packed and cut by the kernels
static size_t gated_bwd_inner_bytes(int B, int T, int H, int dk, int dv, int io_dtype, bool packed, bool packed_cut)
{
    if (!packed) return bwd_workspace((size_t)B * T, B, T, H, dk, dv, io_dtype, false);
    const size_t cut = packed_cut ? scan_bwd_packed_cut_workspace_bytes(B, T, H, dv) : 0;
    return cut > 0 ? cut : bwd_workspace((size_t)T, B, T, H, dk, dv, io_dtype, true);
}

// Dense: B sequences of T tokens.  Packed: B sequences, T tokens in all, lengths in cu_seqlens (device).
static int bwd_gated_entry(const void *q, const void *k, const void *v, const void *z_g, const void *z_tau, const void *z_beta,
                           const float *S0, const void *d_o, const float *dS_T, void *dq, void *dk, void *dv_out, void *dz_g,
                           void *dz_tau, void *dz_beta, float *dS0, int B, int T, int H, int dk_width, int dv, int io_dtype,
                           void *workspace, size_t workspace_bytes, void *stream, bool packed, const int *cu_seqlens, bool packed_cut)
{
    if (io_dtype != RODIMUS_F32 && io_dtype != RODIMUS_BF16) return RODIMUS_ERR_DTYPE;
    if (B < 0 || T < 0 || H < 0 || (long long)B * H > kMaxGridX || (long long)T * H > kMaxGridX) return RODIMUS_ERR_SHAPE;
    if (!scan_bwd_supports(dk_width, dv, io_dtype)) return RODIMUS_ERR_SHAPE;       // matrix-core shapes only
    const size_t tokens = packed ? (size_t)T * H : (size_t)B * T * H;
    if (tokens == 0) return bwd_entry(q, k, v, nullptr, z_beta, S0, d_o, dS_T, dq, dk, dv_out, nullptr, dz_beta, dS0, B, T, H, dk_width,
                                      dv, io_dtype, workspace, workspace_bytes, stream, packed, cu_seqlens, z_beta != nullptr);
    if (!q || !k || !v || !z_g || !z_tau || !d_o || !dq || !dk || !dv_out || !dz_g || !dz_tau) return RODIMUS_ERR_NULL;
    if (z_beta == nullptr && dz_beta != nullptr) return RODIMUS_ERR_NULL;
    if (misaligned(z_g) || misaligned(z_tau) || misaligned(dz_g) || misaligned(dz_tau) || misaligned(workspace)) return RODIMUS_ERR_ALIGN;
    const size_t eb = elem_bytes(io_dtype), key_bytes = tokens * dk_width * eb;
    const size_t front = gated_bwd_front_bytes(tokens, dk_width, io_dtype);
    const size_t need = front + gated_bwd_inner_bytes(B, T, H, dk_width, dv, io_dtype, packed, packed_cut);
    if (workspace == nullptr || workspace_bytes < need) return RODIMUS_ERR_WORKSPACE;
    // the two extra inputs and outputs against everything else (the call below checks the rest, workspace included)
    const void *others[16] = {q, k, v, z_beta, S0, d_o, dS_T, dq, dk, dv_out, dz_beta, dS0, workspace, z_g, z_tau,
                              packed ? cu_seqlens : nullptr};
    const size_t state_bytes = (size_t)B * H * dk_width * dv * 4, val_bytes = tokens * dv * eb;
    const size_t other_bytes[16] = {key_bytes, key_bytes, val_bytes, val_bytes, state_bytes, val_bytes, state_bytes, key_bytes, key_bytes,
                                    val_bytes, val_bytes, state_bytes, need, key_bytes, key_bytes,
                                    packed ? ((size_t)B + 1) * sizeof(int) : 0};
    void *extra_out[2] = {dz_g, dz_tau};
    for (int o = 0; o < 2; ++o)
        for (int i = 0; i < 16; ++i)
            if (overlaps(extra_out[o], key_bytes, others[i], other_bytes[i])) return RODIMUS_ERR_ALIAS;
    if (overlaps(dz_g, key_bytes, dz_tau, key_bytes)) return RODIMUS_ERR_ALIAS;
    const void *extra_in[2] = {z_g, z_tau};
    for (int e = 0; e < 2; ++e)
        for (int i = 7; i < 13; ++i)
            if (overlaps(extra_in[e], key_bytes, others[i], other_bytes[i])) return RODIMUS_ERR_ALIAS;

    char *ws = static_cast<char *>(workspace);
    float *log_alpha = reinterpret_cast<float *>(ws);
    void *q_hat = ws + tokens * dk_width * 4;
    void *k_hat = static_cast<char *>(q_hat) + key_bytes;
    float *dlog_alpha = reinterpret_cast<float *>(static_cast<char *>(k_hat) + key_bytes);
    void *inner_ws = ws + front;

    // validate the inner call's arguments before anything is launched: a dry run with zero sequences is not possible, so
    // the order is gate pass, inner call (which validates and returns before its own launches on error), gate backward
    GateArgs ga{z_g, z_tau, nullptr, q, k, log_alpha, nullptr, q_hat, k_hat, (long long)tokens, dk_width, dv, io_dtype,
                static_cast<hipStream_t>(stream)};
    if (launch_ddts_gates(ga) != hipSuccess) return RODIMUS_ERR_LAUNCH;
    const int inner = bwd_entry(q_hat, k_hat, v, log_alpha, z_beta, S0, d_o, dS_T, dq, dk, dv_out, dlog_alpha, dz_beta, dS0, B, T, H,
                                dk_width, dv, io_dtype, inner_ws, workspace_bytes - front, stream, packed, cu_seqlens, z_beta != nullptr,
                                packed_cut);
    if (inner != RODIMUS_OK) return inner;
    GateBwdArgs gb{z_g, z_tau, k, dq, dk, dlog_alpha, dz_g, dz_tau, dq, dk, (long long)tokens, dk_width, io_dtype,
                   static_cast<hipStream_t>(stream)};
    return launch_ddts_gates_bwd(gb) == hipSuccess ? RODIMUS_OK : RODIMUS_ERR_LAUNCH;
}

size_t rodimus_chunk_scan_bwd_gated_workspace_bytes(int B, int T, int H, int dk, int dv, int io_dtype)
{
    if (B < 0 || T < 0 || H < 0 || !scan_bwd_supports(dk, dv, io_dtype)) return 0;
    return gated_bwd_front_bytes((size_t)B * T * H, dk, io_dtype) + gated_bwd_inner_bytes(B, T, H, dk, dv, io_dtype, false, false);
}

int rodimus_chunk_scan_bwd_gated(const void *q, const void *k, const void *v, const void *z_g, const void *z_tau, const void *z_beta,
                                 const float *S0, const void *d_o, const float *dS_T, void *dq, void *dk, void *dv_out, void *dz_g,
                                 void *dz_tau, void *dz_beta, float *dS0, int B, int T, int H, int dk_width, int dv, int io_dtype,
                                 void *workspace, size_t workspace_bytes, void *stream)
{
    return bwd_gated_entry(q, k, v, z_g, z_tau, z_beta, S0, d_o, dS_T, dq, dk, dv_out, dz_g, dz_tau, dz_beta, dS0, B, T, H, dk_width, dv,
                           io_dtype, workspace, workspace_bytes, stream, false, nullptr, false);
}

size_t rodimus_chunk_scan_varlen_bwd_gated_workspace_bytes(int N, int total_tokens, int H, int dk, int dv, int io_dtype, int cut)
{
    if (N < 0 || total_tokens < 0 || H < 0 || !scan_bwd_supports(dk, dv, io_dtype)) return 0;
    return gated_bwd_front_bytes((size_t)total_tokens * H, dk, io_dtype) +
           gated_bwd_inner_bytes(N, total_tokens, H, dk, dv, io_dtype, true, cut != 0);
}

int rodimus_chunk_scan_varlen_bwd_gated(const void *q, const void *k, const void *v, const void *z_g, const void *z_tau,
                                        const void *z_beta, const float *S0, const void *d_o, const float *dS_T, void *dq, void *dk,
                                        void *dv_out, void *dz_g, void *dz_tau, void *dz_beta, float *dS0, const int *cu_seqlens, int N,
                                        int total_tokens, int H, int dk_width, int dv, int io_dtype, int cut, void *workspace,
                                        size_t workspace_bytes, void *stream)
{
    if (N > 0 && cu_seqlens == nullptr) return RODIMUS_ERR_NULL;
    return bwd_gated_entry(q, k, v, z_g, z_tau, z_beta, S0, d_o, dS_T, dq, dk, dv_out, dz_g, dz_tau, dz_beta, dS0, N, total_tokens, H,
                           dk_width, dv, io_dtype, workspace, workspace_bytes, stream, true, cu_seqlens, cut != 0);
}

int rodimus_chunk_scan_varlen_bwd(const void *q, const void *k, const void *v, const float *log_alpha, const float *beta,
                                  const float *S0, const void *d_o, const float *dS_T, void *dq, void *dk, void *dv_out,
                                  float *dlog_alpha, float *dbeta, float *dS0, const int *cu_seqlens, int N, int total_tokens,
                                  int H, int dk_width, int dv, int io_dtype, void *workspace, size_t workspace_bytes, void *stream)
{
    return bwd_entry(q, k, v, log_alpha, beta, S0, d_o, dS_T, dq, dk, dv_out, dlog_alpha, dbeta, dS0, N, total_tokens, H,
                     dk_width, dv, io_dtype, workspace, workspace_bytes, stream, true, cu_seqlens);
}

size_t rodimus_chunk_scan_varlen_bwd_cut_workspace_bytes(int N, int total_tokens, int H, int dk, int dv, int io_dtype)
{
    if (N < 0 || total_tokens < 0 || H < 0) return 0;
    const size_t cut = scan_bwd_supports(dk, dv, io_dtype) ? scan_bwd_packed_cut_workspace_bytes(N, total_tokens, H, dv) : 0;
    return cut > 0 ? cut : bwd_workspace((size_t)total_tokens, N, total_tokens, H, dk, dv, io_dtype, true);
}

int rodimus_chunk_scan_varlen_bwd_cut(const void *q, const void *k, const void *v, const float *log_alpha, const float *beta,
                                      const float *S0, const void *d_o, const float *dS_T, void *dq, void *dk, void *dv_out,
                                      float *dlog_alpha, float *dbeta, float *dS0, const int *cu_seqlens, int N, int total_tokens,
                                      int H, int dk_width, int dv, int io_dtype, void *workspace, size_t workspace_bytes, void *stream)
{
    return bwd_entry(q, k, v, log_alpha, beta, S0, d_o, dS_T, dq, dk, dv_out, dlog_alpha, dbeta, dS0, N, total_tokens, H,
                     dk_width, dv, io_dtype, workspace, workspace_bytes, stream, true, cu_seqlens, false, true);
}

int rodimus_ddts_gates(const void *z_g, const void *z_tau, const void *z_beta, const void *q, const void *k,
                       float *log_alpha, float *beta, void *q_out, void *k_out, long long rows, int dk, int dv,
                       int io_dtype, void *stream)
{
    if (io_dtype != RODIMUS_F32 && io_dtype != RODIMUS_BF16) return RODIMUS_ERR_DTYPE;
    if (rows < 0 || dk < 8 || dk > 512 || (dk & (dk - 1)) != 0) return RODIMUS_ERR_SHAPE;
    if ((z_beta == nullptr) != (beta == nullptr)) return RODIMUS_ERR_NULL;
    if (z_beta != nullptr && (dv < 8 || (dv & 7) != 0)) return RODIMUS_ERR_SHAPE;
    if (rows * (dk / 8) / 256 >= kMaxGridX || (z_beta && (unsigned long long)rows * dv / 8 / 256 >= (unsigned long long)kMaxGridX))
        return RODIMUS_ERR_SHAPE;
    if (rows > 0 && (!z_g || !z_tau || !q || !k || !log_alpha || !q_out || !k_out)) return RODIMUS_ERR_NULL;
    if (misaligned(z_g) || misaligned(z_tau) || misaligned(z_beta) || misaligned(q) || misaligned(k) ||
        misaligned(log_alpha) || misaligned(beta) || misaligned(q_out) || misaligned(k_out))
        return RODIMUS_ERR_ALIGN;

    const size_t eb = elem_bytes(io_dtype);
    const size_t key_bytes = (size_t)rows * dk * eb, la_bytes = (size_t)rows * dk * 4;
    const size_t zb_bytes = (size_t)rows * (z_beta ? dv : 0) * eb, beta_bytes = (size_t)rows * (z_beta ? dv : 0) * 4;
    // q_out may be q and k_out may be k (same buffer); every other overlap between an output and anything else is refused
    const void *ins[5] = {z_g, z_tau, z_beta, q, k};
    const size_t in_bytes[5] = {key_bytes, key_bytes, zb_bytes, key_bytes, key_bytes};
    const void *outs[4] = {log_alpha, beta, q_out, k_out};
    const size_t out_bytes[4] = {la_bytes, beta_bytes, key_bytes, key_bytes};
    for (int o = 0; o < 4; ++o) {
        for (int i = 0; i < 5; ++i) {
            if ((o == 2 && i == 3 && q_out == q) || (o == 3 && i == 4 && k_out == k)) continue;
            if (overlaps(outs[o], out_bytes[o], ins[i], in_bytes[i])) return RODIMUS_ERR_ALIAS;
        }
        for (int p = o + 1; p < 4; ++p)
            if (overlaps(outs[o], out_bytes[o], outs[p], out_bytes[p])) return RODIMUS_ERR_ALIAS;
    }

    GateArgs a{z_g, z_tau, z_beta, q, k, log_alpha, beta, q_out, k_out, rows, dk, dv, io_dtype, static_cast<hipStream_t>(stream)};
    return launch_ddts_gates(a) == hipSuccess ? RODIMUS_OK : RODIMUS_ERR_LAUNCH;
}

}  // extern "C"

namespace {

int short_conv_entry(const void *x, const float *w, const float *bias, const void *state_in, void *y, void *state_out,
                     int B, int T, int C, int W, int act, int io_dtype, void *stream, bool in_place_state)
{
    if (io_dtype != RODIMUS_F32 && io_dtype != RODIMUS_BF16) return RODIMUS_ERR_DTYPE;
    if (act != RODIMUS_CONV_NONE && act != RODIMUS_CONV_SILU) return RODIMUS_ERR_DTYPE;
    if (B < 0 || T < 0 || C < 0 || W < 1 || W > 8 || (C & 7) != 0) return RODIMUS_ERR_SHAPE;
    if (B > 65535 || (T + 63) / 64 > 65535) return RODIMUS_ERR_SHAPE;      // grid limits (a run of 64 tokens per thread)
    const size_t eb = elem_bytes(io_dtype);
    const size_t x_bytes = (size_t)B * T * C * eb, st_bytes = (size_t)B * (W - 1) * C * eb;
    if (x_bytes > 0 && (!x || !y || !w)) return RODIMUS_ERR_NULL;
    if (st_bytes > 0 && state_out != nullptr && !w) return RODIMUS_ERR_NULL;
    if (in_place_state && st_bytes > 0 && state_in == nullptr) return RODIMUS_ERR_NULL;
    if (misaligned(x) || misaligned(w) || misaligned(bias) || misaligned(state_in) || misaligned(y) || misaligned(state_out))
        return RODIMUS_ERR_ALIGN;
    const size_t w_bytes = (size_t)C * W * 4, b_bytes = (size_t)C * 4;
    if (overlaps(y, x_bytes, x, x_bytes) || overlaps(y, x_bytes, w, w_bytes) || overlaps(y, x_bytes, bias, b_bytes) ||
        overlaps(y, x_bytes, state_in, st_bytes) || overlaps(y, x_bytes, state_out, st_bytes))
        return RODIMUS_ERR_ALIAS;
    if (overlaps(state_out, st_bytes, x, x_bytes) || overlaps(state_out, st_bytes, w, w_bytes) ||
        overlaps(state_out, st_bytes, bias, b_bytes))
        return RODIMUS_ERR_ALIAS;
    if (!in_place_state && overlaps(state_out, st_bytes, state_in, st_bytes)) return RODIMUS_ERR_ALIAS;
    ShortConvArgs a{x, w, bias, state_in, y, state_out, B, T, C, W, act, io_dtype, static_cast<hipStream_t>(stream)};
    return launch_short_conv(a) == hipSuccess ? RODIMUS_OK : RODIMUS_ERR_LAUNCH;
}

}  // namespace

extern "C" {

int rodimus_short_conv_fwd(const void *x, const float *w, const float *bias, const void *state_in, void *y, void *state_out,
                           int B, int T, int C, int W, int act, int io_dtype, void *stream)
{
    return short_conv_entry(x, w, bias, state_in, y, state_out, B, T, C, W, act, io_dtype, stream, false);
}

// One token per sequence; the kernel's thread reads the W-1 carried rows of its channels before it writes them back
// shifted, and no other thread touches them, so the state is updated in place.
int rodimus_short_conv_step(const void *x, const float *w, const float *bias, void *state, void *y, int N, int C, int W,
                            int act, int io_dtype, void *stream)
{
    return short_conv_entry(x, w, bias, state, y, state, N, 1, C, W, act, io_dtype, stream, true);
}

}  // extern "C"

// ---- the scan for callers that cannot allocate ------------------------------------------------------------------
// Same kernels as rodimus_chunk_scan_fwd; the workspace of a call that is cut along the sequence is a buffer inside the
// library's own device image instead of a caller allocation.  Every GPU holds its own copy of the array at its own
// address; host code may use the array's memory only through the address hipGetSymbolAddress returns for the current device.
namespace {

constexpr size_t kScratchBytes = (size_t)RODIMUS_NOALLOC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kScratchBytes];

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void *g_scratch_ptr[kMaxDevices];       // device address of `scratch` on each device, once looked up

// Address of the current device's copy of `scratch` (looked up once per device), or NULL on failure.
void *scratch_on_current_device()
{
    int device = -1;
    if (hipGetDevice(&device) != hipSuccess || device < 0 || device >= kMaxDevices) return nullptr;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (g_scratch_ptr[device] == nullptr) {
        void *ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess) return nullptr;
        g_scratch_ptr[device] = ptr;
    }
    return g_scratch_ptr[device];
}

}  // namespace

extern "C" {

size_t rodimus_chunk_scan_fwd_noalloc_scratch_bytes(void) { return kScratchBytes; }

int rodimus_chunk_scan_fwd_noalloc(const void *q, const void *k, const void *v, const float *log_alpha, const float *beta,
                                   const float *S0, void *o, float *S_T, int B, int T, int H, int dk, int dv, int chunk,
                                   int io_dtype, void *stream)
{
    const int shape = scan_shape_status(B, T, H, dk, dv, chunk, io_dtype);
    if (shape != RODIMUS_OK) return shape;
    const size_t need = scan_mfma_supports(dk, dv, chunk, io_dtype) ? scan_mfma_workspace_bytes(B, T, H, dv) : 0;
    if (need > kScratchBytes) return RODIMUS_ERR_SCRATCH;
    // the buffer's address on this device; if it cannot be found the call below still validates every argument and then
    // ends at its workspace check, before any launch
    void *ws = need > 0 ? scratch_on_current_device() : nullptr;
    // nothing in the buffer has to start at zero: the segment summaries, decays and entering states are all written by the
    // call's own kernels before they are read
    const int status = scan_entry(q, k, v, log_alpha, beta, false, S0, o, S_T, B, T, H, dk, dv, chunk, io_dtype, ws,
                                  ws != nullptr ? need : 0, stream);
    return status == RODIMUS_ERR_WORKSPACE ? RODIMUS_ERR_SCRATCH : status;
}

}  // extern "C"
