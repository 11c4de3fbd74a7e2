// Backward pass of the recurrence for any supported shape and I/O type, token by token in fp32 on the vector ALUs
// (the matrix-core kernels of scan_bwd.hip cover bf16, dk = 64, dv = 128 / 256).  Reverse-mode differentiation of
//     S_t = diag(a_t) S_{t-1} + k_t^T u_t,   o_t = q_t S_t,   a_t = exp(log_alpha_t), u_t = beta_t .* v_t
// (paper Sec. 3.1.3) with G_t = q_t^T do_t + diag(a_{t+1}) G_{t+1} the cotangent of S_t:
//     forward sweep  (scan_bwd_generic_dq_kernel):   S_t from S0;  dq_t = do_t S_t^T;  q_t .* dq_t kept in fp32
//     reverse sweep  (scan_bwd_generic_dkv_kernel):  dk_t = u_t G_t^T,  du_t = k_t G_t,  dv = beta .* du,  dbeta = v .* du,
//                    dlog_alpha_t = rowsum(S_T .* dS_T) + sum_{s>=t} (q_s .* dq_s - k_s .* dk_s)  (zero where a_t = 0),
//                    dS0 = diag(a_1) G_1
// The gate cotangent uses the same identity as the matrix-core path: the pairs that the gate of step t decays are
// counted once by q .* dq of the later steps and not by k .* dk of the later steps.
//
// One workgroup per (batch, head) keeps the whole dk x dv state (or cotangent) in LDS and walks the tokens in order:
// one elementwise pass over the state and one row (and column) reduction per token.  This is the any-shape path, not a
// fast one.
#include "internal.h"

namespace rodimus {

namespace {

constexpr int kGenThreads = 256;
constexpr int kGenMaxDk = 128;
constexpr int kGenMaxStateFloats = 32768;        // dk * (dv + 1) floats of LDS for the state

struct GenShape {
    int T, H, dk, dv;
    const int *cu_seqlens;      // packed batch (T = total tokens), or null
};

// LDS: state [dk][dv + 1] (padded rows: a row reduction walks along the row, a column reduction down the column),
// then the token's rows.
__host__ __device__ inline size_t gen_lds_floats(int dk, int dv) { return (size_t)dk * (dv + 1) + 3 * (size_t)dk + 3 * (size_t)dv + dk; }

template <typename IO>
__global__ __launch_bounds__(kGenThreads) void scan_bwd_generic_dq_kernel(
    const IO *__restrict__ q, const IO *__restrict__ k, const IO *__restrict__ v, const float *__restrict__ log_alpha,
    const float *__restrict__ beta, const float *__restrict__ S0, const IO *__restrict__ d_o, const float *__restrict__ dS_T,
    IO *__restrict__ dq, float *__restrict__ qdq, float *__restrict__ gate_const, GenShape sh)
{
    extern __shared__ float lds[];
    const int dk = sh.dk, dv = sh.dv, dvp = dv + 1;
    float *S = lds, *sq = S + dk * dvp, *skk = sq + dk, *sa = skk + dk, *su = sa + dk, *sdo = su + dv;
    const int tid = threadIdx.x, bh = blockIdx.x;
    const SeqSpan span = seq_span(bh / sh.H, sh.T, sh.cu_seqlens);
    sh.T = span.length;
    const size_t row0 = span.first * sh.H + bh % sh.H;
    const size_t state0 = (size_t)bh * dk * dv;
    const int elems = dk * dv;

    for (int e = tid; e < elems; e += kGenThreads) S[(e / dv) * dvp + e % dv] = S0 != nullptr ? S0[state0 + e] : 0.f;

    for (int t = 0; t < sh.T; ++t) {
        const size_t row = row0 + (size_t)t * sh.H;
        __syncthreads();                        // the previous token's reduction is done with S and the rows
        for (int r = tid; r < dk; r += kGenThreads) {
            sq[r] = load_as_float(q + row * dk + r);
            skk[r] = load_as_float(k + row * dk + r);
            sa[r] = expf(log_alpha[row * dk + r]);
        }
        for (int j = tid; j < dv; j += kGenThreads) {
            const float b = beta != nullptr ? beta[row * dv + j] : 1.f;
            su[j] = b * load_as_float(v + row * dv + j);
            sdo[j] = load_as_float(d_o + row * dv + j);
        }
        __syncthreads();
        for (int e = tid; e < elems; e += kGenThreads) {
            const int r = e / dv, j = e % dv;
            S[r * dvp + j] = fmaf(sa[r], S[r * dvp + j], skk[r] * su[j]);
        }
        __syncthreads();
        for (int r = tid; r < dk; r += kGenThreads) {
            float acc = 0.f;
            for (int j = 0; j < dv; ++j) acc = fmaf(S[r * dvp + j], sdo[j], acc);
            store_from_float(dq + row * dk + r, acc);
            qdq[row * dk + r] = sq[r] * acc;
        }
    }
    __syncthreads();
    // rowsum(S_T .* dS_T): the constant term of every gate cotangent of this (batch, head)
    for (int r = tid; r < dk; r += kGenThreads) {
        float acc = 0.f;
        if (dS_T != nullptr)
            for (int j = 0; j < dv; ++j) acc = fmaf(S[r * dvp + j], dS_T[state0 + (size_t)r * dv + j], acc);
        gate_const[(size_t)bh * dk + r] = acc;
    }
}

template <typename IO>
__global__ __launch_bounds__(kGenThreads) void scan_bwd_generic_dkv_kernel(
    const IO *__restrict__ q, const IO *__restrict__ k, const IO *__restrict__ v, const float *__restrict__ log_alpha,
    const float *__restrict__ beta, const IO *__restrict__ d_o, const float *__restrict__ dS_T,
    const float *__restrict__ qdq, const float *__restrict__ gate_const, IO *__restrict__ dk_out, IO *__restrict__ dv_out,
    float *__restrict__ dlog_alpha, float *__restrict__ dbeta, float *__restrict__ dS0, GenShape sh)
{
    extern __shared__ float lds[];
    const int dk = sh.dk, dv = sh.dv, dvp = dv + 1;
    float *G = lds, *sq = G + dk * dvp, *skk = sq + dk, *sa = skk + dk, *su = sa + dk, *sdo = su + dv, *sv = sdo + dv;
    float *run = sv + dv;                       // [dk] reverse running sum behind dlog_alpha
    const int tid = threadIdx.x, bh = blockIdx.x;
    const SeqSpan span = seq_span(bh / sh.H, sh.T, sh.cu_seqlens);
    sh.T = span.length;
    const size_t row0 = span.first * sh.H + bh % sh.H;
    const size_t state0 = (size_t)bh * dk * dv;
    const int elems = dk * dv;

    // G holds diag(a_{t+1}) G_{t+1} when token t starts; for the last token that is dS_T
    for (int e = tid; e < elems; e += kGenThreads) G[(e / dv) * dvp + e % dv] = dS_T != nullptr ? dS_T[state0 + e] : 0.f;
    for (int r = tid; r < dk; r += kGenThreads) run[r] = gate_const[(size_t)bh * dk + r];

    for (int t = sh.T - 1; t >= 0; --t) {
        const size_t row = row0 + (size_t)t * sh.H;
        __syncthreads();
        for (int r = tid; r < dk; r += kGenThreads) {
            sq[r] = load_as_float(q + row * dk + r);
            skk[r] = load_as_float(k + row * dk + r);
            sa[r] = expf(log_alpha[row * dk + r]);
        }
        for (int j = tid; j < dv; j += kGenThreads) {
            const float b = beta != nullptr ? beta[row * dv + j] : 1.f;
            const float x = load_as_float(v + row * dv + j);
            sv[j] = x;
            su[j] = b * x;
            sdo[j] = load_as_float(d_o + row * dv + j);
        }
        __syncthreads();
        for (int e = tid; e < elems; e += kGenThreads) {          // G_t = q_t^T do_t + (carried part)
            const int r = e / dv, j = e % dv;
            G[r * dvp + j] = fmaf(sq[r], sdo[j], G[r * dvp + j]);
        }
        __syncthreads();
        for (int r = tid; r < dk; r += kGenThreads) {             // dk_t = u_t G_t^T, and the gate cotangent
            float acc = 0.f;
            for (int j = 0; j < dv; ++j) acc = fmaf(G[r * dvp + j], su[j], acc);
            store_from_float(dk_out + row * dk + r, acc);
            const float total = run[r] + (qdq[row * dk + r] - skk[r] * acc);
            run[r] = total;
            dlog_alpha[row * dk + r] = sa[r] == 0.f ? 0.f : total;
        }
        for (int j = tid; j < dv; j += kGenThreads) {             // du_t = k_t G_t
            float acc = 0.f;
            for (int r = 0; r < dk; ++r) acc = fmaf(G[r * dvp + j], skk[r], acc);
            const float b = beta != nullptr ? beta[row * dv + j] : 1.f;
            store_from_float(dv_out + row * dv + j, b * acc);
            if (dbeta != nullptr) dbeta[row * dv + j] = sv[j] * acc;
        }
        __syncthreads();
        for (int e = tid; e < elems; e += kGenThreads) {          // carried to token t-1: diag(a_t) G_t
            const int r = e / dv;
            G[r * dvp + e % dv] *= sa[r];
        }
    }
    __syncthreads();
    if (dS0 != nullptr)
        for (int e = tid; e < elems; e += kGenThreads) dS0[state0 + e] = G[(e / dv) * dvp + e % dv];
}

template <typename IO>
hipError_t launch_typed(const ScanBwdArgs &a)
{
    const int dk = a.dk_width, dv = a.dv_width;
    const size_t lds = (gen_lds_floats(dk, dv) + dv) * sizeof(float);
    hipError_t err = hipFuncSetAttribute(reinterpret_cast<const void *>(&scan_bwd_generic_dq_kernel<IO>),
                                         hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (err == hipSuccess)
        err = hipFuncSetAttribute(reinterpret_cast<const void *>(&scan_bwd_generic_dkv_kernel<IO>),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (err != hipSuccess) return err;
    const unsigned bh = (unsigned)(a.B * a.H);
    float *qdq = static_cast<float *>(a.workspace);
    float *gate_const = qdq + a.token_rows() * a.H * dk;
    const GenShape sh{a.T, a.H, dk, dv, a.cu_seqlens};
    hipLaunchKernelGGL(scan_bwd_generic_dq_kernel<IO>, dim3(bh), dim3(kGenThreads), lds, a.stream, (const IO *)a.q,
                       (const IO *)a.k, (const IO *)a.v, a.log_alpha, static_cast<const float *>(a.beta), a.S0, (const IO *)a.d_o, a.dS_T, (IO *)a.dq, qdq,
                       gate_const, sh);
    hipLaunchKernelGGL(scan_bwd_generic_dkv_kernel<IO>, dim3(bh), dim3(kGenThreads), lds, a.stream, (const IO *)a.q,
                       (const IO *)a.k, (const IO *)a.v, a.log_alpha, static_cast<const float *>(a.beta), (const IO *)a.d_o, a.dS_T, qdq, gate_const,
                       (IO *)a.dk, (IO *)a.dv, a.dlog_alpha, static_cast<float *>(a.dbeta), a.dS0, sh);
    return hipGetLastError();
}

}  // namespace

bool scan_bwd_generic_supports(int dk, int dv)
{
    return dk >= 1 && dk <= kGenMaxDk && dv >= 1 && (long long)dk * (dv + 1) <= kGenMaxStateFloats;
}

// q .* dq in fp32 for every (token, head, channel) and rowsum(S_T .* dS_T) per (batch, head, channel)
size_t scan_bwd_generic_workspace_bytes(size_t token_rows, int B, int H, int dk)
{
    return (token_rows * H * dk + (size_t)B * H * dk) * sizeof(float);
}

hipError_t launch_scan_bwd_generic(const ScanBwdArgs &a)
{
    if ((long long)a.B * a.H == 0) return hipSuccess;
    return a.io_dtype == RODIMUS_BF16 ? launch_typed<bf16_t>(a) : launch_typed<float>(a);
}

}  // namespace rodimus
