// DDTS gate front-end (paper Sec. 3.1.2, and the pre-processing of q and k in Sec. 3.1.3): from the
// pre-activations of the selection gate, the temperature gate and the value gate, and the raw q and k, produce
// the arguments of the recurrence:
//     g = softplus(z_g), tau = sigmoid(z_tau)
//     log_alpha = -g .* tau                                   (alpha = exp(-g .* tau))
//     k_out     = g^tau .* k / max(||k||_2, 1e-12)            (input gate alpha-hat folded into the normalised key)
//     q_out     = q / sqrt(dk)
//     beta      = sigmoid(z_beta)
// Elementwise apart from the key norm, hence bound by HBM bandwidth: one thread owns 8 consecutive channels of a
// row (a row = one token of one head), the dk/8 lanes of a row reduce the squared norm by butterfly shuffles.
// All arithmetic in fp32 (ddts_channel_gates, shared with the kernels that take the pre-activations directly).
#include "internal.h"

namespace rodimus {

namespace {

constexpr int kGateThreads = 256;

// Every input is read exactly once: the loads are marked non-temporal (measured 3 % faster); the outputs are stored
// normally (non-temporal stores are 25 % slower in this store-dominated kernel).
template <typename IO> struct Vec8;
template <> struct Vec8<float> {
    static __device__ __forceinline__ void load(const float *p, float (&x)[8])
    {
        const floatx4_t a = __builtin_nontemporal_load(reinterpret_cast<const floatx4_t *>(p));
        const floatx4_t b = __builtin_nontemporal_load(reinterpret_cast<const floatx4_t *>(p + 4));
#pragma unroll
        for (int i = 0; i < 4; ++i) { x[i] = a[i]; x[4 + i] = b[i]; }
    }
    static __device__ __forceinline__ void store(float *p, const float (&x)[8])
    {
        *reinterpret_cast<floatx4_t *>(p) = floatx4_t{x[0], x[1], x[2], x[3]};
        *reinterpret_cast<floatx4_t *>(p + 4) = floatx4_t{x[4], x[5], x[6], x[7]};
    }
};
template <> struct Vec8<bf16_t> {
    static __device__ __forceinline__ void load(const bf16_t *p, float (&x)[8])
    {
        const uint4 w = __builtin_bit_cast(uint4, __builtin_nontemporal_load(reinterpret_cast<const floatx4_t *>(p)));
        x[0] = bf16_lo(w.x); x[1] = bf16_hi(w.x); x[2] = bf16_lo(w.y); x[3] = bf16_hi(w.y);
        x[4] = bf16_lo(w.z); x[5] = bf16_hi(w.z); x[6] = bf16_lo(w.w); x[7] = bf16_hi(w.w);
    }
    static __device__ __forceinline__ void store(bf16_t *p, const float (&x)[8])
    {
        uint4 w = {pack_bf16x2(x[0], x[1]), pack_bf16x2(x[2], x[3]), pack_bf16x2(x[4], x[5]), pack_bf16x2(x[6], x[7])};
        *reinterpret_cast<uint4 *>(p) = w;
    }
};

// key side: log_alpha, q_out, k_out.  lanes_per_row = dk / 8 is a power of two <= 64.
template <typename IO>
__global__ __launch_bounds__(kGateThreads) void ddts_key_gates_kernel(
    const IO *__restrict__ z_g, const IO *__restrict__ z_tau, const IO *q, const IO *k,
    float *__restrict__ log_alpha, IO *q_out, IO *k_out, long long rows, int dk, int lanes_per_row)
{
    const long long tid = (long long)blockIdx.x * kGateThreads + threadIdx.x;
    const long long row = tid / lanes_per_row;
    const int piece = (int)(tid % lanes_per_row);
    const bool active = row < rows;                  // inactive lanes still take part in the shuffles
    const size_t off = (size_t)(active ? row : 0) * dk + piece * 8;

    float zg[8], zt[8], qv[8], kv[8];
    Vec8<IO>::load(z_g + off, zg);
    Vec8<IO>::load(z_tau + off, zt);
    Vec8<IO>::load(q + off, qv);
    Vec8<IO>::load(k + off, kv);

    float ss = 0.f;
#pragma unroll
    for (int i = 0; i < 8; ++i) ss = fmaf(kv[i], kv[i], ss);
    for (int m = lanes_per_row >> 1; m > 0; m >>= 1) ss += __shfl_xor(ss, m);     // rows are aligned lane groups
    const float inv_norm = inverse_key_norm(ss);
    const float q_scale = 1.f / sqrtf((float)dk);

    float la[8], qo[8], ko[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        float alpha_hat;
        ddts_channel_gates(zg[i], zt[i], la[i], alpha_hat);
        ko[i] = alpha_hat * kv[i] * inv_norm;                      // g^tau .* k / ||k||
        qo[i] = qv[i] * q_scale;
    }
    if (active) {
        *reinterpret_cast<floatx4_t *>(log_alpha + off) = floatx4_t{la[0], la[1], la[2], la[3]};
        *reinterpret_cast<floatx4_t *>(log_alpha + off + 4) = floatx4_t{la[4], la[5], la[6], la[7]};
        Vec8<IO>::store(q_out + off, qo);
        Vec8<IO>::store(k_out + off, ko);
    }
}

// value side: beta = sigmoid(z_beta), 8 elements per thread
template <typename IO>
__global__ __launch_bounds__(kGateThreads) void ddts_value_gate_kernel(const IO *__restrict__ z_beta, float *__restrict__ beta,
                                                                       size_t n8)
{
    const size_t i = (size_t)blockIdx.x * kGateThreads + threadIdx.x;
    if (i >= n8) return;
    float z[8];
    Vec8<IO>::load(z_beta + i * 8, z);
    *reinterpret_cast<floatx4_t *>(beta + i * 8) = floatx4_t{sigmoid_f(z[0]), sigmoid_f(z[1]), sigmoid_f(z[2]), sigmoid_f(z[3])};
    *reinterpret_cast<floatx4_t *>(beta + i * 8 + 4) = floatx4_t{sigmoid_f(z[4]), sigmoid_f(z[5]), sigmoid_f(z[6]), sigmoid_f(z[7])};
}

// Backward of the key side (reverse mode of ddts_key_gates_kernel), same thread layout.  With g = softplus(z_g),
// tau = sigmoid(z_tau), w = g^tau, n = max(||k||, 1e-12), k_out = w .* k / n, q_out = q / sqrt(dk), log_alpha = -g tau:
//     dq   = dq_hat / sqrt(dk)
//     dk   = dk_hat .* w / n - k (sum_r dk_hat_r w_r k_r) / n^3        (second term only while ||k|| is above the guard)
//     dw   = dk_hat .* k / n
//     dg   = -dlog_alpha tau + dw tau w / g          dtau = -dlog_alpha g + dw w ln g
//     dz_g = dg sigmoid(z_g)                         dz_tau = dtau tau (1 - tau)
// dq / dk may be the buffers dq_hat / dk_hat: every thread reads its eight values before it writes them.
template <typename IO>
__global__ __launch_bounds__(kGateThreads) void ddts_key_gates_bwd_kernel(
    const IO *__restrict__ z_g, const IO *__restrict__ z_tau, const IO *__restrict__ k, const IO *dq_hat, const IO *dk_hat,
    const float *__restrict__ dlog_alpha, IO *__restrict__ dz_g, IO *__restrict__ dz_tau, IO *dq, IO *dk, long long rows,
    int dk_width, int lanes_per_row)
{
    const long long tid = (long long)blockIdx.x * kGateThreads + threadIdx.x;
    const long long row = tid / lanes_per_row;
    const int piece = (int)(tid % lanes_per_row);
    const bool active = row < rows;                  // inactive lanes still take part in the shuffles
    const size_t off = (size_t)(active ? row : 0) * dk_width + piece * 8;

    float zg[8], zt[8], kv[8], dqh[8], dkh[8], dla[8];
    Vec8<IO>::load(z_g + off, zg);
    Vec8<IO>::load(z_tau + off, zt);
    Vec8<IO>::load(k + off, kv);
    Vec8<IO>::load(dq_hat + off, dqh);
    Vec8<IO>::load(dk_hat + off, dkh);
    Vec8<float>::load(dlog_alpha + off, dla);

    float g[8], tau[8], log_g[8], w[8];
    float ss = 0.f, through = 0.f;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        ddts_channel_gates_full(zg[i], zt[i], g[i], tau[i], log_g[i], w[i]);
        ss = fmaf(kv[i], kv[i], ss);
        through = fmaf(dkh[i] * w[i], kv[i], through);
    }
    for (int m = lanes_per_row >> 1; m > 0; m >>= 1) {      // rows are aligned lane groups
        ss += __shfl_xor(ss, m);
        through += __shfl_xor(through, m);
    }
    const float norm = sqrtf(ss);
    const bool guarded = !(norm > 1e-12f);
    const float inv_norm = 1.f / (guarded ? 1e-12f : norm);
    const float pull = guarded ? 0.f : through * inv_norm * inv_norm * inv_norm;
    const float q_scale = 1.f / sqrtf((float)dk_width);

    float o_zg[8], o_zt[8], o_q[8], o_k[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        o_q[i] = dqh[i] * q_scale;
        o_k[i] = dkh[i] * w[i] * inv_norm - kv[i] * pull;
        const float dw = dkh[i] * kv[i] * inv_norm;
        const float w_over_g = g[i] > 0.f ? w[i] / g[i] : 0.f;
        const float dg = -dla[i] * tau[i] + dw * tau[i] * w_over_g;
        const float dtau = -dla[i] * g[i] + (w[i] > 0.f ? dw * w[i] * log_g[i] : 0.f);
        o_zg[i] = dg * sigmoid_f(zg[i]);
        o_zt[i] = dtau * tau[i] * (1.f - tau[i]);
    }
    if (active) {
        Vec8<IO>::store(dz_g + off, o_zg);
        Vec8<IO>::store(dz_tau + off, o_zt);
        Vec8<IO>::store(dq + off, o_q);
        Vec8<IO>::store(dk + off, o_k);
    }
}

template <typename IO>
hipError_t launch_bwd_typed(const GateBwdArgs &a)
{
    if (a.rows == 0) return hipSuccess;
    const int lanes_per_row = a.dk_width / 8;
    const long long threads = a.rows * lanes_per_row;
    hipLaunchKernelGGL(ddts_key_gates_bwd_kernel<IO>, dim3((unsigned)((threads + kGateThreads - 1) / kGateThreads)), dim3(kGateThreads),
                       0, a.stream, (const IO *)a.z_g, (const IO *)a.z_tau, (const IO *)a.k, (const IO *)a.dq_hat, (const IO *)a.dk_hat,
                       a.dlog_alpha, (IO *)a.dz_g, (IO *)a.dz_tau, (IO *)a.dq, (IO *)a.dk, a.rows, a.dk_width, lanes_per_row);
    return hipGetLastError();
}

template <typename IO>
hipError_t launch_typed(const GateArgs &a)
{
    if (a.rows == 0) return hipSuccess;
    const int lanes_per_row = a.dk / 8;
    const long long threads = a.rows * lanes_per_row;
    hipLaunchKernelGGL(ddts_key_gates_kernel<IO>, dim3((unsigned)((threads + kGateThreads - 1) / kGateThreads)), dim3(kGateThreads),
                       0, a.stream, (const IO *)a.z_g, (const IO *)a.z_tau, (const IO *)a.q, (const IO *)a.k, a.log_alpha,
                       (IO *)a.q_out, (IO *)a.k_out, a.rows, a.dk, lanes_per_row);
    if (a.z_beta != nullptr) {
        const size_t n8 = (size_t)a.rows * a.dv / 8;
        hipLaunchKernelGGL(ddts_value_gate_kernel<IO>, dim3((unsigned)((n8 + kGateThreads - 1) / kGateThreads)), dim3(kGateThreads), 0,
                           a.stream, (const IO *)a.z_beta, a.beta, n8);
    }
    return hipGetLastError();
}

}  // namespace

hipError_t launch_ddts_gates(const GateArgs &a)
{
    return a.io_dtype == RODIMUS_BF16 ? launch_typed<bf16_t>(a) : launch_typed<float>(a);
}

hipError_t launch_ddts_gates_bwd(const GateBwdArgs &a)
{
    return a.io_dtype == RODIMUS_BF16 ? launch_bwd_typed<bf16_t>(a) : launch_bwd_typed<float>(a);
}

}  // namespace rodimus
