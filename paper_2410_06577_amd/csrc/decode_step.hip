// Recurrent decode step of the Rodimus block (paper Sec. 3.1.3): for every sequence and head
//     S' = diag(exp(log_alpha)) S + k^T (beta .* v),    o = q S'
// with S (dk x dv, fp32) updated in place.
//
// The step does 4 flop per state element and moves 8 bytes for it, so it is bound by HBM
// bandwidth: the kernel is a streaming read-modify-write of S.  One workgroup of four
// wavefronts owns one state (one sequence, one head) and a tile of 256 value columns:
// lane l holds columns 4l..4l+3 as one 16-byte vector, so a wavefront touches one
// contiguous 1 KB row segment per instruction; wavefront w takes rows w, w+4, w+8, ...
// All row loads of a batch are issued before the first is used.  The q.S' products are
// accumulated per lane and reduced over the four wavefronts through LDS.
//
// Two variants of the state traffic.  kStream: non-temporal loads and stores, 4 rows in flight per
// wavefront -- the state passes through once and should not displace anything; this is the faster form
// whenever the states of a call exceed the 256 MB last-level cache (5.8 TB/s measured at 512 MiB of state,
// against 5.2 TB/s with ordinary accesses).  Otherwise ordinary accesses with 8 rows in flight: a caller
// that steps the same <= 256 MiB of state again finds part of it in that cache (6.7 TB/s effective at
// 256 MiB, against 5.7 TB/s streamed).
#include "internal.h"

namespace rodimus {

namespace {

constexpr int kDecodeThreads = 256;
constexpr int kDecodeWaves = 4;
constexpr int kDecodeCols = 256;   // value columns per workgroup (64 lanes x 4)
constexpr int kDecodeMaxDk = 256;
constexpr size_t kLastLevelCacheBytes = 256u << 20;

// kGeneral: the general transition of Sec. 3.1.1, S' = (alpha^T beta_t) .* S + k^T (beta_hat .* v), with the value-side
// transition gate given as log_beta_t [N, H, dv] fp32.
template <typename IO, bool kStream, bool kGeneral>
__global__ __launch_bounds__(kDecodeThreads) void decode_step_kernel(
    const IO *__restrict__ q, const IO *__restrict__ k, const IO *__restrict__ v,
    const float *__restrict__ log_alpha, const void *__restrict__ beta, bool beta_preact,
    float *__restrict__ S, IO *__restrict__ o, int dk, int dv, int H, OutputStage stage,
    const IO *__restrict__ z_g, const IO *__restrict__ z_tau, const float *__restrict__ log_beta_t)
{
        constexpr int kRowBatch = kStream ? 4 : 8;      // rows in flight per wavefront (streamed: 2 / 4 / 8 / 16 rows give 5.53 / 5.71 / 5.60 / 5.42 TB/s)
    __shared__ float s_q[kDecodeMaxDk];
    __shared__ float s_k[kDecodeMaxDk];
    __shared__ float s_a[kDecodeMaxDk];
    __shared__ floatx4_t s_red[kDecodeWaves][64];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const size_t state = blockIdx.x;                     // index over (sequence, head)
    const int col = blockIdx.y * kDecodeCols + 4 * lane;
    const bool active = col < dv;

    if (z_tau == nullptr) {
        for (int r = tid; r < dk; r += kDecodeThreads) {
            s_q[r] = load_as_float(q + state * dk + r);
            s_k[r] = load_as_float(k + state * dk + r);
            s_a[r] = expf(log_alpha[state * dk + r]);        // exp(-inf) = 0
        }
    } else {
        // gated form (uniform branch): the key-side gates from their pre-activations, the key normalised, the query scaled.
        // dk <= 256 = one channel per thread.
        __shared__ float s_part[kDecodeWaves];
        const bool own = tid < dk;
        float kr = 0.f, alpha_hat = 0.f;
        if (own) {
            float la;
            ddts_channel_gates(load_as_float(z_g + state * dk + tid), load_as_float(z_tau + state * dk + tid), la, alpha_hat);
            kr = load_as_float(k + state * dk + tid);
            s_a[tid] = expf(la);
            s_q[tid] = load_as_float(q + state * dk + tid) * (1.f / sqrtf((float)dk));
        }
        float ss = kr * kr;
#pragma unroll
        for (int m = 32; m > 0; m >>= 1) ss += __shfl_xor(ss, m);
        if (lane == 0) s_part[wave] = ss;
        __syncthreads();
        const float inv_norm = inverse_key_norm(s_part[0] + s_part[1] + s_part[2] + s_part[3]);
        if (own) s_k[tid] = alpha_hat * kr * inv_norm;
    }

    floatx4_t gv = {0.f, 0.f, 0.f, 0.f};                 // beta .* v for this lane's columns
    if (active) {
        gv = load4_as_float(v + state * dv + col);
        if (beta != nullptr && !beta_preact) {
            gv *= *(static_cast<const floatx4_t *>(beta) + (state * dv + col) / 4);
        } else if (beta != nullptr) {                    // the gate arrives as its pre-activation
            const floatx4_t z = load4_as_float(static_cast<const IO *>(beta) + state * dv + col);
            gv *= floatx4_t{sigmoid_f(z[0]), sigmoid_f(z[1]), sigmoid_f(z[2]), sigmoid_f(z[3])};
        }
    }
    floatx4_t bdec = {1.f, 1.f, 1.f, 1.f};               // transition gate of this lane's columns (general form only)
    if (kGeneral && active) {
        const floatx4_t lb = *reinterpret_cast<const floatx4_t *>(log_beta_t + state * dv + col);
        bdec = floatx4_t{expf(lb[0]), expf(lb[1]), expf(lb[2]), expf(lb[3])};
    }
    __syncthreads();

    float *Sp = S + state * (size_t)dk * dv + col;
    floatx4_t acc = {0.f, 0.f, 0.f, 0.f};

    if (active) {
        for (int r0 = wave; r0 < dk; r0 += kDecodeWaves * kRowBatch) {
            floatx4_t s[kRowBatch];
#pragma unroll
            for (int u = 0; u < kRowBatch; ++u) {
                const int r = r0 + u * kDecodeWaves;
                if (r < dk) {
                    const floatx4_t *p = reinterpret_cast<const floatx4_t *>(Sp + (size_t)r * dv);
                    s[u] = kStream ? __builtin_nontemporal_load(p) : *p;
                }
            }
#pragma unroll
            for (int u = 0; u < kRowBatch; ++u) {
                const int r = r0 + u * kDecodeWaves;
                if (r < dk) {
                    const float a = s_a[r], kr = s_k[r], qr = s_q[r];
                    floatx4_t n;
                    if (kGeneral) {
                        n[0] = fmaf(a * bdec[0], s[u][0], kr * gv[0]);
                        n[1] = fmaf(a * bdec[1], s[u][1], kr * gv[1]);
                        n[2] = fmaf(a * bdec[2], s[u][2], kr * gv[2]);
                        n[3] = fmaf(a * bdec[3], s[u][3], kr * gv[3]);
                    } else {
                        n[0] = fmaf(a, s[u][0], kr * gv[0]);
                        n[1] = fmaf(a, s[u][1], kr * gv[1]);
                        n[2] = fmaf(a, s[u][2], kr * gv[2]);
                        n[3] = fmaf(a, s[u][3], kr * gv[3]);
                    }
                    floatx4_t *p = reinterpret_cast<floatx4_t *>(Sp + (size_t)r * dv);
                    if (kStream) __builtin_nontemporal_store(n, p); else *p = n;
                    acc[0] = fmaf(qr, n[0], acc[0]);
                    acc[1] = fmaf(qr, n[1], acc[1]);
                    acc[2] = fmaf(qr, n[2], acc[2]);
                    acc[3] = fmaf(qr, n[3], acc[3]);
                }
            }
        }
    }

    s_red[wave][lane] = acc;
    __syncthreads();
    if (wave == 0 && active) {
        floatx4_t t = s_red[0][lane];
#pragma unroll
        for (int w = 1; w < kDecodeWaves; ++w) t += s_red[w][lane];
        // output stage of the block, if any: y = (o + d .* x') .* act(z)
        if (stage.x_prime != nullptr) {
            const floatx4_t x = load4_as_float(static_cast<const IO *>(stage.x_prime) + state * dv + col);
            const floatx4_t d = *reinterpret_cast<const floatx4_t *>(stage.d + (state % H) * dv + col);
            t += d * x;
        }
        if (stage.z_gate != nullptr) {
            const floatx4_t z = load4_as_float(static_cast<const IO *>(stage.z_gate) + state * dv + col);
            t *= floatx4_t{output_gate(z[0], stage.act), output_gate(z[1], stage.act), output_gate(z[2], stage.act),
                           output_gate(z[3], stage.act)};
        }
        store4_from_float(o + state * dv + col, t);
    }
}

}  // namespace

hipError_t launch_decode_step(const DecodeArgs &a)
{
    const long long states = (long long)a.N * a.H;
    if (states == 0) return hipSuccess;
    const unsigned col_tiles = (unsigned)((a.dv + kDecodeCols - 1) / kDecodeCols);
    // grid.x is limited to 2^31-1 workgroups; the C-ABI layer has checked N*H against it.
    dim3 grid((unsigned)states, col_tiles), block(kDecodeThreads);
    const bool stream = (size_t)states * a.dk * a.dv * sizeof(float) > kLastLevelCacheBytes;
#define RODIMUS_LAUNCH_DECODE(IO, STREAM, GENERAL)                                                                        \
    hipLaunchKernelGGL((decode_step_kernel<IO, STREAM, GENERAL>), grid, block, 0, a.stream, (const IO *)a.q, (const IO *)a.k, \
                       (const IO *)a.v, a.log_alpha, a.beta, a.beta_preact, a.S, (IO *)a.o, a.dk, a.dv, a.H, a.stage,         \
                       (const IO *)a.z_g, (const IO *)a.z_tau, a.log_beta_t)
#define RODIMUS_LAUNCH_DECODE_IO(IO)                                                                    \
    do {                                                                                                \
        if (a.log_beta_t != nullptr) {                                                                  \
            if (stream) RODIMUS_LAUNCH_DECODE(IO, true, true); else RODIMUS_LAUNCH_DECODE(IO, false, true);   \
        } else {                                                                                        \
            if (stream) RODIMUS_LAUNCH_DECODE(IO, true, false); else RODIMUS_LAUNCH_DECODE(IO, false, false); \
        }                                                                                               \
    } while (0)
    if (a.io_dtype == RODIMUS_BF16) RODIMUS_LAUNCH_DECODE_IO(bf16_t); else RODIMUS_LAUNCH_DECODE_IO(float);
#undef RODIMUS_LAUNCH_DECODE_IO
#undef RODIMUS_LAUNCH_DECODE
    return hipGetLastError();
}

}  // namespace rodimus
