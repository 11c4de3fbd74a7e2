// Generic chunkwise forward scan of the Rodimus recurrence in fp32 on the vector ALUs.
//
// Chunkwise form (paper appendix "Chunkwise Parallel Representation of the Rodimus Block"), per
// (batch, head), with A_t the product of the decay gates from the chunk start through row t and
// G_i the product over the rows after i up to the chunk end:
//     o_t   = (q_t .* A_t) S_prev + sum_{i<=t} P[t,i] (beta_i .* v_i)
//     P[t,i]= sum_n q_t[n] k_i[n] prod_{j=i+1..t} alpha_j[n]          (the masked, decayed scores)
//     S_new = diag(A_C) S_prev + sum_i (k_i .* G_i)^T (beta_i .* v_i)
//
// The appendix writes the pairwise decay as A_t / A_i.  That quotient overflows once a channel has
// decayed by more than the fp32 range inside a chunk and is undefined for alpha = 0, so the scores
// are built from PRODUCTS only, by binary splitting of the chunk: for every power of two h, rows
// whose index has bit h set (second half of an aligned group of 2h rows) pair with the rows of the
// first half of the same group;  prod_{j=i+1..t} alpha_j = (prefix product of t inside its half)
// * (suffix product of i inside its half).  Every (t,i), i<t, belongs to exactly one h, every factor
// is a product of gates (<= 1 for log_alpha <= 0, exactly 0 after alpha = 0) and nothing is ever
// divided.  The prefix/suffix products of level 2h follow from level h with one multiply per row;
// after the last level they are A_t and G_i.
//
// One workgroup (256 threads) owns one (batch, head) and a tile of 64 value columns and walks the
// chunks in order with the dk x 64 state tile in LDS.  This kernel is the any-shape path (fp32 I/O,
// odd sizes, small chunks); the MFMA kernel covers the large bf16 shapes.
#include "internal.h"

namespace rodimus {

namespace {

constexpr int kThreads = 256;
constexpr int kColTile = 64;

__host__ __device__ inline int next_pow2(int x)
{
    int p = 1;
    while (p < x) p <<= 1;
    return p;
}

template <typename IO>
__global__ __launch_bounds__(kThreads) void scan_generic_kernel(
    const IO *__restrict__ q, const IO *__restrict__ k, const IO *__restrict__ v,
    const float *__restrict__ log_alpha, const void *__restrict__ beta, bool beta_preact, const float *S0,
    IO *__restrict__ o, float *S_T, int T, int H, int dk, int dv, int C, const int *__restrict__ cu_seqlens,
    OutputStage stage, const IO *__restrict__ z_g, const IO *__restrict__ z_tau, const float *__restrict__ log_beta_t)
{
    extern __shared__ float lds[];
    const int dkp = dk + 1;                 // padded row stride against bank conflicts
    const int Pp = C + 1;
    float *sq = lds;                        // [C][dkp]  q, later q .* A
    float *sk = sq + C * dkp;               // [C][dkp]  k, later k .* G
    float *pp = sk + C * dkp;               // [C][dkp]  prefix products of alpha inside the current half
    float *sp = pp + C * dkp;               // [C][dkp]  suffix products (rows after i, inside the half)
    float *gv = sp + C * dkp;               // [C][64]   beta .* v
    float *P = gv + C * kColTile;           // [C][C+1]  masked decayed scores
    float *S = P + C * Pp;                  // [dk][64]  state tile
    float *LB = S + dk * kColTile;          // [C][64]   general transition only: running sum of log_beta_t inside the chunk
    const bool general = log_beta_t != nullptr;

    const int tid = threadIdx.x;
    const int bh = blockIdx.x;
    const int b = bh / H, h = bh % H;
    size_t tok0 = (size_t)b * T;          // row of the sequence's first token
    if (cu_seqlens != nullptr) {          // packed variable-length batch; bounds clamped to the tensor (T = total tokens)
        const int first = min(max(cu_seqlens[b], 0), T);
        const int last = min(max(cu_seqlens[b + 1], first), T);
        tok0 = first;
        T = last - first;
    }
    const int j0 = blockIdx.y * kColTile;
    const int ncol = min(kColTile, dv - j0);
    const int Cp = next_pow2(C);
    const size_t state_base = (size_t)bh * dk * dv + j0;
    const float q_scale = 1.f / sqrtf((float)dk);

    for (int e = tid; e < dk * kColTile; e += kThreads) {
        const int r = e / kColTile, c = e % kColTile;
        S[e] = (S0 != nullptr && c < ncol) ? S0[state_base + (size_t)r * dv + c] : 0.f;
    }

    for (int s = 0; s < T; s += C) {
        const int n = min(C, T - s);        // valid rows of this chunk; missing rows act as alpha=1, q=k=v=0

        for (int e = tid; e < C * dk; e += kThreads) {
            const int t = e / dk, r = e % dk;
            const size_t g = ((tok0 + s + t) * H + h) * dk + r;
            const bool ok = t < n;
            float qv = ok ? load_as_float(q + g) : 0.f, kv = ok ? load_as_float(k + g) : 0.f, la = 0.f;
            if (z_tau == nullptr) {
                if (ok) la = log_alpha[g];
                sp[t * dkp + r] = 1.f;
            } else {
                // gated form: the key-side gates from their pre-activations; alpha_hat waits in sp for the key's norm
                float alpha_hat = 0.f;
                if (ok) ddts_channel_gates(load_as_float(z_g + g), load_as_float(z_tau + g), la, alpha_hat);
                sp[t * dkp + r] = alpha_hat;
                qv *= q_scale;
            }
            sq[t * dkp + r] = qv;
            sk[t * dkp + r] = kv;
            pp[t * dkp + r] = expf(la);
        }
        if (z_tau != nullptr) {              // uniform branch: k <- alpha_hat .* k / max(||k||_2, 1e-12)
            __syncthreads();
            for (int t = tid; t < C; t += kThreads) {
                float ss = 0.f;
                for (int r = 0; r < dk; ++r) ss = fmaf(sk[t * dkp + r], sk[t * dkp + r], ss);
                P[t * Pp + t] = inverse_key_norm(ss);            // the diagonal is rewritten below
            }
            __syncthreads();
            for (int e = tid; e < C * dk; e += kThreads) {
                const int t = e / dk, r = e % dk;
                sk[t * dkp + r] *= sp[t * dkp + r] * P[t * Pp + t];
                sp[t * dkp + r] = 1.f;
            }
        }
        for (int e = tid; e < C * kColTile; e += kThreads) {
            const int t = e / kColTile, c = e % kColTile;
            float x = 0.f;
            if (t < n && c < ncol) {
                const size_t g = ((tok0 + s + t) * H + h) * dv + j0 + c;
                x = load_as_float(v + g);
                if (beta != nullptr)      // the value gate: given, or the sigmoid of its pre-activation
                    x *= beta_preact ? sigmoid_f(load_as_float(static_cast<const IO *>(beta) + g))
                                     : static_cast<const float *>(beta)[g];
            }
            gv[e] = x;
        }
        if (general) {
            // General transition of Sec. 3.1.1 (a gate beta_t along the value dimension as well): the pair (write i, read t)
            // carries the factor prod_{j=i+1..t} beta_j = exp(LB_t - LB_i) per column, always <= 1; nothing is divided.
            for (int c = tid; c < kColTile; c += kThreads) {
                float run = 0.f;
                for (int t = 0; t < C; ++t) {
                    // clamped per step: exp(-128) is zero in fp32, and the running sums stay finite for a closed gate
                    if (t < n && c < ncol) run += fmaxf(log_beta_t[((tok0 + s + t) * H + h) * dv + j0 + c], -128.f);
                    LB[t * kColTile + c] = run;
                }
            }
        }
        __syncthreads();

        // diagonal of the scores: a token sees its own write undecayed
        for (int t = tid; t < C; t += kThreads) {
            float acc = 0.f;
            for (int r = 0; r < dk; ++r) acc = fmaf(sq[t * dkp + r], sk[t * dkp + r], acc);
            P[t * Pp + t] = acc;
        }

        for (int hh = 1; hh < Cp; hh <<= 1) {
            // scores of this level: t in the second half, i in the first half of each group of 2*hh rows
            const int npairs = (Cp / (2 * hh)) * hh * hh;
            for (int e = tid; e < npairs; e += kThreads) {
                const int grp = e / (hh * hh), rr = e % (hh * hh);
                const int t = grp * 2 * hh + hh + rr / hh;
                const int i = grp * 2 * hh + rr % hh;
                if (t < C) {
                    float acc = 0.f;
                    for (int r = 0; r < dk; ++r)
                        acc = fmaf(sq[t * dkp + r] * pp[t * dkp + r], sk[i * dkp + r] * sp[i * dkp + r], acc);
                    P[t * Pp + i] = acc;
                }
            }
            __syncthreads();
            // suffix products: first-half rows extend over the whole second half
            for (int e = tid; e < C * dk; e += kThreads) {
                const int i = e / dk, r = e % dk;
                if (!(i & hh)) {
                    const int g = i & ~(2 * hh - 1);
                    if (g + hh < C) sp[i * dkp + r] *= pp[min(g + 2 * hh - 1, C - 1) * dkp + r];
                }
            }
            __syncthreads();
            // prefix products: second-half rows extend back over the whole first half
            for (int e = tid; e < C * dk; e += kThreads) {
                const int t = e / dk, r = e % dk;
                if (t & hh) pp[t * dkp + r] *= pp[((t & ~(2 * hh - 1)) + hh - 1) * dkp + r];
            }
            __syncthreads();
        }

        // pp = A (from the chunk start through the row), sp = G (rows after it to the chunk end)
        for (int e = tid; e < C * dk; e += kThreads) {
            const int t = e / dk, r = e % dk;
            sq[t * dkp + r] *= pp[t * dkp + r];
            sk[t * dkp + r] *= sp[t * dkp + r];
        }
        __syncthreads();

        for (int e = tid; e < n * kColTile; e += kThreads) {
            const int t = e / kColTile, c = e % kColTile;
            float acc = 0.f;
            for (int r = 0; r < dk; ++r) acc = fmaf(sq[t * dkp + r], S[r * kColTile + c], acc);
            if (!general) {
                for (int i = 0; i <= t; ++i) acc = fmaf(P[t * Pp + i], gv[i * kColTile + c], acc);
            } else {
                const float lbt = LB[t * kColTile + c];
                acc *= __expf(lbt);                                  // the entering state has decayed by beta_1 .. beta_t
                for (int i = 0; i <= t; ++i)
                    acc = fmaf(P[t * Pp + i] * __expf(lbt - LB[i * kColTile + c]), gv[i * kColTile + c], acc);
            }
            if (c < ncol) {
                const size_t e = ((tok0 + s + t) * H + h) * dv + j0 + c;
                // output stage of the block, if any: y = (o + d .* x') .* act(z)
                if (stage.x_prime != nullptr)
                    acc = fmaf(stage.d[(size_t)h * dv + j0 + c], load_as_float(static_cast<const IO *>(stage.x_prime) + e), acc);
                if (stage.z_gate != nullptr) acc *= output_gate(load_as_float(static_cast<const IO *>(stage.z_gate) + e), stage.act);
                store_from_float(o + e, acc);
            }
        }
        __syncthreads();

        if (general) {
            // writes decay by the gates of the rows after them up to the chunk end; the state by the whole chunk
            for (int e = tid; e < n * kColTile; e += kThreads) {
                const int c = e % kColTile;
                gv[e] *= __expf(LB[(C - 1) * kColTile + c] - LB[e]);
            }
            __syncthreads();
        }
        for (int e = tid; e < dk * kColTile; e += kThreads) {
            const int r = e / kColTile, c = e % kColTile;
            float acc = pp[(C - 1) * dkp + r] * S[e];
            if (general) acc *= __expf(LB[(C - 1) * kColTile + c]);
            for (int i = 0; i < n; ++i) acc = fmaf(sk[i * dkp + r], gv[i * kColTile + c], acc);
            S[e] = acc;
        }
        __syncthreads();
    }

    if (S_T != nullptr) {
        for (int e = tid; e < dk * kColTile; e += kThreads) {
            const int r = e / kColTile, c = e % kColTile;
            if (c < ncol) S_T[state_base + (size_t)r * dv + c] = S[e];
        }
    }
}

}  // namespace

size_t scan_generic_lds_bytes(int dk, int chunk, bool general)
{
    const size_t floats = (size_t)4 * chunk * (dk + 1) + (size_t)chunk * kColTile + (size_t)chunk * (chunk + 1) +
                          (size_t)dk * kColTile + (general ? (size_t)chunk * kColTile : 0);
    return floats * sizeof(float);
}

template <typename IO>
static hipError_t launch_typed(const ScanArgs &a)
{
    const size_t lds = scan_generic_lds_bytes(a.dk, a.chunk, a.log_beta_t != nullptr);
    hipError_t err = hipFuncSetAttribute(reinterpret_cast<const void *>(&scan_generic_kernel<IO>),
                                         hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (err != hipSuccess) return err;
    dim3 grid((unsigned)(a.B * a.H), (unsigned)((a.dv + kColTile - 1) / kColTile)), block(kThreads);
    hipLaunchKernelGGL(scan_generic_kernel<IO>, grid, block, lds, a.stream, (const IO *)a.q, (const IO *)a.k,
                       (const IO *)a.v, a.log_alpha, a.beta, a.beta_preact, a.S0, (IO *)a.o, a.S_T, a.T, a.H, a.dk, a.dv, a.chunk, a.cu_seqlens, a.stage,
                       (const IO *)a.z_g, (const IO *)a.z_tau, a.log_beta_t);
    return hipGetLastError();
}

hipError_t launch_scan_generic(const ScanArgs &a)
{
    if ((long long)a.B * a.H == 0) return hipSuccess;
    // T == 0 still launches when the final state is wanted: the kernel then copies S0 (or zeros) to S_T.
    if (a.T == 0 && (a.S_T == nullptr || a.S_T == a.S0)) return hipSuccess;
    return a.io_dtype == RODIMUS_BF16 ? launch_typed<bf16_t>(a) : launch_typed<float>(a);
}

}  // namespace rodimus
