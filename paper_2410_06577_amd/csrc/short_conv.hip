// ShortConv of the block (paper Sec. 3.1.3): x'_t = act(bias + sum_j w[:, j] .* x_{t-(W-1)+j}), a causal depthwise
// convolution over time of width W <= 8 per channel, optionally followed by SiLU.  Inputs before the call's first token
// come from `state_in` (the last W-1 inputs of the previous call, oldest first) or are zero; `state_out` receives the
// last W-1 inputs seen so far.
//
// One pass over the tensor, bound by HBM bandwidth: a thread owns 8 adjacent channels (one 16-byte piece of a bf16 row)
// and a run of consecutive tokens, keeps the W-1 previous rows of its channels in registers and slides along the run;
// neighbouring threads own neighbouring pieces, so every load and store of a wavefront is a contiguous 1 KB of a row.
// Only the W-1 rows in front of a run are read twice.  fp32 arithmetic, taps accumulated in the order j = 0 .. W-1.
#include "internal.h"

namespace rodimus {

namespace {

constexpr int kConvThreads = 256;
constexpr int kConvRun = 64;           // tokens per thread (32: 8 % slower, 96: 25 % slower on the layer shape)

template <typename IO> struct Row8;
template <> struct Row8<float> {
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
template <> struct Row8<bf16_t> {
    static __device__ __forceinline__ void load(const bf16_t *p, float (&x)[8])
    {
        // every row is read once (plus W-1 rows per run): non-temporal loads are 12 % faster, non-temporal stores are not
        const uint4 w = __builtin_bit_cast(uint4, __builtin_nontemporal_load(reinterpret_cast<const floatx4_t *>(p)));
        x[0] = bf16_lo(w.x); x[1] = bf16_hi(w.x); x[2] = bf16_lo(w.y); x[3] = bf16_hi(w.y);
        x[4] = bf16_lo(w.z); x[5] = bf16_hi(w.z); x[6] = bf16_lo(w.w); x[7] = bf16_hi(w.w);
    }
    static __device__ __forceinline__ void store(bf16_t *p, const float (&x)[8])
    {
        const uint4 w = {pack_bf16x2(x[0], x[1]), pack_bf16x2(x[2], x[3]), pack_bf16x2(x[4], x[5]), pack_bf16x2(x[6], x[7])};
        *reinterpret_cast<uint4 *>(p) = w;
    }
};

// grid: x = blocks of channel pieces, y = runs of kConvRun tokens (one run when T = 0, so that the state is still
// carried over), z = sequence
template <typename IO, int W>
__global__ __launch_bounds__(kConvThreads) void short_conv_kernel(const IO *__restrict__ x, const float *__restrict__ w,
                                                                  const float *__restrict__ bias, const IO *state_in,
                                                                  IO *__restrict__ y, IO *state_out, int T, int C, int act)
{
    const int piece = blockIdx.x * kConvThreads + threadIdx.x;
    if (piece * 8 >= C) return;
    const int c0 = piece * 8, b = blockIdx.z;
    const int t0 = blockIdx.y * kConvRun, t1 = min(T, t0 + kConvRun);

    float tap[W][8], bs[8];
    {
        float flat[8 * W];            // w[c0 .. c0+7][0 .. W-1] is contiguous
#pragma unroll
        for (int i = 0; i < 2 * W; ++i) {
            const floatx4_t v = *reinterpret_cast<const floatx4_t *>(w + (size_t)c0 * W + 4 * i);
            flat[4 * i] = v[0]; flat[4 * i + 1] = v[1]; flat[4 * i + 2] = v[2]; flat[4 * i + 3] = v[3];
        }
#pragma unroll
        for (int e = 0; e < 8; ++e)
#pragma unroll
            for (int j = 0; j < W; ++j) tap[j][e] = flat[e * W + j];
#pragma unroll
        for (int e = 0; e < 8; ++e) bs[e] = 0.f;
        if (bias != nullptr) Row8<float>::load(bias + c0, bs);
    }

    // the W-1 rows in front of the run, oldest first
    float win[W > 1 ? W - 1 : 1][8];
#pragma unroll
    for (int j = 0; j < W - 1; ++j) {
        const int s = t0 - (W - 1) + j;
#pragma unroll
        for (int e = 0; e < 8; ++e) win[j][e] = 0.f;
        if (s >= 0)
            Row8<IO>::load(x + ((size_t)b * T + s) * C + c0, win[j]);
        else if (state_in != nullptr)
            Row8<IO>::load(state_in + ((size_t)b * (W - 1) + (W - 1 + s)) * C + c0, win[j]);
    }

#pragma unroll 8
    for (int t = t0; t < t1; ++t) {
        float cur[8], acc[8];
        Row8<IO>::load(x + ((size_t)b * T + t) * C + c0, cur);
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            float a = bs[e];
#pragma unroll
            for (int j = 0; j < W - 1; ++j) a = fmaf(tap[j][e], win[j][e], a);
            a = fmaf(tap[W - 1][e], cur[e], a);
            acc[e] = act == RODIMUS_CONV_SILU ? a * sigmoid_f(a) : a;
        }
        Row8<IO>::store(y + ((size_t)b * T + t) * C + c0, acc);
#pragma unroll
        for (int j = 0; j + 1 < W - 1; ++j)
#pragma unroll
            for (int e = 0; e < 8; ++e) win[j][e] = win[j + 1][e];
        if (W > 1) {
#pragma unroll
            for (int e = 0; e < 8; ++e) win[W - 2][e] = cur[e];
        }
    }

    if (state_out != nullptr && t1 == T) {            // the run that ends the sequence holds its last W-1 inputs
#pragma unroll
        for (int j = 0; j < W - 1; ++j) Row8<IO>::store(state_out + ((size_t)b * (W - 1) + j) * C + c0, win[j]);
    }
}

template <typename IO, int W>
hipError_t launch_w(const ShortConvArgs &a)
{
    const int pieces = a.C / 8;
    const int runs = a.T > 0 ? (a.T + kConvRun - 1) / kConvRun : 1;
    hipLaunchKernelGGL((short_conv_kernel<IO, W>), dim3((unsigned)((pieces + kConvThreads - 1) / kConvThreads), (unsigned)runs, (unsigned)a.B),
                       dim3(kConvThreads), 0, a.stream, (const IO *)a.x, a.w, a.bias, (const IO *)a.state_in, (IO *)a.y,
                       (IO *)a.state_out, a.T, a.C, a.act);
    return hipGetLastError();
}

template <typename IO>
hipError_t launch_io(const ShortConvArgs &a)
{
    switch (a.W) {
    case 1: return launch_w<IO, 1>(a);
    case 2: return launch_w<IO, 2>(a);
    case 3: return launch_w<IO, 3>(a);
    case 4: return launch_w<IO, 4>(a);
    case 5: return launch_w<IO, 5>(a);
    case 6: return launch_w<IO, 6>(a);
    case 7: return launch_w<IO, 7>(a);
    case 8: return launch_w<IO, 8>(a);
    default: return hipErrorInvalidValue;
    }
}

}  // namespace

hipError_t launch_short_conv(const ShortConvArgs &a)
{
    if (a.B == 0 || a.C == 0) return hipSuccess;
    if (a.T == 0 && (a.state_out == nullptr || a.state_out == a.state_in || a.W == 1)) return hipSuccess;
    return a.io_dtype == RODIMUS_BF16 ? launch_io<bf16_t>(a) : launch_io<float>(a);
}

}  // namespace rodimus
