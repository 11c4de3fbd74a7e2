// Internal declarations shared by the HIP translation units of librodimus_hip (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "../../include/rodimus.h"

namespace rodimus {

typedef __bf16 bf16_t;
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x4_t __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float floatx2_t __attribute__((ext_vector_type(2)));
typedef float floatx4_t __attribute__((ext_vector_type(4)));
typedef float floatx16_t __attribute__((ext_vector_type(16)));

// bf16 is the upper half of an IEEE float: widening is a shift.
__device__ __forceinline__ float bf16_bits_to_float(uint32_t b) { return __uint_as_float(b << 16); }
__device__ __forceinline__ float bf16_lo(uint32_t packed) { return __uint_as_float(packed << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t packed) { return __uint_as_float(packed & 0xffff0000u); }

// Two floats -> packed bf16 pair, round-to-nearest-even in hardware (v_cvt_pk_bf16_f32); `a` in the low half.
__device__ __forceinline__ uint32_t pack_bf16x2(float a, float b)
{
    floatx2_t f = {a, b};
    bf16x2_t h = __builtin_convertvector(f, bf16x2_t);
    return *reinterpret_cast<uint32_t *>(&h);
}

// 1 / (1 + exp(-z)) with the hardware exponential and reciprocal; exact limits 0 and 1 at -inf / +inf.
__device__ __forceinline__ float sigmoid_f(float z)
{
    const float e = __expf(-fabsf(z));               // in (0, 1]: no overflow
    const float r = __builtin_amdgcn_rcpf(1.f + e);
    return z >= 0.f ? r : e * r;
}

// The same without the branch on the sign: exp(-z) overflows to +inf for z < -88 and 1 / (1 + inf) = 0 is the right
// limit; three instructions shorter, for the wavefronts on the critical path of the matrix-core scan.
__device__ __forceinline__ float sigmoid_short(float z) { return __builtin_amdgcn_rcpf(1.f + __expf(-z)); }

// log(1 + e) for e in [0, 1]; the series where 1 + e would round the information away
__device__ __forceinline__ float log1p_unit(float e)
{
    const float series = e * (1.f - e * (0.5f - e * (1.f / 3.f - 0.25f * e)));     // |error| < e^5 / 5
    return e < 0.015625f ? series : __logf(1.f + e);
}

// The two key-side DDTS gates of one channel (paper Sec. 3.1.2) from their pre-activations, with g = softplus(z_g) and
// tau = sigmoid(z_tau):  log_alpha = -g * tau (the decay gate is exp of it), alpha_hat = g^tau (the input gate folded
// into the key).  Hardware exp, log and reciprocal (about 1 ulp each).
// kShortLog1p: log(1 + e) without the series for small e, and the sigmoid without its branch on the sign.  The absolute error of g stays below 1e-7, its relative error
// grows to ~1e-3 only where g < 1e-4 (no visible effect on the decay; 0.1 % on a key that is then rounded to bf16): for
// the matrix-core scan, where this arithmetic sits on the critical wavefronts.
template <bool kShortLog1p = false>
__device__ __forceinline__ void ddts_channel_gates_full(float z_g, float z_tau, float &g, float &tau, float &log_g, float &alpha_hat)
{
    const float e = __expf(-fabsf(z_g));
    g = fmaxf(z_g, 0.f) + (kShortLog1p ? __logf(1.f + e) : log1p_unit(e));             // softplus
    // log g: for very negative z, g = e^z (1 - e^z / 2 + ...) underflows before its logarithm does
    log_g = z_g < -15.f ? z_g - 0.5f * e : __logf(g);
    tau = kShortLog1p ? sigmoid_short(z_tau) : sigmoid_f(z_tau);
    alpha_hat = __expf(tau * log_g);
}
template <bool kShortLog1p = false>
__device__ __forceinline__ void ddts_channel_gates(float z_g, float z_tau, float &log_alpha, float &alpha_hat)
{
    float g, tau, log_g;
    ddts_channel_gates_full<kShortLog1p>(z_g, z_tau, g, tau, log_g, alpha_hat);
    log_alpha = -g * tau;
}

// 1 / max(||k||_2, 1e-12) from the squared norm: the key normalisation of Sec. 3.1.3
__device__ __forceinline__ float inverse_key_norm(float sum_of_squares) { return 1.f / fmaxf(sqrtf(sum_of_squares), 1e-12f); }

// Element loads/stores templated on the I/O element type (float or bf16_t).
template <typename T> __device__ __forceinline__ float load_as_float(const T *p);
template <> __device__ __forceinline__ float load_as_float<float>(const float *p) { return *p; }
template <> __device__ __forceinline__ float load_as_float<bf16_t>(const bf16_t *p)
{
    return bf16_bits_to_float(*reinterpret_cast<const uint16_t *>(p));
}
template <typename T> __device__ __forceinline__ void store_from_float(T *p, float x);
template <> __device__ __forceinline__ void store_from_float<float>(float *p, float x) { *p = x; }
template <> __device__ __forceinline__ void store_from_float<bf16_t>(bf16_t *p, float x) { *p = (bf16_t)x; }

// Four consecutive elements (pointer must be aligned to 4 elements).
template <typename T> __device__ __forceinline__ floatx4_t load4_as_float(const T *p);
template <> __device__ __forceinline__ floatx4_t load4_as_float<float>(const float *p)
{
    return *reinterpret_cast<const floatx4_t *>(p);
}
template <> __device__ __forceinline__ floatx4_t load4_as_float<bf16_t>(const bf16_t *p)
{
    uint2 u = *reinterpret_cast<const uint2 *>(p);
    floatx4_t r = {bf16_lo(u.x), bf16_hi(u.x), bf16_lo(u.y), bf16_hi(u.y)};
    return r;
}
template <typename T> __device__ __forceinline__ void store4_from_float(T *p, floatx4_t x);
template <> __device__ __forceinline__ void store4_from_float<float>(float *p, floatx4_t x)
{
    *reinterpret_cast<floatx4_t *>(p) = x;
}
template <> __device__ __forceinline__ void store4_from_float<bf16_t>(bf16_t *p, floatx4_t x)
{
    uint2 u = {pack_bf16x2(x[0], x[1]), pack_bf16x2(x[2], x[3])};
    *reinterpret_cast<uint2 *>(p) = u;
}

// ---- MFMA and LDS helpers shared by the scan kernels ---------------------------------------------------
__device__ __forceinline__ floatx4_t mfma_k32(bf16x8_t a, bf16x8_t b, floatx4_t c)
{
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0);
}
// Contraction over the 16 tokens of a tile: each lane supplies 4 of them, the other 4 operand slots are zero.
// (The 16x16x32 form is used on purpose: with the 16x16x16 bf16 instruction this compiler consumed MFMA results
// before they were written.)
__device__ __forceinline__ floatx4_t mfma_k16(uint2 a, uint2 b, floatx4_t c)
{
    const uint4 a8 = {a.x, a.y, 0u, 0u}, b8 = {b.x, b.y, 0u, 0u};
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, a8), __builtin_bit_cast(bf16x8_t, b8), c, 0, 0, 0);
}

// k .* G and beta .* v are MFMA operands with the token as the contraction index, but arrive token-major.  They
// are stored token-major (rows of 64 channels / 128 columns, written 8 bytes at a time) and fetched with the
// transposing LDS read: inside each group of 16 lanes, lane 4j + c supplies the address of 4 consecutive bf16 of
// row j, and lane 4c + e receives element e of the four rows j = 0..3.  So a lane ends up with 4 tokens of one
// channel / column, which is the operand layout, without any 2-byte scatter.
__device__ __forceinline__ uint2 lds_read_transposed(const unsigned char *p)
{
    typedef short short4_t __attribute__((ext_vector_type(4)));
    const short4_t r = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
        (short4_t __attribute__((address_space(3))) *)(p));
    return __builtin_bit_cast(uint2, r);
}

// Output stage of the block (paper Sec. 3.1.3): y = (o + d .* x') .* act(z).  x_prime / z_gate have o's shape and dtype, d is
// fp32 [H, dv]; a NULL x_prime drops the feed-through, a NULL z_gate the output gate.
struct OutputStage {
    const void *x_prime;
    const float *d;
    const void *z_gate;
    int act;                         // RODIMUS_GATE_SIGMOID or RODIMUS_GATE_SILU
    bool any() const { return x_prime != nullptr || z_gate != nullptr; }
};

__device__ __forceinline__ float output_gate(float z, int act)
{
    const float sg = sigmoid_f(z);
    return act == RODIMUS_GATE_SILU ? z * sg : sg;
}

// ---- launchers (host).  Arguments are already validated by the C-ABI layer. -------------------------
// `beta` is the value gate: fp32 values, or (beta_preact) its pre-activation in the I/O dtype, or NULL (all ones).
struct ScanArgs {
    const void *q, *k, *v;
    const float *log_alpha;
    const void *beta;
    bool beta_preact;
    const float *S0;
    void *o;
    float *S_T;
    int B, T, H, dk, dv, chunk;      // with cu_seqlens: B sequences, T = total tokens of the packed batch
    int io_dtype;
    const int *cu_seqlens;           // device, B + 1 entries, or NULL for the dense [B, T, H, .] layout
    OutputStage stage;               // feed-through and output gate applied where o is stored (all NULL: plain o)
    void *workspace;
    size_t workspace_bytes;
    hipStream_t stream;
    // Gated form (both non-NULL): the key-side gates arrive as pre-activations in the I/O dtype, q and k raw; the kernels
    // evaluate log_alpha = -softplus(z_g) sigmoid(z_tau), fold softplus(z_g)^sigmoid(z_tau) / ||k|| into k and 1 / sqrt(dk)
    // into q.  `log_alpha` is then unused.
    const void *z_g = nullptr, *z_tau = nullptr;
    bool gated() const { return z_tau != nullptr; }
    // General transition of Sec. 3.1.1: log of the gate along the value dimension, [tokens, H, dv] fp32 (generic kernel only)
    const float *log_beta_t = nullptr;
};

struct DecodeArgs {
    const void *q, *k, *v;
    const float *log_alpha;
    const void *beta;
    bool beta_preact;
    OutputStage stage;
    float *S;
    void *o;
    int N, H, dk, dv;
    int io_dtype;
    hipStream_t stream;
    const void *z_g = nullptr, *z_tau = nullptr;     // gated form, as in ScanArgs
    bool gated() const { return z_tau != nullptr; }
    const float *log_beta_t = nullptr;               // general transition, [N, H, dv] fp32
};

struct GateArgs {
    const void *z_g, *z_tau, *z_beta, *q, *k;
    float *log_alpha, *beta;
    void *q_out, *k_out;
    long long rows;
    int dk, dv, io_dtype;
    hipStream_t stream;
};

// Backward of the dense scan.  d_o, dq, dk, dv in the I/O dtype; dlog_alpha, dbeta, dS0, dS_T fp32.  With beta_preact
// `beta` holds the pre-activations of the value gate in the I/O dtype and `dbeta` receives their cotangent in that dtype
// (matrix-core kernels only).
struct ScanBwdArgs {
    const void *q, *k, *v;
    const float *log_alpha;
    const void *beta;
    const float *S0;
    const void *d_o;
    const float *dS_T;
    void *dq, *dk, *dv;
    float *dlog_alpha;
    void *dbeta;
    float *dS0;
    int B, T, H, dk_width, dv_width;      // with cu_seqlens: B sequences, T = total tokens of the packed batch
    int io_dtype;
    void *workspace;
    size_t workspace_bytes;
    hipStream_t stream;
    const int *cu_seqlens = nullptr;      // device, B + 1 entries, or NULL for the dense [B, T, H, .] layout
    bool beta_preact = false;
    bool packed_cut = false;              // packed batch: let the kernels cut the sequences into segments (matrix-core kernels)
    size_t token_rows() const { return cu_seqlens != nullptr ? (size_t)T : (size_t)B * T; }
};

// Where sequence b of a batch lives in the [tokens, H, .] tensors: dense (b * T, T), or from the length table of a
// packed batch, clamped to the tensor so that a corrupt table cannot take an access outside it.
struct SeqSpan {
    size_t first;
    int length;
};
__device__ __forceinline__ SeqSpan seq_span(int b, int T, const int *cu_seqlens)
{
    if (cu_seqlens == nullptr) return SeqSpan{(size_t)b * T, T};
    const int lo = min(max(cu_seqlens[b], 0), T);
    const int hi = min(max(cu_seqlens[b + 1], lo), T);
    return SeqSpan{(size_t)lo, hi - lo};
}

// Packed batches: workgroups start in index order, so a long sequence that starts last runs on alone at the end of
// the launch.  With up to kRankedSeqs sequences every workgroup ranks the lengths and takes the sequence whose rank by
// descending length (ties by index) is `rank`; larger batches keep their order (the ranking in every workgroup then
// costs more than the order gains: 128 sequences 371 against 349 us in the forward scan).  Called by every thread of the
// workgroup (two barriers); `scratch` is LDS for nseq ints that nothing else uses until the call returns.
constexpr int kRankedSeqs = 64;
__device__ __forceinline__ int sequence_by_length_rank(const int *cu_seqlens, int nseq, int total_tokens, int rank, int *scratch)
{
    if (nseq > kRankedSeqs) return rank;
    __shared__ int chosen;
    const int tid = threadIdx.x, nthreads = 1 << (31 - __clz((int)blockDim.x));      // a power of two; any further threads only wait
    for (int i = tid; i < nseq; i += (int)blockDim.x) {
        const int first = min(max(cu_seqlens[i], 0), total_tokens);
        scratch[i] = min(max(cu_seqlens[i + 1], first), total_tokens) - first;
    }
    __syncthreads();
    // nthreads / npad threads per candidate sequence (npad = nseq rounded up to a power of two), each counting over a
    // stride of the others; the counts of a candidate's threads (neighbouring lanes) are added by shuffles
    int npad = 8;
    while (npad < nseq) npad *= 2;
    const int per = min(nthreads / npad, 64), cand = tid / per, part = tid % per;
    const int mine = scratch[min(cand, nseq - 1)];
    int before = 0;                                     // sequences that come before cand: longer, or as long with a smaller index
    for (int u = part; u < nseq; u += per) before += (scratch[u] > mine || (scratch[u] == mine && u < cand)) ? 1 : 0;
    for (int step = 1; step < per; step *= 2) before += __shfl_xor(before, step);
    if (cand < nseq && part == 0 && before == rank) chosen = cand;
    __syncthreads();
    return chosen;                                      // (every read of scratch lies before this barrier)
}

// A packed batch cut into segments by the kernels (the lengths live in device memory): with segments of `seg_tokens`
// tokens, sequence b owns max(1, ceil(len_b / seg_tokens)) consecutive slots, counted from the sequences before it.  Finds
// the sequence and segment of `slot` by walking the length table (every entry clamped to the tensor); false if the slot lies
// past the batch's last segment.  The same in every lane.
constexpr int kMaxCutSequences = 256;      // larger packed batches are not cut (they hold enough sequences to fill the chip)
struct PackedSlot {
    int b, j, count;      // sequence, segment of the sequence, segments of the sequence
    int first, len;       // first row and length of the sequence
};
__device__ __forceinline__ bool locate_packed_slot(const int *cu_seqlens, int nseq, int total_tokens, int seg_tokens, int slot, PackedSlot &out)
{
    int before = 0;
    for (int i = 0; i < nseq; ++i) {
        const int first = min(max(cu_seqlens[i], 0), total_tokens);
        const int len = min(max(cu_seqlens[i + 1], first), total_tokens) - first;
        const int count = max(1, (len + seg_tokens - 1) / seg_tokens);
        if (slot < before + count) {
            out = PackedSlot{i, slot - before, count, first, len};
            return true;
        }
        before += count;
    }
    return false;
}
// First slot and number of slots of sequence b (see locate_packed_slot).
__device__ __forceinline__ void packed_sequence_slots(const int *cu_seqlens, int b, int total_tokens, int seg_tokens, int &first_slot, int &count)
{
    first_slot = 0;
    count = 1;
    for (int i = 0; i <= b; ++i) {
        const int first = min(max(cu_seqlens[i], 0), total_tokens);
        const int len = min(max(cu_seqlens[i + 1], first), total_tokens) - first;
        count = max(1, (len + seg_tokens - 1) / seg_tokens);
        if (i < b) first_slot += count;
    }
}

hipError_t launch_scan_bwd(const ScanBwdArgs &a);
hipError_t launch_scan_bwd_generic(const ScanBwdArgs &a);       // any other supported shape: fp32 on the vector ALUs
bool scan_bwd_generic_supports(int dk, int dv);
size_t scan_bwd_generic_workspace_bytes(size_t token_rows, int B, int H, int dk);
bool scan_bwd_supports(int dk, int dv, int io_dtype);
size_t scan_bwd_workspace_bytes(size_t token_rows, int B, int T, int H, int dv, bool packed);
size_t scan_bwd_packed_cut_workspace_bytes(int N, int total_tokens, int H, int dv);     // 0: such a batch is not cut
hipError_t launch_decode_step(const DecodeArgs &a);
hipError_t launch_ddts_gates(const GateArgs &a);
// Backward of the key side of the gate front-end: cotangents of z_g, z_tau and of the raw q, k from those of log_alpha
// (fp32) and of the scaled q and folded k (I/O dtype).  dq may be dq_hat and dk may be dk_hat (updated in place).
struct GateBwdArgs {
    const void *z_g, *z_tau, *k;
    const void *dq_hat, *dk_hat;
    const float *dlog_alpha;
    void *dz_g, *dz_tau, *dq, *dk;
    long long rows;
    int dk_width, io_dtype;
    hipStream_t stream;
};
hipError_t launch_ddts_gates_bwd(const GateBwdArgs &a);

// Causal depthwise convolution over time (ShortConv).  x, y [B,T,C], state_in/out [B,W-1,C] in the I/O dtype.
struct ShortConvArgs {
    const void *x;
    const float *w, *bias;
    const void *state_in;
    void *y, *state_out;
    int B, T, C, W, act, io_dtype;
    hipStream_t stream;
};
hipError_t launch_short_conv(const ShortConvArgs &a);
hipError_t launch_scan_generic(const ScanArgs &a);
size_t scan_generic_lds_bytes(int dk, int chunk, bool general = false);
hipError_t launch_scan_mfma(const ScanArgs &a);
bool scan_mfma_supports(int dk, int dv, int chunk, int io_dtype);
size_t scan_mfma_workspace_bytes(int B, int T, int H, int dv);
// measurement aid: a plain streaming kernel, `reads_per_write` (0, 1, 2 or 4) 16-byte units read per unit written
hipError_t launch_hbm_stream_probe(const void *src, void *dst, size_t units, int reads_per_write, int workgroups, hipStream_t stream);
// packed batch of N sequences cut along the sequences by the kernels; 0: the batch is not cut
size_t scan_mfma_packed_workspace_bytes(int N, int total_tokens, int H, int dv);
// State entering each of nseg sequence segments (seg_tokens a multiple of 64) of a dense bf16 batch with dk = 64:
// slots [nseg][B*H][64][dv] and the segment decays gamma [nseg-1][B*H][64], fp32 (used by the backward pass); beta: fp32
// gate values or, with beta_preact, bf16 pre-activations (then not NULL).  With cu_seqlens: a packed batch of B sequences,
// T tokens in all, cut by the kernels (locate_packed_slot); nseg is the slot bound, slots [nseg][H][64][dv], gamma [nseg][H][64]
hipError_t launch_scan_segment_states(const void *k, const void *v, const float *log_alpha, const void *beta, bool beta_preact, const float *S0,
                                      int B, int T, int H, int dv, int nseg, int seg_tokens, float *slots, float *gamma,
                                      hipStream_t stream, const int *cu_seqlens = nullptr);

}  // namespace rodimus
