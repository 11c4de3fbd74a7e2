// Chunkwise forward scan of the Rodimus recurrence on the matrix cores (bf16 MFMA, fp32 accumulate).
// Shape: dk = 64, value columns in tiles of 128, bf16 q/k/v/o.  gfx950 only.
//
// The chunkwise form of the paper's appendix ("Chunkwise Parallel Representation of the Rodimus Block") is
// applied with the state carried every 16 tokens (one MFMA tile); 64 tokens are processed per workgroup
// barrier.  For a tile of rows t = 1..16 with S_prev the state entering it, A_t the product of the decay
// gates from the tile start through row t and G_i the product over the rows after i to the tile end:
//     o_t   = (q_t .* A_t) S_prev + sum_{i<=t} P[t,i] (beta_i .* v_i)
//     P[t,i]= sum_n q_t[n] k_i[n] prod_{j=i+1..t} alpha_j[n]
//     S_new = diag(A_16) S_prev + sum_i (k_i .* G_i)^T (beta_i .* v_i)
// The appendix's quotient A_t / A_i is never formed.  The pairwise decay is built from PRODUCTS of gates by
// binary splitting of the tile: for a power of two h, a row t with bit h set pairs with the rows i of the first
// half of its aligned 2h-block and
//     prod_{j=i+1..t} alpha_j = (prod over t's h-block from its start through t) * (prod over the rows after i
//                               to the end of i's h-block).
// Every pair i < t belongs to exactly one h, all factors are <= 1 for log_alpha <= 0 and exactly 0 after
// alpha = 0, so hard resets and decays beyond the fp32 range are exact.
//
// One workgroup (8 wavefronts) owns one (batch, head) and 128 value columns and walks its tokens in order.
// The wavefronts are specialised and work one chunk apart through double-buffered LDS, with ONE barrier per
// 64 tokens:
//   wavefronts 0-3 ("gate" wavefronts), one 16-row tile each: lane = (row, 16 key channels).  exp of the
//       log-gates, the prefix/suffix products of every split level by DPP across the 16 lanes of a row group,
//       the decayed copies of q and k as bf16 MFMA operands straight from registers, the level scores as
//       masked Gram matrices (MFMA), and for the other half: q .* A, (k .* G)^T, A_16 and P into LDS.
//   wavefronts 4-7 ("state" wavefronts), 32 value columns each: the fp32 state slab (64 x 32) lives in MFMA
//       accumulators for the whole walk; per tile o^T = S^T (q .* A)^T + (beta .* v)^T P^T, the bf16 store of
//       o, S = diag(A_16) S + (k .* G)^T (beta .* v), and the bf16 copy of S that feeds the next tile.
// Global loads are issued one chunk ahead into registers by the wavefront that consumes them.
#include "internal.h"

// Optional cycle counters per wavefront role and loop part (build with -DRODIMUS_PROF; not part of the library's
// interface and not in the shipped build): how the per-chunk clock budgets quoted for this kernel were measured.
#ifdef RODIMUS_PROF
__device__ unsigned long long g_prof[64];
#define PROF_T() clock64()
#define PROF_ADD(slot, t0) do { if (blockIdx.x == 0 && blockIdx.y == 0 && lane == 0) g_prof[slot] += clock64() - (t0); } while (0)
extern "C" int rodimus_debug_read_prof(unsigned long long *out, int reset)
{
    hipError_t e = hipMemcpyFromSymbol(out, HIP_SYMBOL(g_prof), sizeof(unsigned long long) * 64);
    if (reset) { unsigned long long z[64] = {0}; hipMemcpyToSymbol(HIP_SYMBOL(g_prof), z, sizeof(z)); }
    return (int)e;
}
#else
#define PROF_T() 0ull
#define PROF_ADD(slot, t0) do { (void)(t0); } while (0)
#endif

namespace rodimus {

namespace {

constexpr int kK = 64;           // key width
constexpr int kTile = 16;        // rows per state update
constexpr int kChunk = 64;       // tokens per barrier (4 tiles)
constexpr int kColTile = 128;    // value columns per workgroup
constexpr int kThreads = 512;

// ---- LDS map (bytes).  Two buffers (chunk parity) of what the gate wavefronts hand to the state wavefronts.
constexpr int kQnTile = kTile * 128;                 // q .* A,      [16 rows][64 ch] bf16, 16-byte units swizzled by row
constexpr int kKtTile = kTile * 128;                 // k .* G,      [16 rows][64 ch] bf16, 8-byte units placed by lds_key_unit()
constexpr int kPdTile = kTile * 32;                  // P,           [16 t][16 i] bf16
constexpr int kGmTile = kK * 4;                      // A_16,        [64] fp32
constexpr int kOffQn = 0;
constexpr int kOffKt = kOffQn + 4 * kQnTile;
constexpr int kOffPd = kOffKt + 4 * kKtTile;
constexpr int kOffGm = kOffPd + 4 * kPdTile;
constexpr int kBufBytes = kOffGm + 4 * kGmTile;      // 19456
constexpr int kOffVt = 2 * kBufBytes;                // beta .* v, two chunk buffers of [64 t][128 col] bf16, 8-byte units placed by lds_value_unit()
constexpr int kVtBuf = kChunk * 256;
constexpr int kOffOb = kOffVt + 2 * kVtBuf;          // outputs, two chunk buffers of [64 t][128 col] bf16, 16-byte units swizzled by row
constexpr int kObBuf = kChunk * 256;
constexpr int kLdsBytes = kOffOb + 2 * kObBuf;       // 104448

// Where an 8-byte unit lives inside its token row; the XOR with the token index spreads the 32 (reader) or 64
// (writer) lanes of an access over all banks.
//   values: unit (slab, ct, c) = columns 32 slab + 8c + 4ct .. +3 of token row r (row stride 256 bytes)
__device__ __forceinline__ int lds_value_unit(int slab, int ct, int c, int r) { return (c + 4 * ct + 8 * slab) ^ ((r & 7) << 2); }
//   keys: unit (m, par, c) = channels 32m + 8c + 4par .. +3 of token row r of a tile (row stride 128 bytes)
__device__ __forceinline__ int lds_key_unit(int m, int par, int c, int r)
{
    return (c + 4 * par + 8 * m) ^ ((((r >> 1) & 3) << 2) | (((r >> 3) & 1) << 1));
}

// Cross-lane reads inside a row group of 16 lanes (one lane per tile row).
// dpp_any: plain DPP move (quad permute or row shift); lanes without a source read 0, which callers discard.
template <int kCtrl>
__device__ __forceinline__ float dpp_any(float src)
{
    return __int_as_float(__builtin_amdgcn_update_dpp(__float_as_int(src), __float_as_int(src), kCtrl, 0xf, 0xf, true));
}
// row_shift_right: lane n of a 16-lane row reads lane n - kShift of the same row; the first kShift lanes get `fill`
template <int kShift>
__device__ __forceinline__ float row_shift_right(float src, float fill)
{
    return __int_as_float(__builtin_amdgcn_update_dpp(__float_as_int(fill), __float_as_int(src), 0x110 + kShift, 0xf, 0xf, false));
}
// swizzle_lane: every lane reads lane ((lane & kAnd) | kOr) of its 32-lane half
template <int kAnd, int kOr>
__device__ __forceinline__ float swizzle_lane(float src)
{
    return __int_as_float(__builtin_amdgcn_ds_swizzle(__float_as_int(src), kAnd | (kOr << 5)));
}
constexpr int QP(int a, int b, int c, int d) { return a | (b << 2) | (c << 4) | (d << 6); }

struct Geometry {
    const bf16_t *q, *k, *v;
    const float *la;
    const bf16_t *zg, *zt;  // gated form (kGated): pre-activations of the key-side gates instead of la
    const void *beta;       // value gate: fp32 values, or bf16 pre-activations (kZBeta), or null
    bf16_t *o;
    int H, dv;
    size_t tok0;            // row of the sequence's first token in the [tokens, H, .] tensors
    int h, j0;
    int t_end;              // one past the last token this workgroup processes (its segment end, <= sequence length)
};

// =========================================================================================================
// Gate wavefronts
// =========================================================================================================
struct GateLoads {          // one row, 16 channels: 8g..8g+7 and 32+8g..32+8g+7
    uint4 q[2], k[2];
    floatx4_t la[4];        // gated form, until gate_activate(): the bits of z_g (la[0], la[1]) and z_tau (la[2], la[3]), 8 bf16 each
};

// Loads are unconditional (the row index is clamped to the last valid token) so that they stay in flight across
// the barrier; rows at or beyond T are neutralised when consumed (gate_tile: q = k = 0, alpha = 1).
template <bool kSummary, bool kGated>
__device__ __forceinline__ void gate_prefetch(const Geometry &g, int t, int grp, GateLoads &p)
{
    const size_t tok = (g.tok0 + min(t, g.t_end - 1)) * g.H + g.h;
    const bf16_t *qp = g.q + tok * kK + 8 * grp;
    const bf16_t *kp = g.k + tok * kK + 8 * grp;
    if (!kSummary) {
        p.q[0] = *reinterpret_cast<const uint4 *>(qp);
        p.q[1] = *reinterpret_cast<const uint4 *>(qp + 32);
    }
    p.k[0] = *reinterpret_cast<const uint4 *>(kp);
    p.k[1] = *reinterpret_cast<const uint4 *>(kp + 32);
    if (kGated) {
        const bf16_t *gp = g.zg + tok * kK + 8 * grp, *tp = g.zt + tok * kK + 8 * grp;
        p.la[0] = *reinterpret_cast<const floatx4_t *>(gp);
        p.la[1] = *reinterpret_cast<const floatx4_t *>(gp + 32);
        p.la[2] = *reinterpret_cast<const floatx4_t *>(tp);
        p.la[3] = *reinterpret_cast<const floatx4_t *>(tp + 32);
    } else {
        const float *lp = g.la + tok * kK + 8 * grp;
        p.la[0] = *reinterpret_cast<const floatx4_t *>(lp);
        p.la[1] = *reinterpret_cast<const floatx4_t *>(lp + 4);
        p.la[2] = *reinterpret_cast<const floatx4_t *>(lp + 32);
        p.la[3] = *reinterpret_cast<const floatx4_t *>(lp + 36);
    }
}

__device__ __forceinline__ bf16x8_t pack8(const float *x);

__device__ __forceinline__ void unpack_bf16x8(const uint4 &w, float *x)
{
    x[0] = bf16_lo(w.x); x[1] = bf16_hi(w.x); x[2] = bf16_lo(w.y); x[3] = bf16_hi(w.y);
    x[4] = bf16_lo(w.z); x[5] = bf16_hi(w.z); x[6] = bf16_lo(w.w); x[7] = bf16_hi(w.w);
}

// Gated form: turn the loaded pre-activations and raw q, k of one row into what the rest of the gate wavefront expects
// (paper Sec. 3.1.2 and the pre-processing of Sec. 3.1.3): log_alpha = -softplus(z_g) sigmoid(z_tau) in fp32,
// k <- softplus(z_g)^sigmoid(z_tau) .* k / max(||k||_2, 1e-12) and q <- q / sqrt(64), both rounded to bf16 (what a separate
// gate pass would have written; the division by 8 is exact).  The four lanes that share a row (one per channel group)
// add up the squared norm.
template <bool kSummary>
__device__ __forceinline__ void gate_activate(GateLoads &in)
{
    float kf[16], zg[16], zt[16];
    unpack_bf16x8(in.k[0], kf);
    unpack_bf16x8(in.k[1], kf + 8);
    unpack_bf16x8(__builtin_bit_cast(uint4, in.la[0]), zg);
    unpack_bf16x8(__builtin_bit_cast(uint4, in.la[1]), zg + 8);
    unpack_bf16x8(__builtin_bit_cast(uint4, in.la[2]), zt);
    unpack_bf16x8(__builtin_bit_cast(uint4, in.la[3]), zt + 8);
    float ss = 0.f;
#pragma unroll
    for (int c = 0; c < 16; ++c) ss = fmaf(kf[c], kf[c], ss);
    ss += __shfl_xor(ss, 16);
    ss += __shfl_xor(ss, 32);
    const float inv_norm = inverse_key_norm(ss);
    float la[16], kh[16];
#pragma unroll
    for (int c = 0; c < 16; ++c) {
        float alpha_hat;
        ddts_channel_gates<true>(zg[c], zt[c], la[c], alpha_hat);
        kh[c] = alpha_hat * kf[c] * inv_norm;
    }
    in.k[0] = __builtin_bit_cast(uint4, pack8(kh));
    in.k[1] = __builtin_bit_cast(uint4, pack8(kh + 8));
#pragma unroll
    for (int m = 0; m < 4; ++m) in.la[m] = floatx4_t{la[4 * m], la[4 * m + 1], la[4 * m + 2], la[4 * m + 3]};
    if (!kSummary) {
#pragma unroll
        for (int m = 0; m < 2; ++m) {
            float qf[8];
            unpack_bf16x8(in.q[m], qf);
#pragma unroll
            for (int c = 0; c < 8; ++c) qf[c] *= 0.125f;
            in.q[m] = __builtin_bit_cast(uint4, pack8(qf));
        }
    }
}

__device__ __forceinline__ void gate_mask_padding(bool valid, GateLoads &p)
{
    if (!valid) {
        const uint4 z = {0u, 0u, 0u, 0u};
        const floatx4_t zf = {0.f, 0.f, 0.f, 0.f};
        p.q[0] = p.q[1] = p.k[0] = p.k[1] = z;
        p.la[0] = p.la[1] = p.la[2] = p.la[3] = zf;
    }
}

__device__ __forceinline__ bf16x8_t pack8(const float *x)
{
    uint4 w = {pack_bf16x2(x[0], x[1]), pack_bf16x2(x[2], x[3]), pack_bf16x2(x[4], x[5]), pack_bf16x2(x[6], x[7])};
    return __builtin_bit_cast(bf16x8_t, w);
}

// ---- product-only construction of one tile (every split level).  Exact for any gates, including alpha = 0.
// It works on one half of the lane's channels at a time (8 channels = the 8 operand slots of one MFMA), which
// keeps its register footprint small; the two halves add into the same score accumulator.

// scores of one split level from 8 channels: entries (key row m = 4*grp + r, query row n = row) of
// (k .* suffix)(q .* prefix)^T that belong to the level
template <int kLevel>
__device__ __forceinline__ void level_scores(const float (&q)[8], const float (&k)[8], const float (&pre)[8],
                                             const float (&suf)[8], int row, int grp, floatx4_t &acc)
{
    float xq[8], xk[8];
#pragma unroll
    for (int c = 0; c < 8; ++c) {
        xq[c] = q[c] * pre[c];
        xk[c] = k[c] * suf[c];
    }
    const floatx4_t zero = {0.f, 0.f, 0.f, 0.f};
    const floatx4_t d = mfma_k32(pack8(xk), pack8(xq), zero);
    constexpr int h = 1 << kLevel;
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        const int m = 4 * grp + r;
        const bool keep = (row & h) && !(m & h) && ((row >> (kLevel + 1)) == (m >> (kLevel + 1)));
        acc[r] += keep ? d[r] : 0.f;
    }
}

// Channels 32*kHalf + 8grp .. +7 of one tile.
template <bool kSummary, int kHalf>
__device__ __forceinline__ void gate_half_products(unsigned char *buf, int tile, int row, int grp, const GateLoads &in,
                                                   floatx4_t &acc)
{
    float q[8], k[8], a[8];
    {
        const uint32_t qw[4] = {in.q[kHalf].x, in.q[kHalf].y, in.q[kHalf].z, in.q[kHalf].w};
        const uint32_t kw[4] = {in.k[kHalf].x, in.k[kHalf].y, in.k[kHalf].z, in.k[kHalf].w};
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            q[2 * j] = bf16_lo(qw[j]);
            q[2 * j + 1] = bf16_hi(qw[j]);
            k[2 * j] = bf16_lo(kw[j]);
            k[2 * j + 1] = bf16_hi(kw[j]);
            a[j] = __expf(in.la[2 * kHalf][j]);           // exp(-inf) = 0
            a[4 + j] = __expf(in.la[2 * kHalf + 1][j]);
        }
    }
    const bool b0 = row & 1, b1 = row & 2, b2 = row & 4, b3 = row & 8;
    const floatx4_t zero = {0.f, 0.f, 0.f, 0.f};
    if (!kSummary) {
        // undecayed diagonal: a token sees its own write with weight one
        const floatx4_t d = mfma_k32(__builtin_bit_cast(bf16x8_t, in.k[kHalf]), __builtin_bit_cast(bf16x8_t, in.q[kHalf]), zero);
#pragma unroll
        for (int r = 0; r < 4; ++r) acc[r] += (4 * grp + r == row) ? d[r] : 0.f;
    }
    float pre[8], suf[8];         // prefix / suffix products of the current level's blocks
    // h = 1: blocks of one row
#pragma unroll
    for (int c = 0; c < 8; ++c) { pre[c] = a[c]; suf[c] = 1.f; }
    if (!kSummary) level_scores<0>(q, k, pre, suf, row, grp, acc);
    // h = 2: blocks of two rows
#pragma unroll
    for (int c = 0; c < 8; ++c) {
        const float below = dpp_any<QP(0, 0, 2, 2)>(a[c]);     // odd rows: alpha of the row before
        const float above = dpp_any<QP(1, 1, 3, 3)>(a[c]);     // even rows: alpha of the row after
        pre[c] = b0 ? a[c] * below : a[c];
        suf[c] = b0 ? 1.f : above;
    }
    if (!kSummary) level_scores<1>(q, k, pre, suf, row, grp, acc);
    // h = 4: blocks of four rows
#pragma unroll
    for (int c = 0; c < 8; ++c) {
        const float first_pair = dpp_any<QP(1, 1, 1, 1)>(pre[c]);   // product of rows 0,1 of the quad
        const float last_pair = dpp_any<QP(3, 3, 3, 3)>(pre[c]);    // product of rows 2,3 of the quad
        pre[c] = b1 ? pre[c] * first_pair : pre[c];
        suf[c] = b1 ? suf[c] : suf[c] * last_pair;
    }
    if (!kSummary) level_scores<2>(q, k, pre, suf, row, grp, acc);
    // h = 8: blocks of eight rows
#pragma unroll
    for (int c = 0; c < 8; ++c) {
        const float first_quad = swizzle_lane<0x18, 0x03>(pre[c]);  // product of rows 0..3 of the 8-block
        const float last_quad = swizzle_lane<0x18, 0x07>(pre[c]);   // product of rows 4..7 of the 8-block
        pre[c] = b2 ? pre[c] * first_quad : pre[c];
        suf[c] = b2 ? suf[c] : suf[c] * last_quad;
    }
    if (!kSummary) level_scores<3>(q, k, pre, suf, row, grp, acc);
    // h = 16: the whole tile: A_t and G_i
#pragma unroll
    for (int c = 0; c < 8; ++c) {
        const float first_half = swizzle_lane<0x10, 0x07>(pre[c]);  // product of rows 0..7
        const float last_half = swizzle_lane<0x10, 0x0f>(pre[c]);   // product of rows 8..15
        pre[c] = b3 ? pre[c] * first_half : pre[c];
        suf[c] = b3 ? suf[c] : suf[c] * last_half;
    }

    // ---- hand-over to the state wavefronts
    if (!kSummary) {
        float x[8];
#pragma unroll
        for (int c = 0; c < 8; ++c) x[c] = q[c] * pre[c];                      // q .* A
        unsigned char *qn = buf + kOffQn + tile * kQnTile + row * 128;
        *reinterpret_cast<bf16x8_t *>(qn + (((4 * kHalf + grp) ^ (row & 7)) << 4)) = pack8(x);
    }
    {
        // k .* G, channels 32*kHalf + 8grp .. +7 of token `row`: two 8-byte units
        unsigned char *kt = buf + kOffKt + tile * kKtTile + row * 128;
#pragma unroll
        for (int par = 0; par < 2; ++par) {
            const int e = 4 * par;
            const uint2 w = {pack_bf16x2(k[e] * suf[e], k[e + 1] * suf[e + 1]), pack_bf16x2(k[e + 2] * suf[e + 2], k[e + 3] * suf[e + 3])};
            *reinterpret_cast<uint2 *>(kt + (lds_key_unit(kHalf, par, grp, row) << 3)) = w;
        }
    }
    if (row == 15) {              // decay of the whole tile
        float *gm = reinterpret_cast<float *>(buf + kOffGm + tile * kGmTile);
        floatx4_t lo = {pre[0], pre[1], pre[2], pre[3]};
        floatx4_t hi = {pre[4], pre[5], pre[6], pre[7]};
        *reinterpret_cast<floatx4_t *>(gm + 32 * kHalf + 8 * grp) = lo;
        *reinterpret_cast<floatx4_t *>(gm + 32 * kHalf + 8 * grp + 4) = hi;
    }
}

template <bool kSummary>
__device__ __forceinline__ void gate_tile_products(unsigned char *buf, int tile, int row, int grp, const GateLoads &in)
{
    floatx4_t acc = {0.f, 0.f, 0.f, 0.f};
    gate_half_products<kSummary, 0>(buf, tile, row, grp, in, acc);
    gate_half_products<kSummary, 1>(buf, tile, row, grp, in, acc);
    if (!kSummary) {
        // P[t = row][i = 4grp .. 4grp+3]
        uint2 w = {pack_bf16x2(acc[0], acc[1]), pack_bf16x2(acc[2], acc[3])};
        *reinterpret_cast<uint2 *>(buf + kOffPd + tile * kPdTile + row * 32 + grp * 8) = w;
    }
}

// One 16-row tile.  The prefix products A_t of the gates are needed in any case.  When the tile's total decay A_16
// is far from underflow in every channel (the common case), the pairwise decay inside the tile is taken as the
// quotient A_t / A_i of the appendix's parallel form: one version of q (q .* A, which is also the inter-tile
// operand) and one of k (k ./ A), a single masked Gram matrix, and G_i = A_16 / A_i.  Otherwise (a hard reset or
// a very strong decay inside the tile, where 1 / A_i would overflow or divide by zero) the tile falls back to the
// product-only construction above.  The choice is per tile and wavefront-uniform.
constexpr float kSafeTileDecay = 8.2718061e-25f;     // 2^-80: 1 / A_i stays below 2^80, far inside bf16 and fp32 range

// kShiftPrefix picks one of two instruction sequences for the prefix products A_t (same values up to rounding order):
// four doubling steps of DPP row shifts with the identity shifted in (no selects, no LDS-pipe swizzles), or products
// inside blocks of 2, 4, 8, 16 rows.  Measured on the layer workload, same box: the shifts are 1.6 % faster in the
// fp32-beta kernel (224.3 -> 220.7 us) and 1.7 .. 2 % slower in the z_beta and gated kernels (200.6 -> 204.2, 283 -> 289 us),
// so each instance takes the one that is faster for it.
template <bool kSummary, bool kGated, bool kShiftPrefix>
__device__ __forceinline__ void gate_tile(unsigned char *buf, int tile, int row, int grp, GateLoads &in, bool valid)
{
    if (kGated) gate_activate<kSummary>(in);
    if (kSummary) { const uint4 z = {0u, 0u, 0u, 0u}; in.q[0] = in.q[1] = z; }
    gate_mask_padding(valid, in);

    float pre[16];
#pragma unroll
    for (int m = 0; m < 2; ++m)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            pre[8 * m + j] = __expf(in.la[2 * m][j]);           // exp(-inf) = 0
            pre[8 * m + 4 + j] = __expf(in.la[2 * m + 1][j]);
        }
    if (kShiftPrefix) {
#pragma unroll
        for (int c = 0; c < 16; ++c) pre[c] *= row_shift_right<1>(pre[c], 1.f);
#pragma unroll
        for (int c = 0; c < 16; ++c) pre[c] *= row_shift_right<2>(pre[c], 1.f);
#pragma unroll
        for (int c = 0; c < 16; ++c) pre[c] *= row_shift_right<4>(pre[c], 1.f);
#pragma unroll
        for (int c = 0; c < 16; ++c) pre[c] *= row_shift_right<8>(pre[c], 1.f);      // A_t
    } else {
        const bool b0 = row & 1, b1 = row & 2, b2 = row & 4, b3 = row & 8;
        // prefix products inside blocks of 2, 4, 8, 16 rows
#pragma unroll
        for (int c = 0; c < 16; ++c) {
            const float x = pre[c] * dpp_any<QP(0, 0, 2, 2)>(pre[c]);
            pre[c] = b0 ? x : pre[c];
        }
#pragma unroll
        for (int c = 0; c < 16; ++c) {
            const float x = pre[c] * dpp_any<QP(1, 1, 1, 1)>(pre[c]);
            pre[c] = b1 ? x : pre[c];
        }
        float t[16];
#pragma unroll
        for (int c = 0; c < 16; ++c) t[c] = swizzle_lane<0x18, 0x03>(pre[c]);
#pragma unroll
        for (int c = 0; c < 16; ++c) pre[c] = b2 ? pre[c] * t[c] : pre[c];
#pragma unroll
        for (int c = 0; c < 16; ++c) t[c] = swizzle_lane<0x10, 0x07>(pre[c]);
#pragma unroll
        for (int c = 0; c < 16; ++c) pre[c] = b3 ? pre[c] * t[c] : pre[c];      // A_t
    }
    float total[16];
#pragma unroll
    for (int c = 0; c < 16; ++c) total[c] = swizzle_lane<0x10, 0x0f>(pre[c]);    // A_16 (row 15 of the tile)

    bool weak = true;
#pragma unroll
    for (int c = 0; c < 16; ++c) weak = weak && (total[c] >= kSafeTileDecay);     // false for 0 and NaN as well
    if (__any(!weak)) {
        gate_tile_products<kSummary>(buf, tile, row, grp, in);
        return;
    }

    float k[16];
#pragma unroll
    for (int m = 0; m < 2; ++m) {
        const uint32_t kw[4] = {in.k[m].x, in.k[m].y, in.k[m].z, in.k[m].w};
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            k[8 * m + 2 * j] = bf16_lo(kw[j]) * __builtin_amdgcn_rcpf(pre[8 * m + 2 * j]);           // k ./ A
            k[8 * m + 2 * j + 1] = bf16_hi(kw[j]) * __builtin_amdgcn_rcpf(pre[8 * m + 2 * j + 1]);
        }
    }
    if (!kSummary) {
        float q[16];
#pragma unroll
        for (int m = 0; m < 2; ++m) {
            const uint32_t qw[4] = {in.q[m].x, in.q[m].y, in.q[m].z, in.q[m].w};
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                q[8 * m + 2 * j] = bf16_lo(qw[j]) * pre[8 * m + 2 * j];                               // q .* A
                q[8 * m + 2 * j + 1] = bf16_hi(qw[j]) * pre[8 * m + 2 * j + 1];
            }
        }
        const bf16x8_t qa0 = pack8(q), qa1 = pack8(q + 8);
        floatx4_t d = {0.f, 0.f, 0.f, 0.f};
        d = mfma_k32(pack8(k), qa0, d);
        d = mfma_k32(pack8(k + 8), qa1, d);
        unsigned char *qn = buf + kOffQn + tile * kQnTile + row * 128;
        *reinterpret_cast<bf16x8_t *>(qn + (((0 + grp) ^ (row & 7)) << 4)) = qa0;
        *reinterpret_cast<bf16x8_t *>(qn + (((4 + grp) ^ (row & 7)) << 4)) = qa1;
        // P[t = row][i = 4grp .. 4grp+3], keys up to and including the query row
        const int i0 = 4 * grp;
        uint2 w = {pack_bf16x2(i0 <= row ? d[0] : 0.f, i0 + 1 <= row ? d[1] : 0.f),
                   pack_bf16x2(i0 + 2 <= row ? d[2] : 0.f, i0 + 3 <= row ? d[3] : 0.f)};
        *reinterpret_cast<uint2 *>(buf + kOffPd + tile * kPdTile + row * 32 + grp * 8) = w;
    }
    {
        // k .* G with G_i = A_16 / A_i; same LDS placement as in gate_half_products
        unsigned char *kt = buf + kOffKt + tile * kKtTile + row * 128;
#pragma unroll
        for (int m = 0; m < 2; ++m)
#pragma unroll
            for (int par = 0; par < 2; ++par) {
                const int c = 8 * m + 4 * par;
                const uint2 w = {pack_bf16x2(k[c] * total[c], k[c + 1] * total[c + 1]),
                                 pack_bf16x2(k[c + 2] * total[c + 2], k[c + 3] * total[c + 3])};
                *reinterpret_cast<uint2 *>(kt + (lds_key_unit(m, par, grp, row) << 3)) = w;
            }
    }
    if (row == 15) {              // decay of the whole tile
        float *gm = reinterpret_cast<float *>(buf + kOffGm + tile * kGmTile);
#pragma unroll
        for (int m = 0; m < 2; ++m) {
            floatx4_t lo = {pre[8 * m], pre[8 * m + 1], pre[8 * m + 2], pre[8 * m + 3]};
            floatx4_t hi = {pre[8 * m + 4], pre[8 * m + 5], pre[8 * m + 6], pre[8 * m + 7]};
            *reinterpret_cast<floatx4_t *>(gm + 32 * m + 8 * grp) = lo;
            *reinterpret_cast<floatx4_t *>(gm + 32 * m + 8 * grp + 4) = hi;
        }
    }
}

// =========================================================================================================
// State wavefronts
// =========================================================================================================
// State wavefront `w` fetches tile w of every chunk for ALL 128 columns of the workgroup (whole 256-byte rows of v,
// 512-byte rows of beta: long contiguous pieces are what HBM delivers at full rate) and stages beta .* v for
// the four state wavefronts.  Lane = (row 4u + lane/16 for u = 0..3, columns 8(lane%16) .. +7).
// The value gate arrives as fp32 values (kZBeta = false; `has_beta` false: all ones) or as bf16 pre-activations
// whose sigmoid is taken here (kZBeta = true; half the bytes, two transcendentals per element).
// v, the value gate and o are touched exactly once by exactly one workgroup: their loads and stores are marked
// non-temporal so that they do not displace q, k and log_alpha, which the workgroups of the other column tiles of
// the same (batch, head) read again from the cache.
__device__ __forceinline__ uint4 load_streaming(const bf16_t *p)
{
    return __builtin_bit_cast(uint4, __builtin_nontemporal_load(reinterpret_cast<const floatx4_t *>(p)));
}

struct StateLoads {
    uint4 v[4];
    floatx4_t beta[4][2];
    uint4 zbeta[4];
};

template <bool kZBeta>
__device__ __forceinline__ void state_prefetch(const Geometry &g, int s, int tile, int lane, bool has_beta, StateLoads &p)
{
    const int rsub = lane >> 4, piece = lane & 15;
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        const int t = min(s + 16 * tile + 4 * u + rsub, g.t_end - 1);   // clamped: padded rows are zeroed in stage_values
        const size_t off = ((g.tok0 + t) * g.H + g.h) * g.dv + g.j0 + 8 * piece;
        p.v[u] = load_streaming(g.v + off);
        if (kZBeta) {
            p.zbeta[u] = load_streaming(static_cast<const bf16_t *>(g.beta) + off);
        } else if (has_beta) {
            p.beta[u][0] = __builtin_nontemporal_load(reinterpret_cast<const floatx4_t *>(static_cast<const float *>(g.beta) + off));
            p.beta[u][1] = __builtin_nontemporal_load(reinterpret_cast<const floatx4_t *>(static_cast<const float *>(g.beta) + off + 4));
        }
    }
}

// beta .* v of one tile, rounded to bf16, into the chunk buffer `vt` (token-major, see lds_value_unit).  The lane's
// 8 columns 8*piece .. +7 are the units (slab = piece/4, c = piece%4, ct = 0 and 1) of its token row.
template <bool kZBeta>
__device__ __forceinline__ void stage_values(unsigned char *vt, int tile, int lane, bool has_beta, const StateLoads &p, int s, int t_end)
{
    const int rsub = lane >> 4, piece = lane & 15;
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        const int tok = 4 * u + rsub;
        const bool valid = s + 16 * tile + tok < t_end;
        const uint32_t w[4] = {valid ? p.v[u].x : 0u, valid ? p.v[u].y : 0u, valid ? p.v[u].z : 0u, valid ? p.v[u].w : 0u};
        float gv[8];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            gv[2 * j] = bf16_lo(w[j]);
            gv[2 * j + 1] = bf16_hi(w[j]);
        }
        if (kZBeta) {
            const uint32_t z[4] = {p.zbeta[u].x, p.zbeta[u].y, p.zbeta[u].z, p.zbeta[u].w};
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                gv[2 * j] *= sigmoid_short(bf16_lo(z[j]));
                gv[2 * j + 1] *= sigmoid_short(bf16_hi(z[j]));
            }
        } else if (has_beta) {
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                gv[j] *= p.beta[u][0][j];
                gv[4 + j] *= p.beta[u][1][j];
            }
        }
        unsigned char *row = vt + (16 * tile + tok) * 256;
        const int unit = lds_value_unit(piece >> 2, 0, piece & 3, tok);
        const uint2 lo = {pack_bf16x2(gv[0], gv[1]), pack_bf16x2(gv[2], gv[3])};
        const uint2 hi = {pack_bf16x2(gv[4], gv[5]), pack_bf16x2(gv[6], gv[7])};
        *reinterpret_cast<uint2 *>(row + (unit << 3)) = lo;
        *reinterpret_cast<uint2 *>(row + ((unit ^ 4) << 3)) = hi;        // ct = 1
    }
}

// Outputs of a finished chunk: LDS -> global, whole 256-byte rows.  Done by the gate wavefronts (they have slack),
// wavefront w taking rows 16w .. 16w+15.
__device__ __forceinline__ void store_outputs(const Geometry &g, const unsigned char *ob, int s, int wave, int lane)
{
    const int rsub = lane >> 4, unit = lane & 15;
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        const int row = 16 * wave + 4 * u + rsub;
        const uint4 w = *reinterpret_cast<const uint4 *>(ob + row * 256 + ((unit ^ (row & 15)) << 4));
        const int t = s + row;
        if (t < g.t_end)
            __builtin_nontemporal_store(__builtin_bit_cast(floatx4_t, w),
                                        reinterpret_cast<floatx4_t *>(g.o + ((g.tok0 + t) * g.H + g.h) * g.dv + g.j0 + 8 * unit));
    }
}

struct StateSlab {
    floatx4_t S[4][2];      // [row tile kt][column tile ct]: lane (n, grp) holds rows 4grp..4grp+3 of the tile, column n
    bf16x8_t Sa[2][2];      // bf16 copy as MFMA operand: [ct][k half]
};
// Row (kt, mu) of the slab is key channel 32(kt/2) + 8(mu/4) + 4(kt%2) + mu%4, so that the 8 operand slots of a
// lane (rows 4grp..4grp+3 of tiles 2m and 2m+1) are the 8 consecutive channels 32m + 8grp .. +7: the same
// channels a 16-byte read of a row of q .* A delivers.
__device__ __forceinline__ int slab_channel(int kt, int mu) { return 32 * (kt >> 1) + 8 * (mu >> 2) + 4 * (kt & 1) + (mu & 3); }
// Column index n of column tile ct is value column 8(n/4) + 4ct + n%4 of the slab: a lane's 2 x 4 outputs are 8
// consecutive columns, one 16-byte store.
__device__ __forceinline__ int slab_column(int ct, int n) { return 8 * (n >> 2) + 4 * ct + (n & 3); }

__device__ __forceinline__ void refresh_operands(StateSlab &st)
{
#pragma unroll
    for (int ct = 0; ct < 2; ++ct)
#pragma unroll
        for (int m = 0; m < 2; ++m) {
            const floatx4_t lo = st.S[2 * m][ct], hi = st.S[2 * m + 1][ct];
            uint4 w = {pack_bf16x2(lo[0], lo[1]), pack_bf16x2(lo[2], lo[3]), pack_bf16x2(hi[0], hi[1]), pack_bf16x2(hi[2], hi[3])};
            st.Sa[ct][m] = __builtin_bit_cast(bf16x8_t, w);
        }
}

struct TileOperands {       // what one tile of the state recurrence reads from LDS
    bf16x8_t qb[2];         // rows of q .* A
    uint2 pb;               // row of P
    uint2 va[2], ka[4];     // (beta .* v)^T and (k .* G)^T
    floatx4_t dec[4];       // A_16 for this lane's state rows
};

template <bool kSummary>
__device__ __forceinline__ void load_tile_operands(const unsigned char *buf, const unsigned char *vt, int tile, int slab, int n,
                                                   int grp, TileOperands &op)
{
    // transposing reads: this lane supplies the address of token row 4grp + j, unit c, with n = 4j + c
    const int j = n >> 2, c = n & 3, r = 4 * grp + j;
    if (!kSummary) {
        const unsigned char *qn = buf + kOffQn + tile * kQnTile + n * 128;
        op.qb[0] = *reinterpret_cast<const bf16x8_t *>(qn + (((0 + grp) ^ (n & 7)) << 4));
        op.qb[1] = *reinterpret_cast<const bf16x8_t *>(qn + (((4 + grp) ^ (n & 7)) << 4));
        op.pb = *reinterpret_cast<const uint2 *>(buf + kOffPd + tile * kPdTile + n * 32 + grp * 8);
    }
#pragma unroll
    for (int ct = 0; ct < 2; ++ct)
        op.va[ct] = lds_read_transposed(vt + (16 * tile + r) * 256 + (lds_value_unit(slab, ct, c, r) << 3));
    const float *gm = reinterpret_cast<const float *>(buf + kOffGm + tile * kGmTile);
#pragma unroll
    for (int kt = 0; kt < 4; ++kt) {
        op.ka[kt] = lds_read_transposed(buf + kOffKt + tile * kKtTile + r * 128 + (lds_key_unit(kt >> 1, kt & 1, c, r) << 3));
        op.dec[kt] = *reinterpret_cast<const floatx4_t *>(gm + slab_channel(kt, 4 * grp));
    }
}

// One chunk (4 tiles) of the state recurrence and the outputs for this wavefront's 32 columns.  The LDS operands
// of tile i+1 are requested before tile i is computed.
template <bool kSummary>
__device__ __forceinline__ void state_chunk(const unsigned char *buf, const unsigned char *vt, unsigned char *ob,
                                            int slab, int n, int grp, StateSlab &st, floatx4_t (&decay)[4])
{
    TileOperands ops[2];
    load_tile_operands<kSummary>(buf, vt, 0, slab, n, grp, ops[0]);
#pragma unroll
    for (int tile = 0; tile < 4; ++tile) {
        if (tile + 1 < 4) load_tile_operands<kSummary>(buf, vt, tile + 1, slab, n, grp, ops[(tile + 1) & 1]);
        const TileOperands &op = ops[tile & 1];

        // o^T[column][t] = S^T (q .* A)^T + (beta .* v)^T P^T
        floatx4_t O[2];
        if (!kSummary) {
#pragma unroll
            for (int ct = 0; ct < 2; ++ct) {
                floatx4_t acc = {0.f, 0.f, 0.f, 0.f};
                acc = mfma_k32(st.Sa[ct][0], op.qb[0], acc);
                acc = mfma_k32(st.Sa[ct][1], op.qb[1], acc);
                O[ct] = mfma_k16(op.va[ct], op.pb, acc);
            }
        } else {
            // summary pass: only the segment's decay and state increment are wanted
#pragma unroll
            for (int kt = 0; kt < 4; ++kt) decay[kt] *= op.dec[kt];
        }
        // S = diag(A_16) S + (k .* G)^T (beta .* v)
#pragma unroll
        for (int kt = 0; kt < 4; ++kt) {
#pragma unroll
            for (int ct = 0; ct < 2; ++ct) {
                floatx4_t x = st.S[kt][ct];
                x[0] *= op.dec[kt][0]; x[1] *= op.dec[kt][1]; x[2] *= op.dec[kt][2]; x[3] *= op.dec[kt][3];
                st.S[kt][ct] = mfma_k16(op.ka[kt], op.va[ct], x);
            }
        }
        if (!kSummary) {
            // row 16tile + n of the chunk's output buffer, columns 32slab + 8grp .. +7 (16-byte unit 4slab + grp)
            uint4 w = {pack_bf16x2(O[0][0], O[0][1]), pack_bf16x2(O[0][2], O[0][3]),
                       pack_bf16x2(O[1][0], O[1][1]), pack_bf16x2(O[1][2], O[1][3])};
            *reinterpret_cast<uint4 *>(ob + (16 * tile + n) * 256 + (((4 * slab + grp) ^ n) << 4)) = w;
            refresh_operands(st);
        }
    }
}

// Workspace of a sequence-split call: `nseg` state slots [seg][B*H][64][dv] fp32 followed by the segment decays
// [nseg-1][B*H][64] fp32.  Slot 0 receives the initial state, slot s > 0 first the state increment of segment s-1
// (summary pass), then the state entering segment s (segment_state_scan_kernel), which the main pass reads.
struct SegmentPlan {
    int nseg;              // 1: no split, no workspace
    int seg_tokens;        // tokens per segment, a multiple of 64
    float *slots;
    float *gamma;
};

// kSummary = false: the scan proper over this workgroup's segment (blockIdx.z), reading its entering state.
// kSummary = true : same walk from a zero state without q, scores or outputs; leaves the segment's state
//                   increment in slot seg+1 and the segment's total decay in gamma[seg].
// kZBeta: `beta` holds bf16 pre-activations of the value gate instead of fp32 gate values (and is not NULL).
// kGated: `log_alpha` holds the bf16 pre-activations z_g and `z_tau` those of the temperature gate; q and k are raw.
template <bool kSummary, bool kZBeta, bool kGated>
__global__ __launch_bounds__(kThreads) void scan_mfma_kernel(
    const bf16_t *__restrict__ q, const bf16_t *__restrict__ k, const bf16_t *__restrict__ v,
    const void *__restrict__ log_alpha, const bf16_t *__restrict__ z_tau, const void *__restrict__ beta, const float *S0,
    bf16_t *__restrict__ o, float *S_T, int T, int H, int dv, SegmentPlan plan, const int *__restrict__ cu_seqlens,
    int total_tokens, int total_seqs)
{
    extern __shared__ __align__(16) unsigned char lds[];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int n = lane & 15, grp = lane >> 4;
    int bh = blockIdx.x, col_tile = blockIdx.y;
    const int seg = blockIdx.z;
    const int BH = gridDim.x;
    const bool has_beta = beta != nullptr;
    if (!kSummary && cu_seqlens == nullptr && gridDim.y == 1 && gridDim.z == 1 && dv > kColTile) {
        // Dense batch with more workgroups than compute units, launched flat: workgroups go round-robin over the eight XCDs
        // (each with its own L2), so in every run of 8 * col_tiles workgroups the column tiles of a (batch, head) are 8
        // apart: on the same XCD and started together, they share q, k and the gates in its L2.
        const int col_tiles = dv / kColTile;
        col_tile = (blockIdx.x / 8) % col_tiles;
        bh = (blockIdx.x / (8 * col_tiles)) * 8 + blockIdx.x % 8;
        if (bh >= total_seqs * H) return;                   // the grid is rounded up to whole runs
    }
    if (!kSummary && cu_seqlens != nullptr) {
        // Packed batch, launched as a flat grid: the column tiles of one (sequence, head) are neighbours in dispatch order
        // (they read the same q, k and gates while those are in the cache), and the workgroups take the sequences by
        // descending length (small batches).
        const int col_tiles = dv / kColTile, nseq = (int)(gridDim.x / (unsigned)(col_tiles * H));
        col_tile = blockIdx.x % col_tiles;
        const int slot = blockIdx.x / col_tiles, rank = slot / H;
        const int b = sequence_by_length_rank(cu_seqlens, nseq, total_tokens, rank, reinterpret_cast<int *>(lds));   // the dynamic LDS is free until the walk starts
        bh = b * H + slot % H;
    }

    Geometry g;
    g.q = q; g.k = k; g.v = v; g.beta = beta; g.o = o;
    g.la = kGated ? nullptr : static_cast<const float *>(log_alpha);
    g.zg = kGated ? static_cast<const bf16_t *>(log_alpha) : nullptr;
    g.zt = z_tau;
    g.H = H; g.dv = dv;
    g.h = bh % H; g.j0 = col_tile * kColTile;
    g.tok0 = (size_t)(bh / H) * T;
    if (cu_seqlens != nullptr) {
        // packed variable-length batch: sequence bh / H owns the token rows [cu[b], cu[b+1]); the bounds are clamped
        // to the tensor so that a corrupt table cannot take an access outside it
        const int first = min(max(cu_seqlens[bh / H], 0), total_tokens);
        const int last = min(max(cu_seqlens[bh / H + 1], first), total_tokens);
        g.tok0 = first;
        T = last - first;
    }
    const int t_begin = seg * plan.seg_tokens;
    g.t_end = min(T, t_begin + plan.seg_tokens);

    const int nchunks = (g.t_end - t_begin + kChunk - 1) / kChunk;
    const size_t slot_elems = (size_t)BH * kK * dv;

    if (wave < 4) {
        // ------------------------------------------------------------------ gate wavefront, tile = wave
        constexpr bool kShiftPrefix = !kSummary && !kZBeta && !kGated;      // see gate_tile
        GateLoads even, odd;      // loads of even / odd chunks: no register copies between iterations
        const int row0 = t_begin + 16 * wave + n;
        if (nchunks > 0) gate_prefetch<kSummary, kGated>(g, row0, grp, even);
        // Iteration `it`: store the outputs of chunk it-2 (finished by the state wavefronts in iteration it-1), then
        // build chunk it.  nchunks + 2 iterations, one barrier each, for both kinds of wavefront.
        for (int it = 0;;) {
            unsigned long long t0 = PROF_T();
            if (!kSummary && it >= 2) store_outputs(g, lds + kOffOb, t_begin + (it - 2) * kChunk, wave, lane);
            if (it < nchunks) {
                gate_prefetch<kSummary, kGated>(g, row0 + (it + 1) * kChunk, grp, odd);   // unconditional (clamped): keeps the wait counts exact
                gate_tile<kSummary, kGated, kShiftPrefix>(lds, wave, n, grp, even, row0 + it * kChunk < g.t_end);
            }
            PROF_ADD(wave * 2, t0);
            t0 = PROF_T();
            __syncthreads();
            PROF_ADD(wave * 2 + 1, t0);
            if (++it > nchunks + 1) break;
            t0 = PROF_T();
            if (!kSummary && it >= 2) store_outputs(g, lds + kOffOb + kObBuf, t_begin + (it - 2) * kChunk, wave, lane);
            if (it < nchunks) {
                gate_prefetch<kSummary, kGated>(g, row0 + (it + 1) * kChunk, grp, even);
                gate_tile<kSummary, kGated, kShiftPrefix>(lds + kBufBytes, wave, n, grp, odd, row0 + it * kChunk < g.t_end);
            }
            PROF_ADD(wave * 2, t0);
            t0 = PROF_T();
            __syncthreads();
            PROF_ADD(wave * 2 + 1, t0);
            if (++it > nchunks + 1) break;
        }
    } else {
        // ------------------------------------------------------------------ state wavefront, slab = wave - 4
        const int slab = wave - 4;
        StateSlab st;
        const size_t state_base = (size_t)bh * kK * dv + g.j0 + 32 * slab;
        // entering state: zero (summary), the caller's S0 (no split), or this segment's workspace slot.  The state is read
        // once here and written once at the end: streaming accesses (layer workload 225 -> 221 us, gated form 288 -> 277 us)
        const float *S_in = kSummary ? nullptr : (plan.nseg > 1 ? plan.slots + seg * slot_elems : S0);
#pragma unroll
        for (int kt = 0; kt < 4; ++kt)
#pragma unroll
            for (int ct = 0; ct < 2; ++ct)
#pragma unroll
                for (int r = 0; r < 4; ++r)
                    st.S[kt][ct][r] = (S_in != nullptr)
                                          ? __builtin_nontemporal_load(S_in + state_base + (size_t)slab_channel(kt, 4 * grp + r) * dv + slab_column(ct, n))
                                          : 0.f;
        refresh_operands(st);
        floatx4_t decay[4];       // summary pass: product of the tile decays for this lane's state rows
#pragma unroll
        for (int kt = 0; kt < 4; ++kt) decay[kt] = floatx4_t{1.f, 1.f, 1.f, 1.f};

        StateLoads pf;            // tile `slab` of the next chunk to stage, all 128 columns
        if (nchunks > 0) state_prefetch<kZBeta>(g, t_begin, slab, lane, has_beta, pf);
        for (int it = 0; it <= nchunks + 1; ++it) {
            unsigned long long t0 = PROF_T();
            if (it >= 1 && it <= nchunks)      // chunk it-1: its values were staged at the end of the previous iteration
                state_chunk<kSummary>(lds + ((it - 1) & 1) * kBufBytes, lds + kOffVt + ((it - 1) & 1) * kVtBuf,
                                      lds + kOffOb + ((it - 1) & 1) * kObBuf, slab, n, grp, st, decay);
            PROF_ADD(16 + slab * 3 + 1, t0);
            t0 = PROF_T();
            if (it < nchunks) {
                // values of chunk `it` (requested one iteration ago) -> LDS, then request the next chunk's
                stage_values<kZBeta>(lds + kOffVt + (it & 1) * kVtBuf, slab, lane, has_beta, pf, t_begin + it * kChunk, g.t_end);
                state_prefetch<kZBeta>(g, t_begin + (it + 1) * kChunk, slab, lane, has_beta, pf);   // unconditional (clamped), see gate_prefetch
            }
            PROF_ADD(16 + slab * 3, t0);
            t0 = PROF_T();
            __syncthreads();
            PROF_ADD(16 + slab * 3 + 2, t0);
        }

        float *S_out = kSummary ? plan.slots + (size_t)(seg + 1) * slot_elems : (seg == plan.nseg - 1 ? S_T : nullptr);
        if (S_out != nullptr) {
#pragma unroll
            for (int kt = 0; kt < 4; ++kt)
#pragma unroll
                for (int ct = 0; ct < 2; ++ct)
#pragma unroll
                    for (int r = 0; r < 4; ++r)
                        __builtin_nontemporal_store(st.S[kt][ct][r], S_out + state_base + (size_t)slab_channel(kt, 4 * grp + r) * dv + slab_column(ct, n));
        }
        if (kSummary && col_tile == 0 && slab == 0 && n == 0) {
            float *gam = plan.gamma + ((size_t)seg * BH + bh) * kK;
#pragma unroll
            for (int kt = 0; kt < 4; ++kt) *reinterpret_cast<floatx4_t *>(gam + slab_channel(kt, 4 * grp)) = decay[kt];
        }
    }
}

// Entering state of every segment from the summary pass: slot 0 = S0 (or zero), and for s >= 1
// slot s <- gamma[s-1] .* slot[s-1] + slot[s] (the increment left there by the summary pass).  One thread per
// four adjacent state elements; the segments are walked in order.
__global__ __launch_bounds__(256) void segment_state_scan_kernel(const float *S0, SegmentPlan plan, int dv, size_t quads_per_slot)
{
    const size_t e4 = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (e4 >= quads_per_slot) return;
    const size_t elem = e4 * 4;                           // element index inside a slot: ((bh * 64) + n) * dv + column
    const size_t row = elem / dv;                         // bh * 64 + n
    floatx4_t s = (S0 != nullptr) ? *reinterpret_cast<const floatx4_t *>(S0 + elem) : floatx4_t{0.f, 0.f, 0.f, 0.f};
    const size_t slot_elems = quads_per_slot * 4;
    *reinterpret_cast<floatx4_t *>(plan.slots + elem) = s;
    for (int sg = 1; sg < plan.nseg; ++sg) {
        const float gmm = plan.gamma[(size_t)(sg - 1) * (slot_elems / dv) + row];
        floatx4_t *p = reinterpret_cast<floatx4_t *>(plan.slots + (size_t)sg * slot_elems + elem);
        const floatx4_t inc = *p;
        s[0] = fmaf(gmm, s[0], inc[0]); s[1] = fmaf(gmm, s[1], inc[1]);
        s[2] = fmaf(gmm, s[2], inc[2]); s[3] = fmaf(gmm, s[3], inc[3]);
        *p = s;
    }
}

// How a call is cut into sequence segments.  A single pass runs one workgroup per (batch, head, 128 columns); when
// that leaves most of the 256 compute units idle the sequence is cut so that about 256 workgroups exist, each
// segment keeping at least four 64-token chunks.
struct SplitShape { int nseg, seg_tokens; };
SplitShape choose_split(int B, int T, int H, int dv)
{
    const long long wgs = (long long)B * H * (dv / kColTile);
    const int nchunks = (T + kChunk - 1) / kChunk;
    SplitShape sp{1, nchunks * kChunk};
    if (wgs == 0 || wgs >= 192 || nchunks < 8) return sp;
    long long want = (256 + wgs - 1) / wgs;
    if (want > nchunks / 4) want = nchunks / 4;
    if (want > 64) want = 64;
    if (want < 2) return sp;
    const int seg_chunks = (int)((nchunks + want - 1) / want);
    sp.nseg = (nchunks + seg_chunks - 1) / seg_chunks;
    sp.seg_tokens = seg_chunks * kChunk;
    if (sp.nseg < 2) sp = SplitShape{1, nchunks * kChunk};
    return sp;
}

// Output stage of the block applied to the stored outputs, in place: o <- (o + d .* x') .* act(z), 8 columns per thread.
// The scan kernel itself has no registers left for two more input streams, so on this path the stage is a second,
// bandwidth-bound kernel of the same call (the generic and the decode kernels apply it where they store o).
__global__ __launch_bounds__(256) void output_stage_kernel(bf16_t *__restrict__ o, OutputStage stage, size_t pieces, int H, int dv)
{
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= pieces) return;
    const size_t e = i * 8;
    const uint4 w = *reinterpret_cast<const uint4 *>(o + e);
    float y[8] = {bf16_lo(w.x), bf16_hi(w.x), bf16_lo(w.y), bf16_hi(w.y), bf16_lo(w.z), bf16_hi(w.z), bf16_lo(w.w), bf16_hi(w.w)};
    if (stage.x_prime != nullptr) {
        const uint4 xw = load_streaming(static_cast<const bf16_t *>(stage.x_prime) + e);
        const float x[8] = {bf16_lo(xw.x), bf16_hi(xw.x), bf16_lo(xw.y), bf16_hi(xw.y), bf16_lo(xw.z), bf16_hi(xw.z), bf16_lo(xw.w), bf16_hi(xw.w)};
        const float *dp = stage.d + e % ((size_t)H * dv);          // [H, dv] repeats every token
        const floatx4_t d0 = *reinterpret_cast<const floatx4_t *>(dp), d1 = *reinterpret_cast<const floatx4_t *>(dp + 4);
#pragma unroll
        for (int j = 0; j < 4; ++j) { y[j] = fmaf(d0[j], x[j], y[j]); y[4 + j] = fmaf(d1[j], x[4 + j], y[4 + j]); }
    }
    if (stage.z_gate != nullptr) {
        const uint4 zw = load_streaming(static_cast<const bf16_t *>(stage.z_gate) + e);
        const float z[8] = {bf16_lo(zw.x), bf16_hi(zw.x), bf16_lo(zw.y), bf16_hi(zw.y), bf16_lo(zw.z), bf16_hi(zw.z), bf16_lo(zw.w), bf16_hi(zw.w)};
#pragma unroll
        for (int j = 0; j < 8; ++j) y[j] *= output_gate(z[j], stage.act);
    }
    const uint4 out = {pack_bf16x2(y[0], y[1]), pack_bf16x2(y[2], y[3]), pack_bf16x2(y[4], y[5]), pack_bf16x2(y[6], y[7])};
    *reinterpret_cast<uint4 *>(o + e) = out;
}

}  // namespace

bool scan_mfma_supports(int dk, int dv, int chunk, int io_dtype)
{
    return io_dtype == RODIMUS_BF16 && dk == kK && chunk == kChunk && dv >= kColTile && dv % kColTile == 0;
}

size_t scan_mfma_workspace_bytes(int B, int T, int H, int dv)
{
    const SplitShape sp = choose_split(B, T, H, dv);
    if (sp.nseg <= 1) return 0;
    const size_t bh = (size_t)B * H;
    return ((size_t)sp.nseg * bh * kK * dv + (size_t)(sp.nseg - 1) * bh * kK) * sizeof(float);
}

namespace {

template <bool kZBeta, bool kGated>
hipError_t launch_scan_mfma_typed(const ScanArgs &a)
{
    // a packed variable-length batch is never cut into segments (its lengths live in device memory): one segment
    // that covers any length
    const SplitShape sp = a.cu_seqlens != nullptr ? SplitShape{1, ((a.T + kChunk - 1) / kChunk) * kChunk}
                                                  : choose_split(a.B, a.T, a.H, a.dv);
    const size_t bh = (size_t)a.B * a.H;
    SegmentPlan plan{sp.nseg, sp.seg_tokens, nullptr, nullptr};
    hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void *>(&scan_mfma_kernel<false, kZBeta, kGated>),
                                          hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBytes);
    if (attr == hipSuccess)
        attr = hipFuncSetAttribute(reinterpret_cast<const void *>(&scan_mfma_kernel<true, kZBeta, kGated>),
                                   hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBytes);
    if (attr != hipSuccess) return attr;
    const dim3 block(kThreads);
    const unsigned col_tiles = (unsigned)(a.dv / kColTile);
    const void *gate_a = kGated ? a.z_g : static_cast<const void *>(a.log_alpha);
    if (sp.nseg > 1) {
        plan.slots = static_cast<float *>(a.workspace);
        plan.gamma = plan.slots + (size_t)sp.nseg * bh * kK * a.dv;
        hipLaunchKernelGGL((scan_mfma_kernel<true, kZBeta, kGated>), dim3((unsigned)bh, col_tiles, (unsigned)(sp.nseg - 1)), block,
                           kLdsBytes, a.stream, (const bf16_t *)a.q, (const bf16_t *)a.k, (const bf16_t *)a.v, gate_a,
                           (const bf16_t *)a.z_tau, a.beta, (const float *)nullptr, (bf16_t *)nullptr, (float *)nullptr, a.T, a.H, a.dv, plan,
                           (const int *)nullptr, 0, 0);
        const size_t quads = bh * kK * a.dv / 4;
        hipLaunchKernelGGL(segment_state_scan_kernel, dim3((unsigned)((quads + 255) / 256)), dim3(256), 0, a.stream, a.S0,
                           plan, a.dv, quads);
    }
    // dense: (batch, head) x column tile x segment; packed: one flat index (see the kernel)
    const bool flat_dense = a.cu_seqlens == nullptr && sp.nseg == 1 && col_tiles > 1 && bh * col_tiles > 256;
    const dim3 grid = a.cu_seqlens != nullptr ? dim3((unsigned)(bh * col_tiles))
                      : flat_dense ? dim3((unsigned)((bh + 7) / 8 * 8 * col_tiles)) : dim3((unsigned)bh, col_tiles, (unsigned)sp.nseg);
    hipLaunchKernelGGL((scan_mfma_kernel<false, kZBeta, kGated>), grid, block, kLdsBytes,
                       a.stream, (const bf16_t *)a.q, (const bf16_t *)a.k, (const bf16_t *)a.v, gate_a, (const bf16_t *)a.z_tau, a.beta, a.S0,
                       (bf16_t *)a.o, a.S_T, a.T, a.H, a.dv, plan, a.cu_seqlens, a.T, a.B);
    if (a.stage.any()) {
        const size_t tokens = a.cu_seqlens != nullptr ? (size_t)a.T : (size_t)a.B * a.T;
        const size_t pieces = tokens * a.H * a.dv / 8;
        if (pieces > 0)
            hipLaunchKernelGGL(output_stage_kernel, dim3((unsigned)((pieces + 255) / 256)), dim3(256), 0, a.stream, (bf16_t *)a.o,
                               a.stage, pieces, a.H, a.dv);
    }
    return hipGetLastError();
}

}  // namespace

// The state entering every one of `nseg` segments of `seg_tokens` tokens (a multiple of 64) of a dense batch, for the
// backward pass cut along the sequence: summary pass over the first nseg-1 segments, then the chain over the segments.
// slots: [nseg][B*H][64][dv] fp32, gamma: [nseg-1][B*H][64] fp32 (the segment decays); beta: fp32 values or NULL, or
// (beta_preact) bf16 pre-activations.
namespace {

template <bool kZBeta>
hipError_t launch_segment_states_typed(const void *k, const void *v, const float *log_alpha, const void *beta, const float *S0,
                                       int B, int T, int H, int dv, int nseg, int seg_tokens, float *slots, float *gamma,
                                       hipStream_t stream)
{
    const size_t bh = (size_t)B * H;
    SegmentPlan plan{nseg, seg_tokens, slots, gamma};
    hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void *>(&scan_mfma_kernel<true, kZBeta, false>),
                                          hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBytes);
    if (attr != hipSuccess) return attr;
    hipLaunchKernelGGL((scan_mfma_kernel<true, kZBeta, false>), dim3((unsigned)bh, (unsigned)(dv / kColTile), (unsigned)(nseg - 1)),
                       dim3(kThreads), kLdsBytes, stream, (const bf16_t *)nullptr, (const bf16_t *)k, (const bf16_t *)v,
                       static_cast<const void *>(log_alpha), (const bf16_t *)nullptr, beta,
                       (const float *)nullptr, (bf16_t *)nullptr, (float *)nullptr, T, H, dv, plan, (const int *)nullptr, 0, 0);
    const size_t quads = bh * kK * dv / 4;
    hipLaunchKernelGGL(segment_state_scan_kernel, dim3((unsigned)((quads + 255) / 256)), dim3(256), 0, stream, S0, plan, dv, quads);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_scan_segment_states(const void *k, const void *v, const float *log_alpha, const void *beta, bool beta_preact,
                                      const float *S0, int B, int T, int H, int dv, int nseg, int seg_tokens, float *slots,
                                      float *gamma, hipStream_t stream)
{
    if (nseg < 2 || seg_tokens % kChunk != 0 || dv % kColTile != 0 || (beta_preact && beta == nullptr)) return hipErrorInvalidValue;
    return beta_preact ? launch_segment_states_typed<true>(k, v, log_alpha, beta, S0, B, T, H, dv, nseg, seg_tokens, slots, gamma, stream)
                       : launch_segment_states_typed<false>(k, v, log_alpha, beta, S0, B, T, H, dv, nseg, seg_tokens, slots, gamma, stream);
}

hipError_t launch_scan_mfma(const ScanArgs &a)
{
    if ((long long)a.B * a.H == 0) return hipSuccess;
    if (a.T == 0 && (a.S_T == nullptr || a.S_T == a.S0)) return hipSuccess;
    // the gated form takes the value gate as a pre-activation too, or none at all (kZBeta loads through `beta`
    // unconditionally, so a missing gate must take the other instance, where a NULL beta means all ones)
    if (a.gated()) return a.beta != nullptr ? launch_scan_mfma_typed<true, true>(a) : launch_scan_mfma_typed<false, true>(a);
    return (a.beta != nullptr && a.beta_preact) ? launch_scan_mfma_typed<true, false>(a) : launch_scan_mfma_typed<false, false>(a);
}

}  // namespace rodimus
