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
// The pairwise decay inside a tile is built in one of two ways, chosen per tile (wavefront-uniform):
//   * quotient form (the appendix's (Q .* A)(K / A)^T, the common case): one copy of q scaled by A_t, one of k
//     scaled by 1 / A_i, a single masked Gram matrix, G_i = A_16 / A_i.  Taken only when the tile's total decay
//     A_16 is at least 2^-80 in every channel, so that no reciprocal can overflow;
//   * product-only form (a hard reset or a very strong decay inside the tile): binary splitting of the tile.  For a
//     power of two h, a row t with bit h set pairs with the rows i of the first half of its aligned 2h-block and
//         prod_{j=i+1..t} alpha_j = (prod over t's h-block from its start through t) * (prod over the rows after i
//                                   to the end of i's h-block).
//     Every pair i < t belongs to exactly one h, all factors are <= 1 for log_alpha <= 0 and exactly 0 after
//     alpha = 0, so hard resets and decays beyond the fp32 range are exact.
//
// One workgroup (12 wavefronts) owns one (batch, head) and 128 value columns and walks its tokens in order.
// The wavefronts are specialised and work one chunk apart through double-buffered LDS, with ONE barrier per
// 64 tokens:
//   wavefronts 0-3 ("gate" wavefronts), one 16-row tile each: lane = (row, 16 key channels).  exp of the
//       log-gates, the prefix products by DPP across the 16 lanes of a row group, the decayed copies of q and k
//       as bf16 MFMA operands straight from registers, the scores as masked Gram matrices (MFMA), and for the
//       state wavefronts: q .* A, (k .* G)^T, A_16 and P into LDS.  They fetch their own q, k and gates one chunk
//       ahead into registers.
//   wavefronts 4-7 ("state" wavefronts), 32 value columns each: the fp32 state slab (64 x 32) lives in MFMA
//       accumulators for the whole walk; per tile o^T = S^T (q .* A)^T + (beta .* v)^T P^T into LDS,
//       S = diag(A_16) S + (k .* G)^T (beta .* v), and the bf16 copy of S that feeds the next tile.  They touch
//       no global memory inside the walk: the serial chain of the recurrence never waits on a memory queue.
//   wavefronts 8-11 ("value" wavefronts), one 16-row tile each, all 128 columns: fetch v and the value gate one
//       chunk ahead, stage beta .* v into LDS, and move finished outputs from LDS to global memory in whole
//       256-byte rows, applying the block's output stage (feed-through and output gate, Sec. 3.1.3) on the way.
#include "internal.h"

#include <atomic>

#ifndef PRIO_GATE
#define PRIO_GATE 0
#define PRIO_STATE 1
#define PRIO_VALUE 0
#endif

namespace rodimus {

namespace {

constexpr int kK = 64;           // key width
constexpr int kTile = 16;        // rows per state update
constexpr int kChunk = 64;       // tokens per barrier (4 tiles)
constexpr int kColTile = 128;    // value columns per workgroup
constexpr int kThreads = 768;        // 12 wavefronts: 4 gate, 4 state, 4 value

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
constexpr int kOffOb = kOffVt + 2 * kVtBuf;          // outputs, two chunk buffers of [64 t][128 col], 16-byte units swizzled by row:
                                                     // bf16 (256-byte rows), or fp32 (512-byte rows) when the block's output stage
                                                     // follows, so that o is rounded once, after the stage
constexpr int ob_buf_bytes(bool block) { return kChunk * (block ? 512 : 256); }
constexpr int kFeedBytes = kColTile * 4;             // block form: the feed-through weights d of this head and column tile, fp32, after the output buffers
constexpr int lds_bytes(bool block) { return kOffOb + 2 * ob_buf_bytes(block) + (block ? kFeedBytes : 0); }     // 104448 / 137728

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

// Value gate of a call (template parameter kBeta) and parts of the block's output stage it applies (kStage): compile-time,
// so that no load of the walk sits behind a branch.
constexpr int kBetaNone = 0, kBetaValues = 1, kBetaPreact = 2;      // all ones / fp32 gate values / bf16 pre-activations (sigmoid in the kernel)
constexpr int kStageFeed = 1, kStageGate = 2;                       // bit flags: feed-through d .* x', output gate act(z)

struct Geometry {
    const bf16_t *q, *k, *v;
    const float *la;
    const bf16_t *zg, *zt;  // gated form (kGated): pre-activations of the key-side gates instead of la
    const void *beta;       // value gate: fp32 values, or bf16 pre-activations, or null (kBeta)
    bf16_t *o;
    const bf16_t *x_prime, *z_gate;     // output stage of the block (kStage): feed-through input and gate pre-activation, or null
    const float *d;                     // feed-through weights [H, dv]
    int act;
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
    floatx4_t la[4];        // gated form: the bits of z_g (la[0], la[1]) and z_tau (la[2], la[3]), 8 bf16 each
};

// Addressing of the per-chunk global accesses: a base that is uniform over the wavefront (the chunk's first token row of
// this (batch, head), kept in scalar registers) plus a 32-bit byte offset per lane (the lane's row inside the chunk and its
// channels / columns).  One vector register per access instead of a 64-bit address pair: the address registers are what
// the three roles cannot afford at twelve wavefronts per workgroup.
// Loads are unconditional so that they stay in flight across the barrier: a chunk start beyond the sequence end is moved
// back to the last valid token and the lane's row is clamped to it; rows at or beyond the end are neutralised where
// they are consumed (gate_tile: q = k = 0, alpha = 1; stage_values: v = 0) and never stored.
struct ChunkRows {
    size_t first;           // token-head index ((tok0 + s') * H + h) of the chunk's first row, uniform
    int s_clamped;          // s' = min(s, t_end - 1), uniform
};
__device__ __forceinline__ ChunkRows chunk_rows(const Geometry &g, int s)
{
    const int s_clamped = min(s, g.t_end - 1);
    return ChunkRows{(g.tok0 + (size_t)s_clamped) * g.H + g.h, s_clamped};
}
// rows of the lane's token past the chunk's first row (0 for every lane of a chunk that lies beyond the end)
__device__ __forceinline__ uint32_t row_in_chunk(const Geometry &g, const ChunkRows &c, int s, int row)
{
    return (uint32_t)(min(s + row, g.t_end - 1) - c.s_clamped);
}
// A global-memory pointer that is the same in every lane, pinned to scalar registers (when scalar registers run short the
// compiler otherwise keeps such bases in vector register pairs and falls back to 64-bit vector addresses).  The result is
// typed as a global (address space 1) pointer: the round trip through integers hides that from the compiler.
typedef __attribute__((address_space(1))) char global_char_t;
__device__ __forceinline__ global_char_t *scalar_base(const void *p)
{
    const uint64_t a = reinterpret_cast<uint64_t>(p);
    const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)a), hi = __builtin_amdgcn_readfirstlane((uint32_t)(a >> 32));
    return reinterpret_cast<global_char_t *>(((uint64_t)hi << 32) | lo);
}
template <typename T>
__device__ __forceinline__ T load_at(const void *uniform_base, uint32_t byte_offset)
{
    static_assert(sizeof(T) == 16, "16-byte accesses only");
    typedef __attribute__((address_space(1))) const floatx4_t global_t;
    return __builtin_bit_cast(T, *reinterpret_cast<global_t *>(scalar_base(uniform_base) + (size_t)byte_offset));
}
__device__ __forceinline__ uint4 load_streaming_at(const void *uniform_base, uint32_t byte_offset)
{
    typedef __attribute__((address_space(1))) const floatx4_t global_t;
    return __builtin_bit_cast(uint4, __builtin_nontemporal_load(reinterpret_cast<global_t *>(scalar_base(uniform_base) + (size_t)byte_offset)));
}
__device__ __forceinline__ void store_streaming_at(void *uniform_base, uint32_t byte_offset, uint4 w)
{
    typedef __attribute__((address_space(1))) floatx4_t global_t;
    __builtin_nontemporal_store(__builtin_bit_cast(floatx4_t, w), reinterpret_cast<global_t *>(scalar_base(uniform_base) + (size_t)byte_offset));
}

// Chunk starting at token `s`, this lane's row `row` of it (16 * tile + n) and channel group `grp`.
template <bool kSummary, bool kGated>
__device__ __forceinline__ void gate_prefetch(const Geometry &g, int s, int row, int grp, GateLoads &p)
{
    const ChunkRows c = chunk_rows(g, s);
    const uint32_t off = row_in_chunk(g, c, s, row) * (uint32_t)(g.H * kK * 2) + 16u * grp;      // bytes into a bf16 [.., H, 64] tensor
    if (!kSummary) {
        const bf16_t *qb = g.q + c.first * kK;
        p.q[0] = load_at<uint4>(qb, off);
        p.q[1] = load_at<uint4>(qb, off + 64);
    }
    const bf16_t *kb = g.k + c.first * kK;
    p.k[0] = load_at<uint4>(kb, off);
    p.k[1] = load_at<uint4>(kb, off + 64);
    if (kGated) {
        const bf16_t *gb = g.zg + c.first * kK, *tb = g.zt + c.first * kK;
        p.la[0] = load_at<floatx4_t>(gb, off);
        p.la[1] = load_at<floatx4_t>(gb, off + 64);
        p.la[2] = load_at<floatx4_t>(tb, off);
        p.la[3] = load_at<floatx4_t>(tb, off + 64);
    } else {
        const float *lb = g.la + c.first * kK;
        p.la[0] = load_at<floatx4_t>(lb, 2 * off);
        p.la[1] = load_at<floatx4_t>(lb, 2 * off + 16);
        p.la[2] = load_at<floatx4_t>(lb, 2 * off + 128);
        p.la[3] = load_at<floatx4_t>(lb, 2 * off + 144);
    }
}

__device__ __forceinline__ bf16x8_t pack8(const float *x);

__device__ __forceinline__ void unpack_bf16x8(const uint4 &w, float *x)
{
    x[0] = bf16_lo(w.x); x[1] = bf16_hi(w.x); x[2] = bf16_lo(w.y); x[3] = bf16_hi(w.y);
    x[4] = bf16_lo(w.z); x[5] = bf16_hi(w.z); x[6] = bf16_lo(w.w); x[7] = bf16_hi(w.w);
}

__device__ __forceinline__ bf16x8_t pack8(const float *x)
{
    uint4 w = {pack_bf16x2(x[0], x[1]), pack_bf16x2(x[2], x[3]), pack_bf16x2(x[4], x[5]), pack_bf16x2(x[6], x[7])};
    return __builtin_bit_cast(bf16x8_t, w);
}

// ---- product-only construction of one tile (every split level).  Exact for any gates, including alpha = 0.
// It works on one half of the lane's channels at a time (8 channels = the 8 operand slots of one MFMA), which keeps
// its register footprint small; the two halves add into the same score accumulator.
struct HalfRow {            // 8 channels of one row: 8g..8g+7 (half 0) or 32+8g..32+8g+7 (half 1)
    float q[8], k[8], la[8];    // la: log of the decay gate; natural log as loaded, base 2 when the kernel evaluated it (gated form)
};
// the decay gate from its logarithm; exp(-inf) = 0
template <bool kBase2>
__device__ __forceinline__ float gate_from_log(float la) { return kBase2 ? __builtin_amdgcn_exp2f(la) : __expf(la); }

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

// The two key-side gates of one channel (Sec. 3.1.2) for the gated form of this kernel, in base 2 throughout (the hardware
// exponential and logarithm are base 2, so no conversion factors are spent on the wavefronts that are bound by the vector
// ALUs): g = softplus(z_g), tau = sigmoid(z_tau); log2_alpha = -g tau log2(e) (the decay gate is 2^log2_alpha) and
// alpha_hat = g^tau = 2^(tau log2 g).  Same short forms as ddts_channel_gates<true>.
__device__ __forceinline__ void ddts_channel_gates_base2(float z_g, float z_tau, float &log2_alpha, float &alpha_hat)
{
    constexpr float kLog2e = 1.44269504088896341f, kLn2 = 0.693147180559945309f;
    const float e = __builtin_amdgcn_exp2f(-fabsf(z_g) * kLog2e);                                 // exp(-|z_g|)
    const float g = fmaf(kLn2, __builtin_amdgcn_logf(1.f + e), fmaxf(z_g, 0.f));                  // softplus
    // log2 g: for very negative z, g = e^z (1 - e^z / 2 + ...) underflows before its logarithm does
    const float log2_g = z_g < -15.f ? fmaf(z_g, kLog2e, (-0.5f * kLog2e) * e) : __builtin_amdgcn_logf(g);
    const float tau = __builtin_amdgcn_rcpf(1.f + __builtin_amdgcn_exp2f(z_tau * -kLog2e));       // overflows to the right limit 0
    log2_alpha = (g * tau) * -kLog2e;
    alpha_hat = __builtin_amdgcn_exp2f(tau * log2_g);
}

// A value rounded to bf16 and widened again (what a pass that writes bf16 to memory would hand on).
__device__ __forceinline__ float round_to_bf16(float x) { return bf16_lo(pack_bf16x2(x, 0.f)); }

// Channels of `kHalf` of a loaded row as the tile construction wants them: fp32 log_alpha, k and q widened.
// Gated form (Sec. 3.1.2 and the pre-processing of Sec. 3.1.3): log_alpha = -softplus(z_g) sigmoid(z_tau) in fp32 (base 2),
// k <- softplus(z_g)^sigmoid(z_tau) .* k / max(||k||_2, 1e-12) and q <- q / sqrt(64), both rounded to bf16 (what a separate
// gate pass would have written; the division by 8 is exact); `inv_norm` is the reciprocal norm of the whole key row.
// Summary pass: q = 0.  Rows at or beyond the sequence end: q = k = 0, alpha = 1.
template <bool kSummary, bool kGated, int kHalf>
__device__ __forceinline__ void prepare_half_row(const GateLoads &in, bool valid, float inv_norm, HalfRow &r)
{
    unpack_bf16x8(in.k[kHalf], r.k);
    if (!kSummary) unpack_bf16x8(in.q[kHalf], r.q);
    if (kGated) {
        float zg[8], zt[8];
        unpack_bf16x8(__builtin_bit_cast(uint4, in.la[kHalf]), zg);
        unpack_bf16x8(__builtin_bit_cast(uint4, in.la[2 + kHalf]), zt);
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            float alpha_hat;
            ddts_channel_gates_base2(zg[j], zt[j], r.la[j], alpha_hat);
            r.k[j] = round_to_bf16(alpha_hat * r.k[j] * inv_norm);
            if (!kSummary) r.q[j] *= 0.125f;
        }
    } else {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            r.la[j] = in.la[2 * kHalf][j];
            r.la[4 + j] = in.la[2 * kHalf + 1][j];
        }
    }
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        if (kSummary || !valid) r.q[j] = 0.f;
        if (!valid) { r.k[j] = 0.f; r.la[j] = 0.f; }
    }
}

// Channels 32*half + 8grp .. +7 of one tile.
template <bool kSummary, bool kGated>
__device__ __forceinline__ void gate_half_products(unsigned char *buf, int tile, int row, int grp, int half, const HalfRow &in,
                                                   floatx4_t &acc)
{
    const float (&q)[8] = in.q;
    const float (&k)[8] = in.k;
    float a[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) a[j] = gate_from_log<kGated>(in.la[j]);
    const bool b0 = row & 1, b1 = row & 2, b2 = row & 4, b3 = row & 8;
    const floatx4_t zero = {0.f, 0.f, 0.f, 0.f};
    if (!kSummary) {
        // undecayed diagonal: a token sees its own write with weight one
        const floatx4_t d = mfma_k32(pack8(k), pack8(q), zero);
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
        *reinterpret_cast<bf16x8_t *>(qn + (((4 * half + grp) ^ (row & 7)) << 4)) = pack8(x);
    }
    {
        // k .* G, channels 32*half + 8grp .. +7 of token `row`: two 8-byte units
        unsigned char *kt = buf + kOffKt + tile * kKtTile + row * 128;
#pragma unroll
        for (int par = 0; par < 2; ++par) {
            const int e = 4 * par;
            const uint2 w = {pack_bf16x2(k[e] * suf[e], k[e + 1] * suf[e + 1]), pack_bf16x2(k[e + 2] * suf[e + 2], k[e + 3] * suf[e + 3])};
            *reinterpret_cast<uint2 *>(kt + (lds_key_unit(half, par, grp, row) << 3)) = w;
        }
    }
    if (row == 15) {              // decay of the whole tile
        float *gm = reinterpret_cast<float *>(buf + kOffGm + tile * kGmTile);
        floatx4_t lo = {pre[0], pre[1], pre[2], pre[3]};
        floatx4_t hi = {pre[4], pre[5], pre[6], pre[7]};
        *reinterpret_cast<floatx4_t *>(gm + 32 * half + 8 * grp) = lo;
        *reinterpret_cast<floatx4_t *>(gm + 32 * half + 8 * grp + 4) = hi;
    }
}

// One 16-row tile, one half of the lane's channels (8 channels = the 8 operand slots of one MFMA) at a time: the register
// budget of a wavefront does not hold the unpacked copies of all 16.  The prefix products A_t of the gates are needed in
// any case.  When the total decay A_16 of these channels is far from underflow (the common case), the pairwise decay inside
// the tile is taken as the quotient A_t / A_i of the appendix's parallel form: one version of q (q .* A, which is also the
// inter-tile operand) and one of k (k ./ A), a single masked Gram matrix, and G_i = A_16 / A_i.  Otherwise (a hard reset or
// a very strong decay inside the tile, where 1 / A_i would overflow or divide by zero) these channels take the
// product-only construction above.  The scores are a sum over channels, so the choice is made per half; it is
// wavefront-uniform.  `d` collects the scores [key row 4grp + r][query row `row`] of both halves.
constexpr float kSafeTileDecay = 8.2718061e-25f;     // 2^-80: 1 / A_i stays below 2^80, far inside bf16 and fp32 range

template <bool kSummary, bool kGated, int kHalf>
__device__ __forceinline__ void gate_half_tile(unsigned char *buf, int tile, int row, int grp, const GateLoads &in, bool valid,
                                               float inv_norm, floatx4_t &d)
{
    HalfRow r;
    prepare_half_row<kSummary, kGated, kHalf>(in, valid, inv_norm, r);
    float pre[8];
#pragma unroll
    for (int c = 0; c < 8; ++c) pre[c] = gate_from_log<kGated>(r.la[c]);
    // prefix products A_t over the 16 rows: four doubling steps of DPP row shifts with the identity shifted in
#pragma unroll
    for (int c = 0; c < 8; ++c) pre[c] *= row_shift_right<1>(pre[c], 1.f);
#pragma unroll
    for (int c = 0; c < 8; ++c) pre[c] *= row_shift_right<2>(pre[c], 1.f);
#pragma unroll
    for (int c = 0; c < 8; ++c) pre[c] *= row_shift_right<4>(pre[c], 1.f);
#pragma unroll
    for (int c = 0; c < 8; ++c) pre[c] *= row_shift_right<8>(pre[c], 1.f);
    // the total decay A_16 is row 15's prefix product: that lane decides for its channels
    bool weak = true;
#pragma unroll
    for (int c = 0; c < 8; ++c) weak = weak && (pre[c] >= kSafeTileDecay);        // false for 0 and NaN as well
    if (__any(row == 15 && !weak)) {
        gate_half_products<kSummary, kGated>(buf, tile, row, grp, kHalf, r, d);
        return;
    }

    float total[8];
#pragma unroll
    for (int c = 0; c < 8; ++c) {
        r.k[c] *= __builtin_amdgcn_rcpf(pre[c]);                                   // k ./ A
        total[c] = swizzle_lane<0x10, 0x0f>(pre[c]);                               // A_16 (row 15 of the tile)
    }
    if (!kSummary) {
#pragma unroll
        for (int c = 0; c < 8; ++c) r.q[c] *= pre[c];                              // q .* A
        const bf16x8_t qa = pack8(r.q);
        d = mfma_k32(pack8(r.k), qa, d);
        unsigned char *qn = buf + kOffQn + tile * kQnTile + row * 128;
        *reinterpret_cast<bf16x8_t *>(qn + (((4 * kHalf + grp) ^ (row & 7)) << 4)) = qa;
    }
    // k .* G with G_i = A_16 / A_i; same LDS placement as in gate_half_products
    unsigned char *kt = buf + kOffKt + tile * kKtTile + row * 128;
#pragma unroll
    for (int par = 0; par < 2; ++par) {
        const int c = 4 * par;
        const uint2 w = {pack_bf16x2(r.k[c] * total[c], r.k[c + 1] * total[c + 1]),
                         pack_bf16x2(r.k[c + 2] * total[c + 2], r.k[c + 3] * total[c + 3])};
        *reinterpret_cast<uint2 *>(kt + (lds_key_unit(kHalf, par, grp, row) << 3)) = w;
    }
    if (row == 15) {              // decay of the whole tile
        float *gm = reinterpret_cast<float *>(buf + kOffGm + tile * kGmTile);
        floatx4_t lo = {pre[0], pre[1], pre[2], pre[3]};
        floatx4_t hi = {pre[4], pre[5], pre[6], pre[7]};
        *reinterpret_cast<floatx4_t *>(gm + 32 * kHalf + 8 * grp) = lo;
        *reinterpret_cast<floatx4_t *>(gm + 32 * kHalf + 8 * grp + 4) = hi;
    }
}

template <bool kSummary, bool kGated>
__device__ __forceinline__ void gate_tile(unsigned char *buf, int tile, int row, int grp, const GateLoads &in, bool valid)
{
    float inv_norm = 1.f;
    if (kGated) {
        // squared norm of the raw key row: this lane's 16 channels, then the four lanes that share the row
        float kf[16];
        unpack_bf16x8(in.k[0], kf);
        unpack_bf16x8(in.k[1], kf + 8);
        float ss = 0.f;
#pragma unroll
        for (int c = 0; c < 16; ++c) ss = fmaf(kf[c], kf[c], ss);
        ss += __shfl_xor(ss, 16);
        ss += __shfl_xor(ss, 32);
        inv_norm = inverse_key_norm(ss);
    }
    floatx4_t d = {0.f, 0.f, 0.f, 0.f};
    gate_half_tile<kSummary, kGated, 0>(buf, tile, row, grp, in, valid, inv_norm, d);
    gate_half_tile<kSummary, kGated, 1>(buf, tile, row, grp, in, valid, inv_norm, d);
    if (!kSummary) {
        // P[t = row][i = 4grp .. 4grp+3], keys up to and including the query row (the product-only construction adds nothing
        // beyond the diagonal, the quotient form does)
        const int i0 = 4 * grp;
        uint2 w = {pack_bf16x2(i0 <= row ? d[0] : 0.f, i0 + 1 <= row ? d[1] : 0.f),
                   pack_bf16x2(i0 + 2 <= row ? d[2] : 0.f, i0 + 3 <= row ? d[3] : 0.f)};
        *reinterpret_cast<uint2 *>(buf + kOffPd + tile * kPdTile + row * 32 + grp * 8) = w;
    }
}

// =========================================================================================================
// State wavefronts
// =========================================================================================================
// State wavefront `w` fetches tile w of every chunk for ALL 128 columns of the workgroup (whole 256-byte rows of v,
// 512-byte rows of beta: long contiguous pieces are what HBM delivers at full rate) and stages beta .* v for
// the four state wavefronts.  Lane = (row 4u + lane/16 for u = 0..3, columns 8(lane%16) .. +7).
// The value gate arrives as fp32 values, as bf16 pre-activations whose sigmoid is taken here (half the bytes, two
// transcendentals per element), or not at all (all ones).
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

template <int kBeta>
__device__ __forceinline__ void state_prefetch(const Geometry &g, int s, int tile, int lane, StateLoads &p)
{
    const int rsub = lane >> 4, piece = lane & 15;
    const ChunkRows c = chunk_rows(g, s);
    const size_t first = c.first * g.dv + g.j0;              // element index of the chunk's first row, this column tile
    const bf16_t *vb = g.v + first;
    const uint32_t row_bytes = (uint32_t)(g.H * g.dv * 2);
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        const uint32_t off = row_in_chunk(g, c, s, 16 * tile + 4 * u + rsub) * row_bytes + 16u * piece;    // bytes, bf16 tensors
        p.v[u] = load_streaming_at(vb, off);
        if (kBeta == kBetaPreact) {
            p.zbeta[u] = load_streaming_at(static_cast<const bf16_t *>(g.beta) + first, off);
        } else if (kBeta == kBetaValues) {
            const float *bb = static_cast<const float *>(g.beta) + first;
            p.beta[u][0] = __builtin_bit_cast(floatx4_t, load_streaming_at(bb, 2 * off));
            p.beta[u][1] = __builtin_bit_cast(floatx4_t, load_streaming_at(bb, 2 * off + 16));
        }
    }
}

// beta .* v of one tile, rounded to bf16, into the chunk buffer `vt` (token-major, see lds_value_unit).  The lane's
// 8 columns 8*piece .. +7 are the units (slab = piece/4, c = piece%4, ct = 0 and 1) of its token row.
template <int kBeta>
__device__ __forceinline__ void stage_values(unsigned char *vt, int tile, int lane, const StateLoads &p, int s, int t_end)
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
        if (kBeta == kBetaPreact) {
            const uint32_t z[4] = {p.zbeta[u].x, p.zbeta[u].y, p.zbeta[u].z, p.zbeta[u].w};
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                gv[2 * j] *= sigmoid_short(bf16_lo(z[j]));
                gv[2 * j + 1] *= sigmoid_short(bf16_hi(z[j]));
            }
        } else if (kBeta == kBetaValues) {
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

// Outputs of a finished chunk: LDS -> global, whole 256-byte rows.  Done by the value wavefronts, wavefront w taking
// rows 16w .. 16w+15; lane = (row 4u + lane/16 for u = 0..3, columns 8(lane%16) .. +7).
__device__ __forceinline__ void store_row(const Geometry &g, int s, int row, int unit, uint4 w)
{
    // chunk start s <= t_end - 1 here (the chunk exists); rows at or beyond the end are not stored
    bf16_t *ob = g.o + ((g.tok0 + (size_t)s) * g.H + g.h) * g.dv + g.j0;
    const uint32_t off = (uint32_t)row * (uint32_t)(g.H * g.dv * 2) + 16u * unit;
    if (s + row < g.t_end) store_streaming_at(ob, off, w);
}

__device__ __forceinline__ void store_outputs(const Geometry &g, const unsigned char *ob, int s, int wave, int lane)
{
    asm volatile("" : "+v"(lane));       // offsets recomputed per chunk: hoisted out of the loop they would cost ten registers
    const int rsub = lane >> 4, unit = lane & 15;
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        const int row = 16 * wave + 4 * u + rsub;
        const uint4 w = *reinterpret_cast<const uint4 *>(ob + row * 256 + ((unit ^ (row & 15)) << 4));
        store_row(g, s, row, unit, w);
    }
}

// Output stage of the block (Sec. 3.1.3: y = (o + d .* x') .* act(z)), applied where the outputs leave LDS.  The rows of x'
// and z that belong to a chunk are requested one iteration before that chunk is stored.
struct StageLoads {
    uint4 x[4], z[4];
};

// The 16 rows of a tile come in four groups u (rows 4u + lane/16); a wavefront handles the groups kU0 .. kU1-1 (the value
// wavefront of the tile takes the first two, its gate wavefront the last two: each has the registers for two).
template <int kStage, int kU0, int kU1>
__device__ __forceinline__ void stage_prefetch(const Geometry &g, int s, int t_begin, int wave, int lane, StageLoads &p)
{
    const int rsub = lane >> 4, unit = lane & 15;
    s = max(s, t_begin);                                     // the first iteration asks for the chunk before the segment
    const ChunkRows c = chunk_rows(g, s);
    const size_t first = c.first * g.dv + g.j0;
    const uint32_t row_bytes = (uint32_t)(g.H * g.dv * 2);
#pragma unroll
    for (int u = kU0; u < kU1; ++u) {
        const uint32_t off = row_in_chunk(g, c, s, 16 * wave + 4 * u + rsub) * row_bytes + 16u * unit;
        if (kStage & kStageFeed) p.x[u] = load_streaming_at(g.x_prime + first, off);
        if (kStage & kStageGate) p.z[u] = load_streaming_at(g.z_gate + first, off);
    }
}

// fp32 outputs of a finished chunk in LDS (512-byte rows, 32-byte units swizzled by row): the stage in fp32, one rounding
// to bf16, and the eight results written back over the first half of the unit they came from (a lane touches its own
// units only).  The state wavefronts move them to global memory one iteration later (store_outputs_block).
// feed: the 128 feed-through weights of this column tile in LDS.
template <int kStage, int kU0, int kU1>
__device__ __forceinline__ void finish_outputs_block(const Geometry &g, unsigned char *ob, int wave, int lane,
                                                     const StageLoads &p, const unsigned char *feed)
{
    const int rsub = lane >> 4, unit = lane & 15;
    float d8[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    if (kStage & kStageFeed) {
        const floatx4_t lo = *reinterpret_cast<const floatx4_t *>(feed + 32 * unit), hi = *reinterpret_cast<const floatx4_t *>(feed + 32 * unit + 16);
        d8[0] = lo[0]; d8[1] = lo[1]; d8[2] = lo[2]; d8[3] = lo[3]; d8[4] = hi[0]; d8[5] = hi[1]; d8[6] = hi[2]; d8[7] = hi[3];
    }
#pragma unroll
    for (int u = kU0; u < kU1; ++u) {
        const int row = 16 * wave + 4 * u + rsub;
        unsigned char *src = ob + row * 512 + ((unit ^ (row & 15)) << 5);
        const floatx4_t lo = *reinterpret_cast<const floatx4_t *>(src), hi = *reinterpret_cast<const floatx4_t *>(src + 16);
        float y[8] = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
        if (kStage & kStageFeed) {
            float x[8];
            unpack_bf16x8(p.x[u], x);
#pragma unroll
            for (int j = 0; j < 8; ++j) y[j] = fmaf(d8[j], x[j], y[j]);
        }
        if (kStage & kStageGate) {
            float z[8];
            unpack_bf16x8(p.z[u], z);
#pragma unroll
            for (int j = 0; j < 8; ++j) y[j] *= output_gate(z[j], g.act);
        }
        *reinterpret_cast<uint4 *>(src) = uint4{pack_bf16x2(y[0], y[1]), pack_bf16x2(y[2], y[3]), pack_bf16x2(y[4], y[5]), pack_bf16x2(y[6], y[7])};
    }
}

// The finished bf16 outputs of a chunk (see finish_outputs_block) to global memory, by the state wavefronts: wavefront
// `slab` takes ITS OWN 32 columns of all 64 rows, 64 bytes per row, because it is about to overwrite exactly those bytes
// with the next chunk's outputs (program order inside the wavefront is the only ordering there is between the two).
__device__ __forceinline__ void store_outputs_block(const Geometry &g, const unsigned char *ob, int s, int slab, int lane)
{
    asm volatile("" : "+v"(lane));       // offsets recomputed per chunk, see store_outputs
    const int rsub = lane >> 2, piece = lane & 3;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int row = 16 * j + rsub, unit = 4 * slab + piece;
        const uint4 w = *reinterpret_cast<const uint4 *>(ob + row * 512 + ((unit ^ (row & 15)) << 5));
        store_row(g, s, row, unit, w);
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
#pragma unroll
    for (int kt = 0; kt < 4; ++kt)
        op.ka[kt] = lds_read_transposed(buf + kOffKt + tile * kKtTile + r * 128 + (lds_key_unit(kt >> 1, kt & 1, c, r) << 3));
}

// One chunk (4 tiles) of the state recurrence and the outputs for this wavefront's 32 columns.  The LDS operands
// of tile i+1 are requested before tile i is computed.
template <bool kSummary, bool kBlock>
__device__ __forceinline__ void state_chunk(const unsigned char *buf, const unsigned char *vt, unsigned char *ob,
                                            int slab, int n, int grp, StateSlab &st, floatx4_t (&decay)[4])
{
    TileOperands ops[2];
    load_tile_operands<kSummary>(buf, vt, 0, slab, n, grp, ops[0]);
#pragma unroll
    for (int tile = 0; tile < 4; ++tile) {
        if (tile + 1 < 4) load_tile_operands<kSummary>(buf, vt, tile + 1, slab, n, grp, ops[(tile + 1) & 1]);
        const TileOperands &op = ops[tile & 1];
        // the tile's decay A_16 for this lane's state rows: wanted only after the output products, so it is fetched here
        // rather than a tile ahead with the rest (16 registers)
        floatx4_t dec[4];
        const float *gm = reinterpret_cast<const float *>(buf + kOffGm + tile * kGmTile);
#pragma unroll
        for (int kt = 0; kt < 4; ++kt) dec[kt] = *reinterpret_cast<const floatx4_t *>(gm + slab_channel(kt, 4 * grp));

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
            for (int kt = 0; kt < 4; ++kt) decay[kt] *= dec[kt];
        }
        // S = diag(A_16) S + (k .* G)^T (beta .* v)
#pragma unroll
        for (int kt = 0; kt < 4; ++kt) {
#pragma unroll
            for (int ct = 0; ct < 2; ++ct) {
                floatx4_t x = st.S[kt][ct];
                x[0] *= dec[kt][0]; x[1] *= dec[kt][1]; x[2] *= dec[kt][2]; x[3] *= dec[kt][3];
                st.S[kt][ct] = mfma_k16(op.ka[kt], op.va[ct], x);
            }
        }
        if (!kSummary) {
            // row 16tile + n of the chunk's output buffer, columns 32slab + 8grp .. +7 (16-byte unit 4slab + grp)
            if (kBlock) {
                // fp32, 32-byte unit 4slab + grp of the row: the output stage and the rounding follow where the row leaves LDS
                unsigned char *dst = ob + (16 * tile + n) * 512 + (((4 * slab + grp) ^ n) << 5);
                *reinterpret_cast<floatx4_t *>(dst) = O[0];
                *reinterpret_cast<floatx4_t *>(dst + 16) = O[1];
            } else {
                uint4 w = {pack_bf16x2(O[0][0], O[0][1]), pack_bf16x2(O[0][2], O[0][3]),
                           pack_bf16x2(O[1][0], O[1][1]), pack_bf16x2(O[1][2], O[1][3])};
                *reinterpret_cast<uint4 *>(ob + (16 * tile + n) * 256 + (((4 * slab + grp) ^ n) << 4)) = w;
            }
            refresh_operands(st);
        }
    }
}

// Workspace of a sequence-split call: `nseg` state slots [seg][B*H][64][dv] fp32 followed by the segment decays
// [nseg-1][B*H][64] fp32.  Slot 0 receives the initial state, slot s > 0 first the state increment of segment s-1
// (summary pass), then the state entering segment s (segment_state_scan_kernel), which the main pass reads.
//
// Packed batch cut on the device (`packed_cut`): the host knows only the total token count, so it fixes the segment length
// and an upper bound on the number of segments; every sequence owns consecutive slots, counted from the sequences before it
// (locate_packed_slot).  Slots are [slot][H][64][dv], decays [slot][H][64]; `nseg` is then the slot bound.
struct SegmentPlan {
    int nseg;              // 1: no split, no workspace
    int seg_tokens;        // tokens per segment, a multiple of 64
    float *slots;
    float *gamma;
    bool packed_cut;
};

// Row range of sequence b of a packed batch; every entry is clamped to the tensor so that a corrupt table cannot take an
// access outside it.
__device__ __forceinline__ void packed_rows(const int *__restrict__ cu_seqlens, int b, int total_tokens, int &first, int &last)
{
    first = min(max(cu_seqlens[b], 0), total_tokens);
    last = min(max(cu_seqlens[b + 1], first), total_tokens);
}

// Flat grids over (pair, column tile), a pair being a (sequence or slot, head): workgroups go round-robin over the eight
// XCDs (each with its own L2), so in every run of 8 * col_tiles workgroups the column tiles of a pair are 8 apart: on the
// same XCD and started together, they share q, k and the gates in its L2.  The grid holds whole runs (packed_grid).
__device__ __forceinline__ void xcd_pair_mapping(unsigned x, int col_tiles, int &pair, int &col_tile)
{
    const unsigned group = x / 8;
    col_tile = (int)(group % (unsigned)col_tiles);
    pair = (int)((group / (unsigned)col_tiles) * 8 + x % 8);
}

// kSummary = false: the scan proper over this workgroup's segment (blockIdx.z), reading its entering state.
// kSummary = true : same walk from a zero state without q, scores or outputs; leaves the segment's state
//                   increment in slot seg+1 and the segment's total decay in gamma[seg].
// kBeta: what `beta` holds: nothing (NULL, all ones), fp32 gate values, or bf16 pre-activations of the value gate.
// kGated: `log_alpha` holds the bf16 pre-activations z_g and `z_tau` those of the temperature gate; q and k are raw.
// kStage: the parts of the block's output stage (`stage`) applied to the outputs on their way from LDS to global memory.
template <bool kSummary, int kBeta, bool kGated, int kStage>
__global__ __launch_bounds__(kThreads) void scan_mfma_kernel(
    const bf16_t *__restrict__ q, const bf16_t *__restrict__ k, const bf16_t *__restrict__ v,
    const void *__restrict__ log_alpha, const bf16_t *__restrict__ z_tau, const void *__restrict__ beta, const float *S0,
    bf16_t *__restrict__ o, float *S_T, int T, int H, int dv, SegmentPlan plan, const int *__restrict__ cu_seqlens,
    int total_tokens, int total_seqs, OutputStage stage)
{
    extern __shared__ __align__(16) unsigned char lds[];
    constexpr bool kBlock = kStage != 0;
    constexpr int kObBuf = ob_buf_bytes(kBlock);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int n = lane & 15, grp = lane >> 4;
    int bh = blockIdx.x, col_tile = blockIdx.y;
    int seg = blockIdx.z;                      // slot of the workspace this segment's entering state sits in
    int BH = gridDim.x, slot_bh = bh;          // (batch, head) pairs per slot and this workgroup's index among them
    bool last_seg = seg == plan.nseg - 1;
    int t_begin = seg * plan.seg_tokens;
    size_t tok0 = 0;
    if (plan.packed_cut) {
        // Flat grid over (slot, head, column tile).  Which sequence the slot belongs to follows from the lengths of the
        // sequences before it: a short walk (the cut is only made when the batch holds few sequences), the same in every
        // lane, out of scalar registers.
        int rest;
        xcd_pair_mapping(blockIdx.x, dv / kColTile, rest, col_tile);
        if (rest >= plan.nseg * H) return;                   // the grid is rounded up to whole runs of eight pairs
        const int slot = rest / H;
        PackedSlot ps;
        if (!locate_packed_slot(cu_seqlens, total_seqs, total_tokens, plan.seg_tokens, slot, ps)) return;      // the grid covers the largest possible number of slots
        last_seg = ps.j == ps.count - 1;
        // nothing continues from a sequence's last segment; with a valid table the segments fit the slots, a corrupt one
        // (overlapping sequences) must not reach past them
        if (kSummary && (last_seg || slot + 1 >= plan.nseg)) return;
        bh = __builtin_amdgcn_readfirstlane(ps.b * H + rest % H);
        seg = slot; BH = H; slot_bh = rest % H;
        t_begin = ps.j * plan.seg_tokens;
        tok0 = ps.first;
        T = ps.len;
    } else if (!kSummary && cu_seqlens == nullptr && gridDim.y == 1 && gridDim.z == 1 && dv > kColTile) {
        // Dense batch with more workgroups than compute units, launched flat: workgroups go round-robin over the eight XCDs
        // (each with its own L2), so in every run of 8 * col_tiles workgroups the column tiles of a (batch, head) are 8
        // apart: on the same XCD and started together, they share q, k and the gates in its L2.
        const int col_tiles = dv / kColTile;
        col_tile = (blockIdx.x / 8) % col_tiles;
        bh = (blockIdx.x / (8 * col_tiles)) * 8 + blockIdx.x % 8;
        if (bh >= total_seqs * H) return;                   // the grid is rounded up to whole runs
        slot_bh = bh;
    } else if (!kSummary && cu_seqlens != nullptr) {
        // Packed batch, launched as a flat grid: the column tiles of one (sequence, head) start together on one XCD (they
        // read the same q, k and gates while those are in its L2), and the workgroups take the sequences by descending
        // length (small batches).
        int slot;
        xcd_pair_mapping(blockIdx.x, dv / kColTile, slot, col_tile);
        if (slot >= total_seqs * H) return;                  // the grid is rounded up to whole runs of eight pairs
        const int rank = slot / H;
        const int b = sequence_by_length_rank(cu_seqlens, total_seqs, total_tokens, rank, reinterpret_cast<int *>(lds));   // the dynamic LDS is free until the walk starts
        bh = __builtin_amdgcn_readfirstlane(b * H + slot % H);      // the same in every lane: keeps the row bases in scalar registers
        slot_bh = bh;
    }

    Geometry g;
    g.q = q; g.k = k; g.v = v; g.beta = beta; g.o = o;
    g.la = kGated ? nullptr : static_cast<const float *>(log_alpha);
    g.zg = kGated ? static_cast<const bf16_t *>(log_alpha) : nullptr;
    g.zt = z_tau;
    g.x_prime = (kStage & kStageFeed) ? static_cast<const bf16_t *>(stage.x_prime) : nullptr;
    g.z_gate = (kStage & kStageGate) ? static_cast<const bf16_t *>(stage.z_gate) : nullptr;
    g.d = stage.d; g.act = stage.act;
    g.H = H; g.dv = dv;
    g.h = bh % H; g.j0 = col_tile * kColTile;
    g.tok0 = (size_t)(bh / H) * T;
    if (plan.packed_cut) {
        g.tok0 = tok0;
    } else if (cu_seqlens != nullptr) {
        // packed variable-length batch: sequence bh / H owns the token rows [cu[b], cu[b+1])
        int first, last;
        packed_rows(cu_seqlens, bh / H, total_tokens, first, last);
        g.tok0 = first;
        T = last - first;
    }
    g.t_end = min(T, t_begin + plan.seg_tokens);

    const int nchunks = max(0, (g.t_end - t_begin + kChunk - 1) / kChunk);
    const size_t slot_elems = (size_t)BH * kK * dv;

    // Every role runs nchunks + 2 iterations with one barrier each.  Iteration `it`: the gate wavefronts build chunk `it`,
    // the value wavefronts stage the values of chunk `it` and store the outputs of chunk it-2, the state wavefronts
    // advance the recurrence over chunk it-1.
    // The three wavefronts of a SIMD compete for its issue slots; the ones with the least slack go first.
    if (wave < 4) {
        // ------------------------------------------------------------------ gate wavefront, tile = wave
        __builtin_amdgcn_s_setprio(PRIO_GATE);
        if (kBlock && !kSummary) {
            // With the block's output stage these wavefronts also finish half of their tile's output rows (the value
            // wavefronts are the busiest otherwise).  They then keep ONE set of loads: the next chunk's rows are requested after
            // the current chunk is built, into the registers it has just freed, and are in flight across the barrier; with the
            // stage the iteration is long enough to cover them.
            GateLoads in;
            StageLoads sl;
            const unsigned char *feed = lds + kOffOb + 2 * kObBuf;
            const int row = 16 * wave + n;
            constexpr int kDrain = 2;          // iterations after the last chunk is built: state, finish, store
            if (nchunks > 0) gate_prefetch<kSummary, kGated>(g, t_begin, row, grp, in);
            for (int it = 0; it <= nchunks + kDrain; ++it) {
                if (it < nchunks) {
                    const int s = t_begin + it * kChunk;
                    gate_tile<kSummary, kGated>(lds + (it & 1) * kBufBytes, wave, n, grp, in, s + row < g.t_end);
                    gate_prefetch<kSummary, kGated>(g, s + kChunk, row, grp, in);
                }
                if (it >= 2 && it <= nchunks + 1)
                    finish_outputs_block<kStage, 2, 4>(g, lds + kOffOb + (it & 1) * kObBuf, wave, lane, sl, feed);
                if (nchunks > 0) stage_prefetch<kStage, 2, 4>(g, t_begin + (it - 1) * kChunk, t_begin, wave, lane, sl);
                __syncthreads();
            }
            return;
        }
        GateLoads even, odd;      // loads of even / odd chunks, requested one chunk ahead: no register copies between iterations
        const int row = 16 * wave + n;             // this lane's row of every chunk
        if (nchunks > 0) gate_prefetch<kSummary, kGated>(g, t_begin, row, grp, even);
        for (int it = 0;;) {
            if (it < nchunks) {
                const int s = t_begin + it * kChunk;
                gate_prefetch<kSummary, kGated>(g, s + kChunk, row, grp, odd);     // unconditional (clamped): keeps the wait counts exact
                gate_tile<kSummary, kGated>(lds, wave, n, grp, even, s + row < g.t_end);
            }
            __syncthreads();
            if (++it > nchunks + 1) break;
            if (it < nchunks) {
                const int s = t_begin + it * kChunk;
                gate_prefetch<kSummary, kGated>(g, s + kChunk, row, grp, even);
                gate_tile<kSummary, kGated>(lds + kBufBytes, wave, n, grp, odd, s + row < g.t_end);
            }
            __syncthreads();
            if (++it > nchunks + 1) break;
        }
    } else if (wave < 8) {
        // ------------------------------------------------------------------ state wavefront, slab = wave - 4
        const int slab = wave - 4;
        __builtin_amdgcn_s_setprio(PRIO_STATE);
        StateSlab st;
        // offsets of this wavefront's slab in the caller's state tensors and inside a workspace slot
        const size_t cache_base = (size_t)bh * kK * dv + g.j0 + 32 * slab, slot_base = (size_t)slot_bh * kK * dv + g.j0 + 32 * slab;
        // entering state: zero (summary), the caller's S0 (no split), or this segment's workspace slot.  The state is read
        // once here and written once at the end: streaming accesses
        const float *S_in = kSummary ? nullptr
                                     : (plan.nseg > 1 ? plan.slots + seg * slot_elems + slot_base : (S0 != nullptr ? S0 + cache_base : nullptr));
#pragma unroll
        for (int kt = 0; kt < 4; ++kt)
#pragma unroll
            for (int ct = 0; ct < 2; ++ct)
#pragma unroll
                for (int r = 0; r < 4; ++r)
                    st.S[kt][ct][r] = (S_in != nullptr)
                                          ? __builtin_nontemporal_load(S_in + (size_t)slab_channel(kt, 4 * grp + r) * dv + slab_column(ct, n))
                                          : 0.f;
        refresh_operands(st);
        floatx4_t decay[4];       // summary pass: product of the tile decays for this lane's state rows
#pragma unroll
        for (int kt = 0; kt < 4; ++kt) decay[kt] = floatx4_t{1.f, 1.f, 1.f, 1.f};

        for (int it = 0; it <= nchunks + (kBlock ? 2 : 1); ++it) {
            // outputs of chunk it-2 (finished in iteration it-1), rows 16 slab .. +15: these wavefronts wait for no loads, so the
            // slow completion of the stores holds nothing up (memory operations of a wavefront retire in order)
            if (!kSummary && !kBlock && it >= 2) store_outputs(g, lds + kOffOb + (it & 1) * kObBuf, t_begin + (it - 2) * kChunk, slab, lane);
            // with the output stage: chunk it-3, which the other wavefronts finished in place in iteration it-1, from the buffer
            // that this iteration's chunk is about to overwrite
            if (!kSummary && kBlock && it >= 3) store_outputs_block(g, lds + kOffOb + ((it - 1) & 1) * kObBuf, t_begin + (it - 3) * kChunk, slab, lane);
            if (it >= 1 && it <= nchunks)      // chunk it-1: built and staged by the other wavefronts in the previous iteration
                state_chunk<kSummary, kBlock>(lds + ((it - 1) & 1) * kBufBytes, lds + kOffVt + ((it - 1) & 1) * kVtBuf,
                                              lds + kOffOb + ((it - 1) & 1) * kObBuf, slab, n, grp, st, decay);
            __syncthreads();
        }

        float *S_out = kSummary ? plan.slots + (size_t)(seg + 1) * slot_elems + slot_base
                                : (last_seg && S_T != nullptr ? S_T + cache_base : nullptr);
        if (S_out != nullptr) {
#pragma unroll
            for (int kt = 0; kt < 4; ++kt)
#pragma unroll
                for (int ct = 0; ct < 2; ++ct)
#pragma unroll
                    for (int r = 0; r < 4; ++r)
                        __builtin_nontemporal_store(st.S[kt][ct][r], S_out + (size_t)slab_channel(kt, 4 * grp + r) * dv + slab_column(ct, n));
        }
        if (kSummary && col_tile == 0 && slab == 0 && n == 0) {
            float *gam = plan.gamma + ((size_t)seg * BH + slot_bh) * kK;
#pragma unroll
            for (int kt = 0; kt < 4; ++kt) *reinterpret_cast<floatx4_t *>(gam + slab_channel(kt, 4 * grp)) = decay[kt];
        }
    } else {
        // ------------------------------------------------------------------ value wavefront, tile = wave - 8
        const int tile = wave - 8;
        __builtin_amdgcn_s_setprio(PRIO_VALUE);
        StateLoads pf;            // tile `tile` of the next chunk to stage, all 128 columns
        StageLoads sl;            // kBlock: rows of x' and z for the next chunk to store
        unsigned char *feed = lds + kOffOb + 2 * kObBuf;
        if ((kStage & kStageFeed) && tile == 0 && lane < kColTile / 4)      // read back two or more barriers later
            *reinterpret_cast<floatx4_t *>(feed + 16 * lane) = *reinterpret_cast<const floatx4_t *>(g.d + (size_t)g.h * dv + g.j0 + 4 * lane);
        // Iteration `it`: stage the values of chunk `it`, store the outputs of chunk it-2 (finished by the state wavefronts in
        // iteration it-1), then request the stage inputs of chunk it-1 and the values of chunk it+2 into the registers just
        // freed.  Every request has most of an iteration to arrive.  Requests are unconditional (clamped rows).
        auto iteration = [&](int it, StateLoads &cur) {
            if (it < nchunks)
                stage_values<kBeta>(lds + kOffVt + (it & 1) * kVtBuf, tile, lane, cur, t_begin + it * kChunk, g.t_end);
            if (!kSummary && it >= 2) {
                unsigned char *ob = lds + kOffOb + (it & 1) * kObBuf;
                if (kBlock && it <= nchunks + 1) finish_outputs_block<kStage, 0, 2>(g, ob, tile, lane, sl, feed);

            }
            if (kBlock && !kSummary && nchunks > 0) stage_prefetch<kStage, 0, 2>(g, t_begin + (it - 1) * kChunk, t_begin, tile, lane, sl);
            if (it < nchunks) state_prefetch<kBeta>(g, t_begin + (it + 2) * kChunk, tile, lane, cur);
        };
        StateLoads pf_odd;
        if (nchunks > 0) {
            state_prefetch<kBeta>(g, t_begin, tile, lane, pf);
            state_prefetch<kBeta>(g, t_begin + kChunk, tile, lane, pf_odd);
        }
        const int last_it = nchunks + (kBlock ? 2 : 1);
        for (int it = 0;;) {
            iteration(it, pf);
            __syncthreads();
            if (++it > last_it) break;
            iteration(it, pf_odd);
            __syncthreads();
            if (++it > last_it) break;
        }
    }
}

// Entering state of every segment from the summary pass: slot 0 = S0 (or zero), and for s >= 1
// slot s <- gamma[s-1] .* slot[s-1] + slot[s] (the increment left there by the summary pass).  One thread per
// four adjacent state elements; the segments are walked in order.  With a packed batch cut on the device the thread
// first finds the slots of its sequence (the first one and how many) from the lengths before it.
__global__ __launch_bounds__(256) void segment_state_scan_kernel(const float *S0, SegmentPlan plan, int dv, size_t quads_per_slot,
                                                                 const int *__restrict__ cu_seqlens, int total_seqs, int total_tokens)
{
    const size_t e4 = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const size_t slot_elems = quads_per_slot * 4;
    size_t elem = e4 * 4;                                 // element index inside a slot: ((bh * 64) + n) * dv + column
    size_t first_slot = 0;
    int count = plan.nseg;
    if (plan.packed_cut) {
        // here a slot holds the H heads of ONE sequence and e4 runs over [sequence][slot element]
        const int b = (int)(e4 / quads_per_slot);
        if (b >= total_seqs) return;
        elem = (e4 % quads_per_slot) * 4;
        int first;
        packed_sequence_slots(cu_seqlens, b, total_tokens, plan.seg_tokens, first, count);
        first_slot = (size_t)first;
        if (first_slot >= (size_t)plan.nseg) return;         // only with a corrupt table: stay inside the slots
        count = min(count, plan.nseg - (int)first_slot);
        S0 = (S0 != nullptr) ? S0 + (size_t)b * slot_elems : nullptr;
    } else if (e4 >= quads_per_slot) {
        return;
    }
    const size_t row = elem / dv;                         // bh * 64 + n
    const size_t rows_per_slot = slot_elems / dv;
    float *slots = plan.slots + first_slot * slot_elems;
    const float *gamma = plan.gamma + first_slot * rows_per_slot;
    floatx4_t s = (S0 != nullptr) ? *reinterpret_cast<const floatx4_t *>(S0 + elem) : floatx4_t{0.f, 0.f, 0.f, 0.f};
    *reinterpret_cast<floatx4_t *>(slots + elem) = s;
    // eight segments at a time: their increments and decays are requested together, so that the walk costs one memory
    // latency per eight segments and not one per segment
    constexpr int kBatch = 8;
    for (int s0 = 1; s0 < count; s0 += kBatch) {
        floatx4_t inc[kBatch];
        float gmm[kBatch];
#pragma unroll
        for (int i = 0; i < kBatch; ++i) {
            const int sg = min(s0 + i, count - 1);          // past the end: the last segment again, not used
            inc[i] = *reinterpret_cast<const floatx4_t *>(slots + (size_t)sg * slot_elems + elem);
            gmm[i] = gamma[(size_t)(sg - 1) * rows_per_slot + row];
        }
#pragma unroll
        for (int i = 0; i < kBatch; ++i) {
            const int sg = s0 + i;
            if (sg < count) {
                s[0] = fmaf(gmm[i], s[0], inc[i][0]); s[1] = fmaf(gmm[i], s[1], inc[i][1]);
                s[2] = fmaf(gmm[i], s[2], inc[i][2]); s[3] = fmaf(gmm[i], s[3], inc[i][3]);
                *reinterpret_cast<floatx4_t *>(slots + (size_t)sg * slot_elems + elem) = s;
            }
        }
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

// A packed batch, whose lengths only the device knows, is cut when the caller asks for it: a fixed segment length, and
// the largest number of segments the batch can then have (every sequence adds at most one partial segment, an empty one
// holds one slot).  The segment length is the share of one compute unit when all of them work (one round of workgroups:
// measured against two, four and eight rounds of shorter segments and half a round of longer ones, 405 against 429, 460,
// 502 and 638 us on eight sequences of 32768 tokens in all), and at least eight chunks.
SplitShape choose_packed_cut(int N, int total_tokens, int H, int dv)
{
    const long long per_slot = (long long)H * (dv / kColTile);
    SplitShape none{1, ((total_tokens + kChunk - 1) / kChunk) * kChunk};
    // every workgroup finds its slot by walking the length table: kept to batches where that walk is short
    if (N <= 0 || N > kMaxCutSequences || per_slot == 0 || total_tokens < 16 * kChunk) return none;
    long long seg = ((long long)total_tokens * per_slot / 256 + kChunk - 1) / kChunk * kChunk;
    if (seg < 8 * kChunk) seg = 8 * kChunk;
    const long long slots = total_tokens / seg + N;
    if (slots < 2 || (slots * H + 8) * (dv / kColTile) > 2147483647LL) return none;      // the flat grid, rounded up to whole runs of eight
    return SplitShape{(int)slots, (int)seg};
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

size_t scan_mfma_packed_workspace_bytes(int N, int total_tokens, int H, int dv)
{
    const SplitShape sp = choose_packed_cut(N, total_tokens, H, dv);
    if (sp.nseg <= 1) return 0;
    return ((size_t)sp.nseg * H * kK * dv + (size_t)sp.nseg * H * kK) * sizeof(float);
}

namespace {

// The kernels use more than the default 64 KB of dynamic LDS: raise the limit once per kernel instance and device.
constexpr int kMaxDevices = 64;
template <bool kSummary, int kBeta, bool kGated, int kStage>
hipError_t allow_lds()
{
    static std::atomic<bool> done[kMaxDevices];
    int device = 0;
    hipError_t e = hipGetDevice(&device);
    if (e != hipSuccess) return e;
    if (device < 0 || device >= kMaxDevices) return hipErrorInvalidDevice;
    if (done[device].load(std::memory_order_acquire)) return hipSuccess;
    e = hipFuncSetAttribute(reinterpret_cast<const void *>(&scan_mfma_kernel<kSummary, kBeta, kGated, kStage>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes(kStage != 0));
    if (e == hipSuccess) done[device].store(true, std::memory_order_release);
    return e;
}

template <int kBeta, bool kGated, int kStage>
hipError_t launch_scan_mfma_typed(const ScanArgs &a)
{
    // a packed variable-length batch is cut only when the caller brought a workspace for it (its lengths live in device
    // memory, so the cut is made by the kernels); otherwise one segment that covers any length
    const bool packed = a.cu_seqlens != nullptr;
    const bool packed_cut = packed && a.workspace != nullptr && choose_packed_cut(a.B, a.T, a.H, a.dv).nseg > 1;
    const SplitShape sp = packed_cut ? choose_packed_cut(a.B, a.T, a.H, a.dv)
                          : packed   ? SplitShape{1, ((a.T + kChunk - 1) / kChunk) * kChunk}
                                     : choose_split(a.B, a.T, a.H, a.dv);
    const size_t bh = (size_t)a.B * a.H;
    SegmentPlan plan{sp.nseg, sp.seg_tokens, nullptr, nullptr, packed_cut};
    hipError_t attr = allow_lds<false, kBeta, kGated, kStage>();
    if (attr == hipSuccess && sp.nseg > 1) attr = allow_lds<true, kBeta, kGated, 0>();
    if (attr != hipSuccess) return attr;
    const dim3 block(kThreads);
    const unsigned col_tiles = (unsigned)(a.dv / kColTile);
    const void *gate_a = kGated ? a.z_g : static_cast<const void *>(a.log_alpha);
    const OutputStage no_stage{nullptr, nullptr, nullptr, 0};
    // dense cut: (batch, head) x column tile x segment; packed cut: one flat index over (slot, head, column tile)
    const auto packed_grid = [&](size_t pairs) { return dim3((unsigned)((pairs + 7) / 8 * 8 * col_tiles)); };      // see xcd_pair_mapping
    const dim3 cut_grid = packed_cut ? packed_grid((size_t)sp.nseg * a.H) : dim3((unsigned)bh, col_tiles, (unsigned)(sp.nseg - 1));
    if (sp.nseg > 1) {
        const size_t per_slot = (packed_cut ? (size_t)a.H : bh) * kK;        // state rows in a slot
        plan.slots = static_cast<float *>(a.workspace);
        plan.gamma = plan.slots + (size_t)sp.nseg * per_slot * a.dv;
        hipLaunchKernelGGL((scan_mfma_kernel<true, kBeta, kGated, 0>), cut_grid, block,
                           lds_bytes(false), a.stream, (const bf16_t *)a.q, (const bf16_t *)a.k, (const bf16_t *)a.v, gate_a,
                           (const bf16_t *)a.z_tau, a.beta, (const float *)nullptr, (bf16_t *)nullptr, (float *)nullptr, a.T, a.H, a.dv, plan,
                           packed_cut ? a.cu_seqlens : (const int *)nullptr, packed_cut ? a.T : 0, packed_cut ? a.B : 0, no_stage);
        const size_t quads = per_slot * a.dv / 4;                            // per slot; the packed walk has one thread set per sequence
        const size_t threads = packed_cut ? quads * a.B : quads;
        hipLaunchKernelGGL(segment_state_scan_kernel, dim3((unsigned)((threads + 255) / 256)), dim3(256), 0, a.stream, a.S0,
                           plan, a.dv, quads, a.cu_seqlens, a.B, a.T);
    }
    // dense: (batch, head) x column tile x segment; packed: one flat index (see the kernel)
    const bool flat_dense = !packed && sp.nseg == 1 && col_tiles > 1 && bh * col_tiles > 256;
    const dim3 grid = packed_cut ? cut_grid
                      : packed   ? packed_grid(bh)
                      : flat_dense ? dim3((unsigned)((bh + 7) / 8 * 8 * col_tiles)) : dim3((unsigned)bh, col_tiles, (unsigned)sp.nseg);
    hipLaunchKernelGGL((scan_mfma_kernel<false, kBeta, kGated, kStage>), grid, block, lds_bytes(kStage != 0),
                       a.stream, (const bf16_t *)a.q, (const bf16_t *)a.k, (const bf16_t *)a.v, gate_a, (const bf16_t *)a.z_tau, a.beta, a.S0,
                       (bf16_t *)a.o, a.S_T, a.T, a.H, a.dv, plan, a.cu_seqlens, a.T, a.B, kStage != 0 ? a.stage : no_stage);
    return hipGetLastError();
}

template <int kBeta, bool kGated>
hipError_t launch_scan_mfma_staged(const ScanArgs &a)
{
    switch ((a.stage.x_prime != nullptr ? kStageFeed : 0) | (a.stage.z_gate != nullptr ? kStageGate : 0)) {
    case 0: return launch_scan_mfma_typed<kBeta, kGated, 0>(a);
    case kStageFeed: return launch_scan_mfma_typed<kBeta, kGated, kStageFeed>(a);
    case kStageGate: return launch_scan_mfma_typed<kBeta, kGated, kStageGate>(a);
    default: return launch_scan_mfma_typed<kBeta, kGated, kStageFeed | kStageGate>(a);
    }
}

}  // namespace

// The state entering every one of `nseg` segments of `seg_tokens` tokens (a multiple of 64) of a dense batch, for the
// backward pass cut along the sequence: summary pass over the first nseg-1 segments, then the chain over the segments.
// slots: [nseg][B*H][64][dv] fp32, gamma: [nseg-1][B*H][64] fp32 (the segment decays); beta: fp32 values or NULL, or
// (beta_preact) bf16 pre-activations.
namespace {

template <int kBeta>
hipError_t launch_segment_states_typed(const void *k, const void *v, const float *log_alpha, const void *beta, const float *S0,
                                       int B, int T, int H, int dv, int nseg, int seg_tokens, float *slots, float *gamma,
                                       const int *cu_seqlens, hipStream_t stream)
{
    const bool packed_cut = cu_seqlens != nullptr;
    const size_t bh = (size_t)B * H;
    SegmentPlan plan{nseg, seg_tokens, slots, gamma, packed_cut};
    const hipError_t attr = allow_lds<true, kBeta, false, 0>();
    if (attr != hipSuccess) return attr;
    const unsigned col_tiles = (unsigned)(dv / kColTile);
    const dim3 grid = packed_cut ? dim3((unsigned)(((size_t)nseg * H + 7) / 8 * 8 * col_tiles))      // see xcd_pair_mapping
                                 : dim3((unsigned)bh, col_tiles, (unsigned)(nseg - 1));
    hipLaunchKernelGGL((scan_mfma_kernel<true, kBeta, false, 0>), grid,
                       dim3(kThreads), lds_bytes(false), stream, (const bf16_t *)nullptr, (const bf16_t *)k, (const bf16_t *)v,
                       static_cast<const void *>(log_alpha), (const bf16_t *)nullptr, beta,
                       (const float *)nullptr, (bf16_t *)nullptr, (float *)nullptr, T, H, dv, plan, cu_seqlens, packed_cut ? T : 0,
                       packed_cut ? B : 0, OutputStage{nullptr, nullptr, nullptr, 0});
    const size_t quads = (packed_cut ? (size_t)H : bh) * kK * dv / 4;      // per slot; the packed walk has one thread set per sequence
    const size_t threads = packed_cut ? quads * B : quads;
    hipLaunchKernelGGL(segment_state_scan_kernel, dim3((unsigned)((threads + 255) / 256)), dim3(256), 0, stream, S0, plan, dv, quads,
                       cu_seqlens, B, T);
    return hipGetLastError();
}

}  // namespace

// cu_seqlens != NULL: a packed batch of B sequences with T tokens in all, cut by the kernels into segments of seg_tokens
// tokens; nseg is then the largest number of segments the batch can have and the slots are [nseg][H][64][dv], gamma
// [nseg][H][64].
hipError_t launch_scan_segment_states(const void *k, const void *v, const float *log_alpha, const void *beta, bool beta_preact,
                                      const float *S0, int B, int T, int H, int dv, int nseg, int seg_tokens, float *slots,
                                      float *gamma, hipStream_t stream, const int *cu_seqlens)
{
    if (nseg < 2 || seg_tokens % kChunk != 0 || dv % kColTile != 0 || (beta_preact && beta == nullptr)) return hipErrorInvalidValue;
    if (beta == nullptr) return launch_segment_states_typed<kBetaNone>(k, v, log_alpha, beta, S0, B, T, H, dv, nseg, seg_tokens, slots, gamma, cu_seqlens, stream);
    return beta_preact ? launch_segment_states_typed<kBetaPreact>(k, v, log_alpha, beta, S0, B, T, H, dv, nseg, seg_tokens, slots, gamma, cu_seqlens, stream)
                       : launch_segment_states_typed<kBetaValues>(k, v, log_alpha, beta, S0, B, T, H, dv, nseg, seg_tokens, slots, gamma, cu_seqlens, stream);
}

hipError_t launch_scan_mfma(const ScanArgs &a)
{
    if ((long long)a.B * a.H == 0) return hipSuccess;
    if (a.T == 0 && (a.S_T == nullptr || a.S_T == a.S0)) return hipSuccess;
    // the gated form takes the value gate as a pre-activation too, or none at all
    if (a.gated()) return a.beta != nullptr ? launch_scan_mfma_staged<kBetaPreact, true>(a) : launch_scan_mfma_staged<kBetaNone, true>(a);
    if (a.beta == nullptr) return launch_scan_mfma_staged<kBetaNone, false>(a);
    return a.beta_preact ? launch_scan_mfma_staged<kBetaPreact, false>(a) : launch_scan_mfma_staged<kBetaValues, false>(a);
}

}  // namespace rodimus
