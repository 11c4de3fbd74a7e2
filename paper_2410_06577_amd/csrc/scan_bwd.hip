// Backward pass of the chunkwise scan (training use of the block, paper Sec. 3.1.3; the algebra is the reverse-mode
// differentiation of the chunkwise form of the appendix, with a 16-token tile as the chunk).  bf16 I/O, dk = 64,
// dv = 128 or 256.  With l_t the running sum of log_alpha inside a tile, A_t = exp(l_t), u_t = beta_t .* v_t and
// w[t,i] = exp(l_t - l_i) (always <= 1 for i <= t: no quotient is ever formed):
//
//   forward sweep (sweep_dq), state S entering the tile:
//       dP[t,i] = do_t . u_i  (i <= t)
//       dq_t    = A_t .* (do_t S^T) + sum_{i<=t} dP[t,i] (k_i .* w[t,i])
//       S      <- diag(A_16) S + sum_i (k_i .* exp(l_16 - l_i))^T u_i
//   reverse sweep (sweep_dkv), cotangent G of the state leaving the tile:
//       P[t,i]  = sum_n q_t k_i w[t,i]  (i <= t)
//       du_i    = sum_{t>=i} P[t,i] do_t + (k_i .* exp(l_16 - l_i)) G
//       dk_i    = exp(l_16 - l_i) .* (u_i G^T) + sum_{t>=i} dP[t,i] (q_t .* w[t,i])
//       G      <- diag(A_16) G + sum_t (q_t .* A_t)^T do_t
//       dv = beta .* du, dbeta = v .* du (with the gate given as its pre-activation z, beta = sigmoid(z):
//       dz = dbeta .* beta (1 - beta)), dS0 = G after the first tile
//   gates: dlog_alpha_t = sum_{s>=t} (q_s .* dq_s - k_s .* dk_s) + rowsum(S_T .* dS_T): every pair (i < t <= s) that the
//       gate of step t decays appears once in q_s .* dq_s and not in k .* dk of a step >= t, so the reverse running
//       sum of the difference is the gate's cotangent; it is formed from the fp32 values before dq, dk are rounded
//       (scan_bwd_gate_kernel, from q .* dq and k .* dk left in the workspace by the two sweeps).
// The two sweeps do not depend on each other and run concurrently as the two halves of one launch.
//
// log_alpha is clamped at -128 per step (exp(-128) is zero in fp32), which keeps every l finite.
// The contractions run on MFMA with bf16 operands and fp32 accumulation.  The tile-local terms use w[t,i] = A_t / A_i
// (q .* A and k ./ A as operands) when the tile's total decay A_16 is at least 2^-80 in every channel concerned, so
// that 1 / A_i cannot overflow; otherwise (a hard reset or very strong decay inside the tile) they are evaluated pair
// by pair on the vector ALUs in fp32 from exp(l_t - l_i) <= 1.  The choice is uniform per tile.
#include <atomic>

#include "internal.h"

namespace rodimus {

namespace {

constexpr int kK = 64;
constexpr int kTile = 16;
// One wavefront of the reverse sweep per 32 value columns: 4 wavefronts (dv = 128) or 8 (dv = 256); the forward sweep
// computes with 4 wavefronts.
template <int DV> struct BwdShape {
    static constexpr int kWaves = DV / 32;
    static constexpr int kThreads = 64 * kWaves;
    // The sweeps kernel adds half as many helper wavefronts: in the reverse sweep they load and stage the tile inputs and
    // write dv and dbeta, which takes that work and its registers off the wavefronts that carry G (three wavefronts per
    // SIMD instead of two); in the forward sweep (dv = 256) all wavefronts behind the four computing ones fetch, stage and
    // store, so that those keep no loads in registers (dv = 128: the computing wavefronts stage themselves and the helpers
    // only take part in the barriers).
    static constexpr int kHelpers = kWaves / 2;
    static constexpr int kSweepThreads = 64 * (kWaves + kHelpers);
};
constexpr float kMinLogAlpha = -128.f;
constexpr float kSafeTileLog = -55.f;      // ln(2^-80) = -55.45: above it 1 / A_i stays below 2^80
// The gate cotangent is a reverse running sum over the sequence; the sequence is cut into kGateParts runs of whole
// tiles, the sweeps leave the sum of q .* dq (k .* dk) over every run, and the gate kernel starts each run from the
// totals of the later ones.
constexpr int kGateParts = 32;
__host__ __device__ inline int gate_part_tiles(int T) { return (((T + kTile - 1) / kTile) + kGateParts - 1) / kGateParts; }

// How a call is cut along the sequence.  Slots: [segment][B*H][64][dv] fp32.  A packed batch is cut by the kernels
// (`packed_cut`, see locate_packed_slot): `nseg` is then the largest number of segments the batch can have, the slots are
// [slot][H][64][dv], and the grids run over (head, slot) instead of ((batch, head), segment).
struct BwdSegments {
    int nseg;                    // 1: whole sequences, no slots
    int seg_tokens;              // a multiple of 64
    const float *S_slots;        // state entering each segment
    const float *G_slots;        // cotangent of the state leaving each segment
    bool packed_cut;
    int nseq;                    // packed_cut: sequences in the batch
};

// What one workgroup of the sweeps or of the gate kernel works on: (x, s) = ((batch, head), segment) of the grid, or
// (head, slot) for a packed batch cut by the kernels.  `bh` indexes the caller's state tensors, `unit` the per-unit arrays
// and the slots (unit >= bh always, so slot pointers may be formed as base + (unit - bh) * state size and then indexed by bh).
struct BwdUnit {
    int bh;
    size_t unit;
    SeqSpan span;
    bool first_seg;
};

// packed_cut only; false: the slot lies past the batch's last segment (the grid covers the largest possible number)
__device__ __forceinline__ bool packed_cut_unit(int h, int slot, int T, int H, const int *cu_seqlens, const BwdSegments &segs, BwdUnit &u)
{
    PackedSlot ps;
    if (!locate_packed_slot(cu_seqlens, segs.nseq, T, segs.seg_tokens, slot, ps)) return false;
    const int begin = ps.j * segs.seg_tokens;
    u.bh = ps.b * H + h;
    u.unit = (size_t)slot * H + h;
    u.span = SeqSpan{(size_t)ps.first + (size_t)begin, max(min(segs.seg_tokens, ps.len - begin), 0)};
    u.first_seg = ps.j == 0;
    return true;
}

// The tokens of segment `seg` of a sequence (empty beyond its end)
__device__ __forceinline__ SeqSpan segment_span(SeqSpan s, const BwdSegments &sg, int seg)
{
    if (sg.nseg <= 1) return s;
    const int begin = seg * sg.seg_tokens;
    return SeqSpan{s.first + (size_t)begin, max(min(sg.seg_tokens, s.length - begin), 0)};
}

// Value columns are stored in LDS in a permuted order inside every group of 32: column 32s + 16h + 4g + e sits at
// position 32s + 8g + 4h + e.  A 16-byte read at position 32s + 8g then delivers exactly the 8 columns that lane
// group g of an MFMA accumulator pair (column tiles 2s and 2s+1) holds, so the accumulators can serve as the other
// operand of a contraction over columns without being moved.
__device__ __forceinline__ int col_position(int col)
{
    return (col & ~31) | (((col >> 2) & 3) << 3) | (((col >> 4) & 1) << 2) | (col & 3);
}

// x = hi + lo with both parts bf16: products of split operands (hi*hi + hi*lo + lo*hi) are accurate to ~2^-16.  Used for
// the tile-local terms of dq and dk, whose difference feeds the running sum behind dlog_alpha and must cancel closely.
__device__ __forceinline__ void split_bf16(float x, float &hi, float &lo)
{
    hi = (float)(bf16_t)x;
    lo = x - hi;
}

template <int DV> struct BwdLayout {
    static constexpr int kRowBytes = DV * 2 + 16;                 // padded token row of bf16 values (bank spread)
    static constexpr int kPieces = DV / 8;                        // 16-byte pieces per token row
    static constexpr int kPerThread = kTile * kPieces / BwdShape<DV>::kThreads;   // (token, piece) pairs per thread: 1
    static_assert(kPerThread == 1, "one 16-byte piece of v, do (and beta) per thread");
};

// One thread's share of a tile's global inputs, requested one tile ahead.
template <int DV> struct TileLoads {
    uint4 qk;                                          // threads 0..127: q piece, 128..255: k piece
    floatx4_t la;                                      // dv = 128: every thread; dv = 256: threads 256..511
    uint4 v[BwdLayout<DV>::kPerThread], d_o[BwdLayout<DV>::kPerThread];
    floatx4_t beta[BwdLayout<DV>::kPerThread][2];
};

// Input pointers of one (batch, head), already advanced to its first token and its head: token t of the sequence is at
// element offset t * H * width.  t * H fits 32 bits; the byte offset is formed in 64 bits.
struct BwdGeometry {
    const bf16_t *q, *k, *v, *d_o;
    const float *la;
    const void *beta;            // fp32 gate values or bf16 pre-activations, not advanced: element offset beta_row0 + ...
    size_t beta_row0;
    int T, H;
    __device__ BwdGeometry(const bf16_t *q_, const bf16_t *k_, const bf16_t *v_, const bf16_t *do_, const float *la_,
                           const void *beta_, size_t first_token, int h, int T_, int H_, int dv)
        : T(T_), H(H_)
    {
        const size_t row0 = first_token * H_ + h;
        q = q_ + row0 * kK; k = k_ + row0 * kK; la = la_ + row0 * kK;
        v = v_ + row0 * dv; d_o = do_ + row0 * dv;
        beta = beta_;
        beta_row0 = row0 * dv;
    }
    // token index (clamped to the sequence) times H
    __device__ __forceinline__ unsigned row(int t) const { return (unsigned)min(t, T - 1) * (unsigned)H; }
};

__device__ __forceinline__ void unpack8(const uint4 &w, float (&x)[8])
{
    x[0] = bf16_lo(w.x); x[1] = bf16_hi(w.x); x[2] = bf16_lo(w.y); x[3] = bf16_hi(w.y);
    x[4] = bf16_lo(w.z); x[5] = bf16_hi(w.z); x[6] = bf16_lo(w.w); x[7] = bf16_hi(w.w);
}

// The value gate of eight columns as it is loaded: fp32 values (two 16-byte pieces) or, with kZBeta, the bf16
// pre-activations of the gate (one 16-byte piece, raw[1] unused), and its eight values from that (paper Sec. 3.1.2:
// beta_hat = sigmoid(z_beta)).
template <bool kZBeta>
__device__ __forceinline__ void load_gate8(const BwdGeometry &g, size_t off, floatx4_t (&raw)[2])
{
    if (kZBeta) {
        raw[0] = *reinterpret_cast<const floatx4_t *>(static_cast<const bf16_t *>(g.beta) + g.beta_row0 + off);
    } else {
        const float *p = static_cast<const float *>(g.beta) + g.beta_row0 + off;
        raw[0] = *reinterpret_cast<const floatx4_t *>(p);
        raw[1] = *reinterpret_cast<const floatx4_t *>(p + 4);
    }
}
template <bool kZBeta>
__device__ __forceinline__ void gate_values8(const floatx4_t (&raw)[2], float (&gate)[8])
{
    if (kZBeta) {
        float z[8];
        unpack8(__builtin_bit_cast(uint4, raw[0]), z);
#pragma unroll
        for (int e = 0; e < 8; ++e) gate[e] = sigmoid_short(z[e]);
    } else {
#pragma unroll
        for (int e = 0; e < 4; ++e) { gate[e] = raw[0][e]; gate[4 + e] = raw[1][e]; }
    }
}

template <int DV, bool kZBeta>
__device__ __forceinline__ void tile_prefetch(const BwdGeometry &g, int t0, int tid, bool has_beta, TileLoads<DV> &p)
{
    using L = BwdLayout<DV>;
    constexpr bool kWide = BwdShape<DV>::kThreads == 512;      // the log_alpha pieces then go to the upper 256 threads
    if (tid < 256) {
        const int tok = (tid & 127) >> 3, piece = tid & 7;
        p.qk = *reinterpret_cast<const uint4 *>((tid < 128 ? g.q : g.k) + (size_t)g.row(t0 + tok) * kK + 8 * piece);
    }
    if (!kWide || tid >= 256) {
        const int tok = (tid & 255) >> 4, piece = tid & 15;
        p.la = *reinterpret_cast<const floatx4_t *>(g.la + (size_t)g.row(t0 + tok) * kK + 4 * piece);
    }
#pragma unroll
    for (int u = 0; u < L::kPerThread; ++u) {
        const int id = tid, tok = id / L::kPieces, piece = id % L::kPieces;
        const size_t off = (size_t)g.row(t0 + tok) * DV + 8 * piece;
        p.v[u] = *reinterpret_cast<const uint4 *>(g.v + off);
        p.d_o[u] = *reinterpret_cast<const uint4 *>(g.d_o + off);
        if (has_beta) load_gate8<kZBeta>(g, off, p.beta[u]);
    }
}

// Tile inputs from registers into LDS: q, k, log_alpha (clamped) as fp32 [16][64]; u = beta .* v and do as bf16 rows
// with permuted columns.  Rows at or beyond T become q = k = u = do = 0, log_alpha = 0.
template <int DV, bool kZBeta>
__device__ __forceinline__ void tile_stage(const TileLoads<DV> &p, int t0, int T, int tid, bool has_beta, float *qs, float *ks,
                                           float *ls, unsigned char *us, unsigned char *ds)
{
    using L = BwdLayout<DV>;
    constexpr bool kWide = BwdShape<DV>::kThreads == 512;
    if (tid < 256) {
        const int tok = (tid & 127) >> 3, piece = tid & 7;
        const bool valid = t0 + tok < T;
        float x[8];
        unpack8(p.qk, x);
        float *dst = (tid < 128 ? qs : ks) + tok * kK + 8 * piece;
#pragma unroll
        for (int e = 0; e < 8; ++e) dst[e] = valid ? x[e] : 0.f;
    }
    if (!kWide || tid >= 256) {
        const int tok = (tid & 255) >> 4, piece = tid & 15;
        const bool valid = t0 + tok < T;
#pragma unroll
        for (int e = 0; e < 4; ++e) ls[tok * kK + 4 * piece + e] = valid ? fmaxf(p.la[e], kMinLogAlpha) : 0.f;
    }
#pragma unroll
    for (int u = 0; u < L::kPerThread; ++u) {
        const int id = tid, tok = id / L::kPieces, piece = id % L::kPieces;
        const bool valid = t0 + tok < T;
        float x[8], d[8];
        unpack8(p.v[u], x);
        unpack8(p.d_o[u], d);
        if (has_beta) {
            float gate[8];
            gate_values8<kZBeta>(p.beta[u], gate);
#pragma unroll
            for (int e = 0; e < 8; ++e) x[e] *= gate[e];
        }
#pragma unroll
        for (int e = 0; e < 8; ++e) { x[e] = valid ? x[e] : 0.f; d[e] = valid ? d[e] : 0.f; }
        // columns 8*piece .. +3 and +4 .. +7 are two 8-byte units at permuted positions
#pragma unroll
        for (int half = 0; half < 2; ++half) {
            const int pos = col_position(8 * piece + 4 * half);
            const uint2 wu = {pack_bf16x2(x[4 * half], x[4 * half + 1]), pack_bf16x2(x[4 * half + 2], x[4 * half + 3])};
            const uint2 wd = {pack_bf16x2(d[4 * half], d[4 * half + 1]), pack_bf16x2(d[4 * half + 2], d[4 * half + 3])};
            *reinterpret_cast<uint2 *>(us + tok * L::kRowBytes + pos * 2) = wu;
            *reinterpret_cast<uint2 *>(ds + tok * L::kRowBytes + pos * 2) = wd;
        }
    }
}

// ---- the reverse sweep's helper wavefronts: thread `hid` of 32 * kWaves takes two (token, piece) pairs of v, do, beta and
// one (dv = 256) or two (dv = 128) pieces each of q / k and log_alpha
template <int DV> struct HelperLoads {
    uint4 qk[2];
    floatx4_t la[2];
    uint4 v[2], d_o[2];
    floatx4_t beta[2][2];
};

template <int DV, bool kZBeta>
__device__ __forceinline__ void helper_prefetch(const BwdGeometry &g, int t0, int hid, bool has_beta, HelperLoads<DV> &p)
{
    using L = BwdLayout<DV>;
    constexpr int kHelp = 32 * BwdShape<DV>::kWaves;
#pragma unroll
    for (int s = 0; s < 2; ++s) {
        const int idx = hid + s * kHelp;
        if (s * kHelp < 256) {                             // 256 pieces of q and k together, 256 of log_alpha
            const int tok = (idx & 127) >> 3, piece = idx & 7;
            p.qk[s] = *reinterpret_cast<const uint4 *>((idx < 128 ? g.q : g.k) + (size_t)g.row(t0 + tok) * kK + 8 * piece);
            p.la[s] = *reinterpret_cast<const floatx4_t *>(g.la + (size_t)g.row(t0 + (idx >> 4)) * kK + 4 * (idx & 15));
        }
        const int tok = idx / L::kPieces, piece = idx % L::kPieces;
        const size_t off = (size_t)g.row(t0 + tok) * DV + 8 * piece;
        p.v[s] = *reinterpret_cast<const uint4 *>(g.v + off);
        p.d_o[s] = *reinterpret_cast<const uint4 *>(g.d_o + off);
        if (has_beta) load_gate8<kZBeta>(g, off, p.beta[s]);
    }
}

// The same LDS image as tile_stage leaves
template <int DV, bool kZBeta>
__device__ __forceinline__ void helper_stage(const HelperLoads<DV> &p, int t0, int T, int hid, bool has_beta, float *qs, float *ks,
                                             float *ls, unsigned char *us, unsigned char *ds)
{
    using L = BwdLayout<DV>;
    constexpr int kHelp = 32 * BwdShape<DV>::kWaves;
#pragma unroll
    for (int s = 0; s < 2; ++s) {
        const int idx = hid + s * kHelp;
        if (s * kHelp < 256) {
            {
                const int tok = (idx & 127) >> 3, piece = idx & 7;
                const bool valid = t0 + tok < T;
                float x[8];
                unpack8(p.qk[s], x);
                float *dst = (idx < 128 ? qs : ks) + tok * kK + 8 * piece;
#pragma unroll
                for (int e = 0; e < 8; ++e) dst[e] = valid ? x[e] : 0.f;
            }
            {
                const int tok = idx >> 4, piece = idx & 15;
                const bool valid = t0 + tok < T;
#pragma unroll
                for (int e = 0; e < 4; ++e) ls[tok * kK + 4 * piece + e] = valid ? fmaxf(p.la[s][e], kMinLogAlpha) : 0.f;
            }
        }
        const int tok = idx / L::kPieces, piece = idx % L::kPieces;
        const bool valid = t0 + tok < T;
        float x[8], d[8];
        unpack8(p.v[s], x);
        unpack8(p.d_o[s], d);
        if (has_beta) {
            float gate[8];
            gate_values8<kZBeta>(p.beta[s], gate);
#pragma unroll
            for (int e = 0; e < 8; ++e) x[e] *= gate[e];
        }
#pragma unroll
        for (int e = 0; e < 8; ++e) { x[e] = valid ? x[e] : 0.f; d[e] = valid ? d[e] : 0.f; }
#pragma unroll
        for (int half = 0; half < 2; ++half) {
            const int pos = col_position(8 * piece + 4 * half);
            const uint2 wu = {pack_bf16x2(x[4 * half], x[4 * half + 1]), pack_bf16x2(x[4 * half + 2], x[4 * half + 3])};
            const uint2 wd = {pack_bf16x2(d[4 * half], d[4 * half + 1]), pack_bf16x2(d[4 * half + 2], d[4 * half + 3])};
            *reinterpret_cast<uint2 *>(us + tok * L::kRowBytes + pos * 2) = wu;
            *reinterpret_cast<uint2 *>(ds + tok * L::kRowBytes + pos * 2) = wd;
        }
    }
}

// =========================================================================================================
// Forward sweep: dq (and q .* dq in fp32 for the gate cotangent, and rowsum(S_T .* dS_T))
// =========================================================================================================
// One workgroup per (batch, head); wavefront w owns key channels 16w .. 16w+15: its slab of the state is kept
// transposed in MFMA accumulators (lane = channel, registers = value columns), so that do_t S^T contracts over the
// columns without any exchange between wavefronts.
template <int DV, bool kZBeta>
__device__ __forceinline__ void sweep_dq(
    const bf16_t *__restrict__ q, const bf16_t *__restrict__ k, const bf16_t *__restrict__ v,
    const float *__restrict__ log_alpha, const void *__restrict__ beta, const float *__restrict__ S0,
    const bf16_t *__restrict__ d_o, const float *__restrict__ dS_T, bf16_t *__restrict__ dq,
    float *__restrict__ qdq, float *__restrict__ gate_const, float *__restrict__ qtot, int T, int H,
    const int *__restrict__ cu_seqlens, const BwdSegments &segs)
{
    using L = BwdLayout<DV>;
    constexpr int kColTiles = DV / 16, kSteps = DV / 32;
    // LDS (the workgroup's dynamic allocation, sized for the reverse sweep): tile inputs, then this sweep's buffers
    extern __shared__ __align__(16) unsigned char lds_raw[];
    float *qs = reinterpret_cast<float *>(lds_raw), *ks = qs + kTile * kK, *ls = ks + kTile * kK;
    unsigned char *us = reinterpret_cast<unsigned char *>(ls + kTile * kK), *ds = us + kTile * L::kRowBytes;
    float (*dPw)[kTile][kTile + 4] = reinterpret_cast<float (*)[kTile][kTile + 4]>(ds + kTile * L::kRowBytes);     // [4][16][16], rows padded: the four token groups write different banks
    float *qdq_s = reinterpret_cast<float *>(dPw + 4);
    bf16_t *dq_s = reinterpret_cast<bf16_t *>(qdq_s + kTile * kK);

    // wavefronts 0..3 compute (16 key channels each); any further wavefronts of the workgroup only fetch and stage
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const bool computes = wave < 4;
    const int c = lane & 15, tg = lane >> 4;          // vector-ALU role: channel 16*wave + c, tokens 4tg .. 4tg+3
    const int ch = 16 * (wave & 3) + c;
    int bh = blockIdx.x;
    const int seg = blockIdx.y;
    BwdUnit u;
    if (segs.packed_cut) {
        if (!packed_cut_unit(blockIdx.x, seg, T, H, cu_seqlens, segs, u)) return;      // the whole workgroup, before any barrier
        bh = u.bh;
    } else {
        if (cu_seqlens != nullptr)                                // packed batch: sequences by descending length (small batches)
            bh = sequence_by_length_rank(cu_seqlens, (int)gridDim.x / H, T, bh / H, reinterpret_cast<int *>(lds_raw)) * H + bh % H;
        u = BwdUnit{bh, (size_t)seg * gridDim.x + bh, segment_span(seq_span(bh / H, T, cu_seqlens), segs, seg), seg == 0};
    }
    const size_t unit = u.unit;                                   // (segment, batch, head): index of the per-unit totals
    const bool has_beta = beta != nullptr;
    const SeqSpan span = u.span;
    T = span.length;
    const BwdGeometry g(q, k, v, d_o, log_alpha, beta, span.first, bh % H, T, H, DV);
    const size_t row0 = span.first * H + bh % H;                  // outputs: same layout as the inputs
    if (segs.nseg > 1) {                                          // the segment's own boundary states
        const size_t slot = (unit - (size_t)bh) * kK * DV;        // state_base below adds the (batch, head)
        S0 = segs.S_slots + slot;
        dS_T = segs.G_slots + slot;
    }

    // state slab, transposed: acc[ct][r] = S[ch][16ct + 4tg + r]
    floatx4_t acc[kColTiles];
    const size_t state_base = (size_t)bh * kK * DV + (size_t)ch * DV;
#pragma unroll
    for (int ct = 0; ct < kColTiles; ++ct)
        acc[ct] = (S0 != nullptr && computes) ? *reinterpret_cast<const floatx4_t *>(S0 + state_base + 16 * ct + 4 * tg)
                                              : floatx4_t{0.f, 0.f, 0.f, 0.f};

    const int ntiles = (T + kTile - 1) / kTile;
    const int part_tiles = gate_part_tiles(T);
    int run_index = 0, run_last = part_tiles - 1;      // the current run of tiles and its last tile
    float qpart = 0.f;                                 // sum of q .* dq over this lane's tokens of the current run of tiles
    // coalesced stores of a finished tile's dq (bf16) and q .* dq (fp32) from the staging buffers, by 256 threads
    auto store_tile = [&](int t0, int stid) {
        const int tok = stid >> 4, piece = stid & 15;
        if (stid < 256 && t0 + tok < T) {
            const size_t row = row0 + (size_t)((unsigned)(t0 + tok) * (unsigned)H);
            *reinterpret_cast<floatx4_t *>(qdq + row * kK + 4 * piece) = *reinterpret_cast<const floatx4_t *>(qdq_s + tok * kK + 4 * piece);
            if (piece < 8)
                *reinterpret_cast<uint4 *>(dq + row * kK + 8 * piece) = *reinterpret_cast<const uint4 *>(dq_s + tok * kK + 8 * piece);
        }
    };

    // With 512 threads behind the four computing wavefronts (dv = 256) those fetch, stage and store, and the computing
    // wavefronts keep no loads in registers; otherwise (dv = 128) the computing wavefronts stage as well and the helper
    // wavefronts of the kernel only take part in the barriers.
    constexpr bool kSplitRoles = BwdShape<DV>::kSweepThreads >= 256 + BwdShape<DV>::kThreads;
    if (kSplitRoles && wave >= 4) {
        const int stid = tid - 256;
        TileLoads<DV> pf;
        if (ntiles > 0) tile_prefetch<DV, kZBeta>(g, 0, stid, has_beta, pf);
        for (int it = 0; it < ntiles; ++it) {
            const int t0 = it * kTile;
            __syncthreads();                               // the previous tile is computed: its results are staged, its inputs free
            tile_stage<DV, kZBeta>(pf, t0, T, stid, has_beta, qs, ks, ls, us, ds);
            tile_prefetch<DV, kZBeta>(g, t0 + kTile, stid, has_beta, pf);   // clamped addresses; masked when staged
            // the stores come after the next tile's loads are requested: memory operations of a wavefront retire in order and
            // stores retire slowly, so a load must not queue behind a fresh store
            if (it > 0) store_tile(t0 - kTile, stid);
            __syncthreads();
        }
        __syncthreads();
        if (ntiles > 0) store_tile((ntiles - 1) * kTile, stid);
        return;
    }
    TileLoads<DV> pf;
    const bool stages = !kSplitRoles && tid < BwdShape<DV>::kThreads;
    if (ntiles > 0 && stages) tile_prefetch<DV, kZBeta>(g, 0, tid, has_beta, pf);

    for (int it = 0; it < ntiles; ++it) {
        const int t0 = it * kTile;
        __syncthreads();                                   // the previous tile is computed: its results are staged, its inputs free
        if (stages) {
            if (it > 0) store_tile(t0 - kTile, tid);
            tile_stage<DV, kZBeta>(pf, t0, T, tid, has_beta, qs, ks, ls, us, ds);
            tile_prefetch<DV, kZBeta>(g, t0 + kTile, tid, has_beta, pf);    // clamped addresses; masked when staged
        }
        __syncthreads();
        if (!computes) continue;          // wavefront-uniform; the two barriers above are reached by every wavefront

        // ---- this lane's channel: running sums of log_alpha, keys
        float lsum[kTile], kk[kTile];
        {
            float run = 0.f;
#pragma unroll
            for (int i = 0; i < kTile; ++i) {
                run += ls[i * kK + ch];
                lsum[i] = run;
                kk[i] = ks[i * kK + ch];
            }
        }
        float lt[4];                                       // l of this lane's own four tokens
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            lt[r] = lsum[r];
#pragma unroll
            for (int gsel = 1; gsel < 4; ++gsel) lt[r] = (tg == gsel) ? lsum[4 * gsel + r] : lt[r];
        }
        const float a_tile = __expf(lsum[kTile - 1]);      // A_16

        // ---- MFMA operands: rows of do (A operand, M = token) for every 32-column step
        bf16x8_t a_do[kSteps];
#pragma unroll
        for (int s = 0; s < kSteps; ++s)
            a_do[s] = *reinterpret_cast<const bf16x8_t *>(ds + c * L::kRowBytes + (32 * s + 8 * tg) * 2);
        // dP[t][i] = do_t . u_i, kept for i <= t
        {
            floatx4_t d = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int s = 0; s < kSteps; ++s) {
                const bf16x8_t b_u = *reinterpret_cast<const bf16x8_t *>(us + c * L::kRowBytes + (32 * s + 8 * tg) * 2);
                d = mfma_k32(a_do[s], b_u, d);
            }
            // lane (i = c, token group tg) holds t = 4tg + r
#pragma unroll
            for (int r = 0; r < 4; ++r) dPw[wave][4 * tg + r][c] = (c <= 4 * tg + r) ? d[r] : 0.f;
        }
        // do_t S^T for this wavefront's 16 channels: B operand = the state slab, straight from the accumulators
        floatx4_t dqt = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int s = 0; s < kSteps; ++s) {
            const floatx4_t lo = acc[2 * s], hi = acc[2 * s + 1];
            const uint4 w = {pack_bf16x2(lo[0], lo[1]), pack_bf16x2(lo[2], lo[3]), pack_bf16x2(hi[0], hi[1]), pack_bf16x2(hi[2], hi[3])};
            dqt = mfma_k32(a_do[s], __builtin_bit_cast(bf16x8_t, w), dqt);
        }
        // lane (channel c, token group tg) now holds (do_t S^T)[ch] for t = 4tg + r
        // tile-local term: with a safe total decay, sum_i dP[t,i] k_i exp(l_t - l_i) = A_t .* (dP (k ./ A)) joins the same
        // accumulator (one MFMA); otherwise it is summed pair by pair below
        const bool pairwise = __any(lsum[kTile - 1] < kSafeTileLog);
        if (!pairwise) {
            float kq_hi[4], kq_lo[4], dp_hi[4], dp_lo[4];
            const floatx4_t dp4 = *reinterpret_cast<const floatx4_t *>(&dPw[wave][c][4 * tg]);     // dP[t = c][i = 4tg ..]
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                float kv = kk[r];
#pragma unroll
                for (int gsel = 1; gsel < 4; ++gsel) kv = (tg == gsel) ? kk[4 * gsel + r] : kv;
                split_bf16(kv * __expf(-lt[r]), kq_hi[r], kq_lo[r]);
                split_bf16(dp4[r], dp_hi[r], dp_lo[r]);
            }
            const uint2 b_hi = {pack_bf16x2(kq_hi[0], kq_hi[1]), pack_bf16x2(kq_hi[2], kq_hi[3])};
            const uint2 b_lo = {pack_bf16x2(kq_lo[0], kq_lo[1]), pack_bf16x2(kq_lo[2], kq_lo[3])};
            const uint2 a_hi = {pack_bf16x2(dp_hi[0], dp_hi[1]), pack_bf16x2(dp_hi[2], dp_hi[3])};
            const uint2 a_lo = {pack_bf16x2(dp_lo[0], dp_lo[1]), pack_bf16x2(dp_lo[2], dp_lo[3])};
            dqt = mfma_k16(a_lo, b_hi, dqt);
            dqt = mfma_k16(a_hi, b_lo, dqt);
            dqt = mfma_k16(a_hi, b_hi, dqt);
        }

        // ---- state update S <- diag(A_16) S + sum_i (k_i .* exp(l_16 - l_i))^T u_i   (uses the state before the update above)
        {
            float kh[4];
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                float kv = kk[r];
#pragma unroll
                for (int gsel = 1; gsel < 4; ++gsel) kv = (tg == gsel) ? kk[4 * gsel + r] : kv;
                kh[r] = kv * __expf(lsum[kTile - 1] - lt[r]);
            }
            const uint2 b_k = {pack_bf16x2(kh[0], kh[1]), pack_bf16x2(kh[2], kh[3])};
            const int j = c >> 2, cc = c & 3;              // transposing read: this lane addresses token 4tg + j, unit cc
#pragma unroll
            for (int ct = 0; ct < kColTiles; ++ct) {
                const int pos = 32 * (ct >> 1) + 8 * cc + 4 * (ct & 1);
                const uint2 a_u = lds_read_transposed(us + (4 * tg + j) * L::kRowBytes + pos * 2);
                floatx4_t x = acc[ct];
                x[0] *= a_tile; x[1] *= a_tile; x[2] *= a_tile; x[3] *= a_tile;
                acc[ct] = mfma_k16(a_u, b_k, x);
            }
        }

        // ---- dq_t = A_t .* (do_t S^T) + sum_{i<=t} dP[t,i] k_i exp(l_t - l_i)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int t = 4 * tg + r;
            float intra = 0.f;
            if (pairwise) {
#pragma unroll
                for (int i = 0; i < kTile; ++i) {
                    const float wgt = (i <= t) ? __expf(lt[r] - lsum[i]) : 0.f;
                    intra = fmaf(dPw[wave][t][i] * kk[i], wgt, intra);
                }
            }
            const float val = fmaf(__expf(lt[r]), dqt[r], intra);
            dq_s[t * kK + ch] = (bf16_t)val;
            const float qd = qs[t * kK + ch] * val;        // zero for rows beyond the sequence (q is staged as zero)
            qdq_s[t * kK + ch] = qd;
            qpart += qd;
        }
        if (it == run_last || it == ntiles - 1) {          // the run ends: its total over the four token groups
            float x = qpart;
            x += __shfl_xor(x, 16);
            x += __shfl_xor(x, 32);
            if (tg == 0) qtot[(unit * kGateParts + run_index) * kK + ch] = x;
            qpart = 0.f;
            ++run_index;
            run_last += part_tiles;
        }
    }
    __syncthreads();
    if (ntiles > 0 && stages) store_tile((ntiles - 1) * kTile, tid);

    // rowsum(S_T .* dS_T) for this lane's channel: constant term of every gate cotangent of this (batch, head)
    if (!computes) return;
    float part = 0.f;
    if (dS_T != nullptr) {
#pragma unroll
        for (int ct = 0; ct < kColTiles; ++ct) {
            const floatx4_t gS = *reinterpret_cast<const floatx4_t *>(dS_T + state_base + 16 * ct + 4 * tg);
            part += acc[ct][0] * gS[0] + acc[ct][1] * gS[1] + acc[ct][2] * gS[2] + acc[ct][3] * gS[3];
        }
    }
    part += __shfl_xor(part, 16);
    part += __shfl_xor(part, 32);
    if (tg == 0) gate_const[unit * kK + ch] = part;
}


// =========================================================================================================
// Reverse sweep: dk, dv, dbeta, dlog_alpha, dS0
// =========================================================================================================
// One workgroup per (batch, head); wavefront w owns 32 value columns: its slab of the state cotangent G lives in MFMA
// accumulators (lane = column, registers = key channels), as the state does in the forward kernel.
// Per tile, last to first:  du^T = G^T khat^T + do^T P   (khat_i = k_i .* exp(l_16 - l_i));  partial u G^T over the slab's
// columns, summed over the wavefronts through LDS;  G <- diag(A_16) G + (q .* A)^T do.
// Only these products depend on G; the rest of a tile's work (staging, running sums, decayed operands, dP, and after
// the products dk, dv, dbeta) does not, and is laid out so that it overlaps the G-dependent work of a neighbouring tile
// inside the same wavefronts.  Between two workgroup barriers a wavefront therefore always has two independent
// instruction streams:
//   phase X: products of tile `it` (P, du, u G^T, the tile-local part of dk, G update)  |  staging of tile it-1 into
//            the other input buffer, request of tile it-2
//   phase Y: dk, dv, dbeta of tile `it`                                                   |  running sums, decayed
//            operands and this wavefront's share of dP for tile it-1
// Two barriers per tile (three on the pair-by-pair route).
template <int DV> struct DkvLds {       // byte offsets of the reverse kernel's dynamic LDS
    static constexpr int kWaves = BwdShape<DV>::kWaves;
    static constexpr int kSlabCols = 32;
    // one tile's inputs: q, k, log_alpha (clamped) as fp32 [16][64]; u and do as bf16 rows.  Two such buffers.
    static constexpr int kInKs = kTile * kK * 4;
    static constexpr int kInLs = 2 * kTile * kK * 4;
    static constexpr int kInUs = 3 * kTile * kK * 4;
    static constexpr int kInDs = kInUs + kTile * BwdLayout<DV>::kRowBytes;
    static constexpr int kInBytes = kInDs + kTile * BwdLayout<DV>::kRowBytes;
    static constexpr int kQa = 2 * kInBytes;                           // q .* A (high part), token-major, padded rows
    static constexpr int kKh = kQa + kTile * (kK + 8) * 2;             // khat
    static constexpr int kKq = kKh + kTile * (kK + 8) * 2;             // k ./ A
    static constexpr int kQaLo = kKq + kTile * (kK + 8) * 2;           // low part of q .* A (split bf16)
    static constexpr int kPt = kQaLo + kTile * (kK + 8) * 2;           // P^T [i][t] (pair-by-pair route)
    static constexpr int kDp = kPt + kTile * kTile * 2;                // dP [t][i], padded rows (pair-by-pair route)
    static constexpr int kGt = kDp + ((kTile * (kTile + 1) * 4 + 15) / 16) * 16;
    // per wavefront: its G slab as bf16 [column][channel] (padded rows), and afterwards, in the same bytes, its partial
    // u G^T as fp32 [16][64] (the slab is read before the partial exists)
    static constexpr int kGtWave = kSlabCols * (kK + 8) * 2;
    static constexpr int kRedRow = kK + 4;                             // floats per token row of a partial: the four token groups of a wavefront land in different banks
    static_assert(kGtWave >= kTile * kRedRow * 4, "the partial u G^T must fit the slab's bytes");
    static constexpr int kDu = kGt + kWaves * kGtWave;
    static constexpr int kIntra = kDu + kTile * (DV + 4) * 4;          // (dP^T (q .* A))[i][channel]
    static constexpr int kLt = kIntra + kTile * kRedRow * 4;           // running sums l_t, fp32 [16][64], two buffers
    static constexpr int kA16 = kLt + 2 * kTile * kK * 4;              // A_16 per channel, fp32 [64]
    static constexpr int kFlag = kA16 + kK * 4;                        // two flags (tile parity): != 0 = pair-by-pair route
    static constexpr int kDpPart = kFlag + 16;                         // partial dP per wavefront, fp32 [kWaves][i][t]
    static constexpr int kBytes = kDpPart + kWaves * kTile * kTile * 4;
};

struct TileBuffers {
    float *qs, *ks, *ls;
    unsigned char *us, *ds;
};

template <int DV, bool kZBeta>
__device__ __forceinline__ void sweep_dkv(
    const bf16_t *__restrict__ q, const bf16_t *__restrict__ k, const bf16_t *__restrict__ v,
    const float *__restrict__ log_alpha, const void *__restrict__ beta, const bf16_t *__restrict__ d_o,
    const float *__restrict__ dS_T, bf16_t *__restrict__ dk, bf16_t *__restrict__ dv, float *__restrict__ kdk,
    void *__restrict__ dbeta, float *__restrict__ dS0, float *__restrict__ ktot, int T, int H,
    const int *__restrict__ cu_seqlens, const BwdSegments &segs)
{
    using L = BwdLayout<DV>;
    constexpr int kWaves = BwdShape<DV>::kWaves;     // 4 (dv = 128) or 8 (dv = 256)
    constexpr int kSlab = 32;                        // columns per wavefront
    constexpr int kCt = kSlab / 16;                  // column tiles per wavefront
    constexpr int kTok = kTile / kWaves;             // tokens per thread in the vector-ALU phases: 4 or 2
    constexpr int kDuRow = DV + 4;                   // padded fp32 row of du
    using M = DkvLds<DV>;
    extern __shared__ __align__(16) unsigned char lds_raw[];
    auto tile_buffers = [&](int parity) {
        unsigned char *b = lds_raw + parity * M::kInBytes;
        return TileBuffers{reinterpret_cast<float *>(b), reinterpret_cast<float *>(b + M::kInKs),
                           reinterpret_cast<float *>(b + M::kInLs), b + M::kInUs, b + M::kInDs};
    };
    float *a16_s = reinterpret_cast<float *>(lds_raw + M::kA16);
    bf16_t *qa_s = reinterpret_cast<bf16_t *>(lds_raw + M::kQa);
    bf16_t *kh_s = reinterpret_cast<bf16_t *>(lds_raw + M::kKh);
    bf16_t *kq_s = reinterpret_cast<bf16_t *>(lds_raw + M::kKq);
    bf16_t *qa_lo_s = reinterpret_cast<bf16_t *>(lds_raw + M::kQaLo);
    bf16_t *pt_s = reinterpret_cast<bf16_t *>(lds_raw + M::kPt);             // P^T: [i][t]
    float *dp_s = reinterpret_cast<float *>(lds_raw + M::kDp);               // dP: [t][i], padded rows
    bf16_t *gt_s = reinterpret_cast<bf16_t *>(lds_raw + M::kGt + (threadIdx.x >> 6) * M::kGtWave);
    float *red_own = reinterpret_cast<float *>(lds_raw + M::kGt + (threadIdx.x >> 6) * M::kGtWave);
    float *du_s = reinterpret_cast<float *>(lds_raw + M::kDu);
    float *intra_s = reinterpret_cast<float *>(lds_raw + M::kIntra);
    int *flag_s = reinterpret_cast<int *>(lds_raw + M::kFlag);
    float *dpp_s = reinterpret_cast<float *>(lds_raw + M::kDpPart);

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int n = lane & 15, grp = lane >> 4;
    int bh = blockIdx.x;
    const int seg = blockIdx.y;
    BwdUnit u;
    if (segs.packed_cut) {
        if (!packed_cut_unit(blockIdx.x, seg, T, H, cu_seqlens, segs, u)) return;      // the whole workgroup, before any barrier
        bh = u.bh;
    } else {
        if (cu_seqlens != nullptr)                                // packed batch: sequences by descending length (small batches)
            bh = sequence_by_length_rank(cu_seqlens, (int)gridDim.x / H, T, bh / H, reinterpret_cast<int *>(lds_raw)) * H + bh % H;
        u = BwdUnit{bh, (size_t)seg * gridDim.x + bh, segment_span(seq_span(bh / H, T, cu_seqlens), segs, seg), seg == 0};
    }
    const size_t unit = u.unit;
    const bool has_beta = beta != nullptr;
    const SeqSpan span = u.span;
    T = span.length;
    const BwdGeometry g(q, k, v, d_o, log_alpha, beta, span.first, bh % H, T, H, DV);
    const size_t row0 = span.first * H + bh % H;                  // outputs: same layout as the inputs
    const int col0 = wave * kSlab;
    if (segs.nseg > 1) {
        dS_T = segs.G_slots + (unit - (size_t)bh) * kK * DV;      // state_base below adds the (batch, head)
        if (!u.first_seg) dS0 = nullptr;                          // only the first segment's cotangent leaves the call
    }

    // cotangent slab: acc[kt][ct][r] = G[16kt + 4grp + r][col0 + 16ct + n]
    floatx4_t acc[4][kCt];
    const size_t state_base = (size_t)bh * kK * DV;
#pragma unroll
    for (int kt = 0; kt < 4; ++kt)
#pragma unroll
        for (int ct = 0; ct < kCt; ++ct)
#pragma unroll
            for (int r = 0; r < 4; ++r)
                acc[kt][ct][r] = (dS_T != nullptr && wave < kWaves) ? dS_T[state_base + (size_t)(16 * kt + 4 * grp + r) * DV + col0 + 16 * ct + n] : 0.f;

    // vector-ALU role of the gate and dk phases: channel vc, tokens kTok * vg .. + kTok - 1
    const int vc = tid & 63, vg = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int j = n >> 2, cc = n & 3;                  // transposing reads: this lane addresses row 4grp + j, unit cc

    const int ntiles = (T + kTile - 1) / kTile;
    const int part_tiles = gate_part_tiles(T);
    int run_index = ntiles > 0 ? (ntiles - 1) / part_tiles : 0;      // the current run of tiles, walked from the last one back
    int run_first = run_index * part_tiles;                           // its first tile (the last one in this direction)
    float kpart = 0.f;                                 // sum of k .* dk over this thread's tokens of the current run of tiles

    // ---- running sums, decayed operands and this wavefront's share of dP for the tile staged in `in` (thread = channel
    // vc, token group vg); leaves l of the thread's own tokens and of the whole tile in registers
    auto gate_phase = [&](const TileBuffers &in, float *lt_s, int *flag, float (&l_own)[kTok], float &l_tile) {
        float lsum[kTile];
        {
            float run = 0.f;
#pragma unroll
            for (int i = 0; i < kTile; ++i) {
                run += in.ls[i * kK + vc];
                lsum[i] = run;
            }
        }
        l_tile = lsum[kTile - 1];
        if (l_tile < kSafeTileLog) *flag = 1;
        if (vg == 0) a16_s[vc] = __expf(l_tile);
#pragma unroll
        for (int r = 0; r < kTok; ++r) {
            float l = lsum[r];
#pragma unroll
            for (int gsel = 1; gsel < kWaves; ++gsel) l = (vg == gsel) ? lsum[kTok * gsel + r] : l;
            l_own[r] = l;
            const int t = kTok * vg + r;
            lt_s[t * kK + vc] = l;
            float qa_hi, qa_lo;
            split_bf16(in.qs[t * kK + vc] * __expf(l), qa_hi, qa_lo);
            qa_s[t * (kK + 8) + vc] = (bf16_t)qa_hi;
            qa_lo_s[t * (kK + 8) + vc] = (bf16_t)qa_lo;
            kh_s[t * (kK + 8) + vc] = (bf16_t)(in.ks[t * kK + vc] * __expf(l_tile - l));
            kq_s[t * (kK + 8) + vc] = (bf16_t)(in.ks[t * kK + vc] * __expf(-l));       // used only by the quotient route
        }
        // dP[t][i] = do_t . u_i over the 32 columns of this wavefront's slab; summed over the wavefronts by the readers
        const bf16x8_t a_do = *reinterpret_cast<const bf16x8_t *>(in.ds + n * L::kRowBytes + (col0 + 8 * grp) * 2);
        const bf16x8_t b_u = *reinterpret_cast<const bf16x8_t *>(in.us + n * L::kRowBytes + (col0 + 8 * grp) * 2);
        const floatx4_t d = mfma_k32(a_do, b_u, floatx4_t{0.f, 0.f, 0.f, 0.f});
        *reinterpret_cast<floatx4_t *>(&dpp_s[(wave * kTile + n) * kTile + 4 * grp]) = d;      // [wave][i = n][t = 4grp ..]
    };

    // Roles (wavefront-uniform): the first kWaves wavefronts carry G and do the products, dk and the running sums; the
    // helper wavefronts behind them load and stage the tile inputs and write dv and dbeta.
    constexpr int kHelp = 32 * kWaves;
    const bool helper = wave >= kWaves;
    const int hid = tid - 64 * kWaves;
    if (helper) {
        // The helper wavefronts' whole walk: the same barriers as the other wavefronts, in the same order.
        HelperLoads<DV> pf;
        uint4 v_cur[2], v_nxt[2];                      // this thread's v and beta pieces of the tile in phase Y and of the next
        floatx4_t beta_cur[2][2], beta_nxt[2][2];
        if (ntiles > 0) {
            const int last = ntiles - 1;
            const TileBuffers in = tile_buffers(last & 1);
            helper_prefetch<DV, kZBeta>(g, last * kTile, hid, has_beta, pf);
            helper_stage<DV, kZBeta>(pf, last * kTile, T, hid, has_beta, in.qs, in.ks, in.ls, in.us, in.ds);
#pragma unroll
            for (int s = 0; s < 2; ++s) { v_cur[s] = pf.v[s]; beta_cur[s][0] = pf.beta[s][0]; beta_cur[s][1] = pf.beta[s][1]; }
            helper_prefetch<DV, kZBeta>(g, max(last - 1, 0) * kTile, hid, has_beta, pf);
            __syncthreads();
            __syncthreads();
        }
        for (int it = ntiles - 1; it >= 0; --it) {
            const int t0 = it * kTile, par = it & 1;
            const TileBuffers nxt = tile_buffers(par ^ 1);
            // phase X: tile it-1 (at it = 0: a harmless repeat of tile 0) into the other buffer, tile it-2 requested
            const bool pairwise = flag_s[par] != 0;
            helper_stage<DV, kZBeta>(pf, t0 - kTile, T, hid, has_beta, nxt.qs, nxt.ks, nxt.ls, nxt.us, nxt.ds);
#pragma unroll
            for (int s = 0; s < 2; ++s) { v_nxt[s] = pf.v[s]; beta_nxt[s][0] = pf.beta[s][0]; beta_nxt[s][1] = pf.beta[s][1]; }
            helper_prefetch<DV, kZBeta>(g, max(t0 - 2 * kTile, 0), hid, has_beta, pf);
            if (pairwise) __syncthreads();                 // the pair-by-pair route of the other wavefronts has a barrier of its own
            __syncthreads();
            // phase Y
            // dv = beta .* du, dbeta = v .* du: coalesced, by the helper thread that loaded the same pieces of v and beta;
            // streaming stores (nothing on this GPU reads them again soon: -2 % on the layer workload)
    #pragma unroll
            for (int s = 0; s < 2; ++s) {
                const int idx = hid + s * kHelp, tok = idx / L::kPieces, piece = idx % L::kPieces;
                if (t0 + tok < T) {
                    const size_t off = (row0 + (size_t)((unsigned)(t0 + tok) * (unsigned)H)) * DV + 8 * piece;
                    const floatx4_t d0 = *reinterpret_cast<const floatx4_t *>(&du_s[tok * kDuRow + 8 * piece]);
                    const floatx4_t d1 = *reinterpret_cast<const floatx4_t *>(&du_s[tok * kDuRow + 8 * piece + 4]);
                    float x[8];
                    unpack8(v_cur[s], x);
                    const float du8[8] = {d0[0], d0[1], d0[2], d0[3], d1[0], d1[1], d1[2], d1[3]};
                    float gate[8] = {1.f, 1.f, 1.f, 1.f, 1.f, 1.f, 1.f, 1.f};
                    if (has_beta) gate_values8<kZBeta>(beta_cur[s], gate);
                    const uint4 wv = {pack_bf16x2(gate[0] * du8[0], gate[1] * du8[1]), pack_bf16x2(gate[2] * du8[2], gate[3] * du8[3]),
                                      pack_bf16x2(gate[4] * du8[4], gate[5] * du8[5]), pack_bf16x2(gate[6] * du8[6], gate[7] * du8[7])};
                    __builtin_nontemporal_store(__builtin_bit_cast(floatx4_t, wv), reinterpret_cast<floatx4_t *>(dv + off));
                    if (dbeta != nullptr) {
                        float db[8];                       // cotangent of the gate; of its pre-activation: times sigmoid' = gate (1 - gate)
#pragma unroll
                        for (int e = 0; e < 8; ++e) db[e] = x[e] * du8[e] * (kZBeta ? gate[e] * (1.f - gate[e]) : 1.f);
                        if (kZBeta) {
                            const uint4 wz = {pack_bf16x2(db[0], db[1]), pack_bf16x2(db[2], db[3]), pack_bf16x2(db[4], db[5]), pack_bf16x2(db[6], db[7])};
                            __builtin_nontemporal_store(__builtin_bit_cast(floatx4_t, wz), reinterpret_cast<floatx4_t *>(static_cast<bf16_t *>(dbeta) + off));
                        } else {
                            float *dst = static_cast<float *>(dbeta) + off;
                            __builtin_nontemporal_store(floatx4_t{db[0], db[1], db[2], db[3]}, reinterpret_cast<floatx4_t *>(dst));
                            __builtin_nontemporal_store(floatx4_t{db[4], db[5], db[6], db[7]}, reinterpret_cast<floatx4_t *>(dst + 4));
                        }
                    }
                }
                v_cur[s] = v_nxt[s]; beta_cur[s][0] = beta_nxt[s][0]; beta_cur[s][1] = beta_nxt[s][1];
            }
            __syncthreads();
        }
        return;
    }

    float l_cur[kTok], l_cur_tile = 0.f;
#pragma unroll
    for (int r = 0; r < kTok; ++r) l_cur[r] = 0.f;
    if (ntiles > 0) {
        // the last tile (staged by the helpers) is prepared before the loop
        const int last = ntiles - 1;
        const TileBuffers in = tile_buffers(last & 1);
        if (tid < 2) flag_s[tid] = 0;
        __syncthreads();
        gate_phase(in, reinterpret_cast<float *>(lds_raw + M::kLt) + (last & 1) * kTile * kK, flag_s + (last & 1), l_cur, l_cur_tile);
        __syncthreads();
    }

    for (int it = ntiles - 1; it >= 0; --it) {
        const int t0 = it * kTile, par = it & 1;
        const TileBuffers cur = tile_buffers(par), nxt = tile_buffers(par ^ 1);
        float *lt_cur = reinterpret_cast<float *>(lds_raw + M::kLt) + par * kTile * kK;
        float *lt_nxt = reinterpret_cast<float *>(lds_raw + M::kLt) + (par ^ 1) * kTile * kK;

        // =============================== phase X ===============================
        const bool pairwise = flag_s[par] != 0;
        if (tid == 0) flag_s[par ^ 1] = 0;

        // this wavefront's G slab, bf16, as [column][channel] for the transposing read of the u G^T product
#pragma unroll
        for (int kt = 0; kt < 4; ++kt)
#pragma unroll
            for (int ct = 0; ct < kCt; ++ct) {
                const floatx4_t x = acc[kt][ct];
                const uint2 w = {pack_bf16x2(x[0], x[1]), pack_bf16x2(x[2], x[3])};
                *reinterpret_cast<uint2 *>(&gt_s[(16 * ct + n) * (kK + 8) + 16 * kt + 4 * grp]) = w;
            }
        // dP[t][i] = do_t . u_i (i <= t), the sum of the wavefronts' shares: lane (i = n, group grp) holds t = 4grp + r,
        // which is the operand layout of both later uses.
        floatx4_t dp = {0.f, 0.f, 0.f, 0.f};
        if (wave < 4) {                                    // only the first four wavefronts use it (tile-local part of dk)
#pragma unroll
            for (int w = 0; w < kWaves; ++w) dp += *reinterpret_cast<const floatx4_t *>(&dpp_s[(w * kTile + n) * kTile + 4 * grp]);
#pragma unroll
            for (int r = 0; r < 4; ++r) dp[r] = (n <= 4 * grp + r) ? dp[r] : 0.f;
        }
        // P[t][i] in the same layout (B operand of do^T P)
        uint2 b_p;
        if (!pairwise) {
            floatx4_t d = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int m = 0; m < 2; ++m) {
                const bf16x8_t a_qa = *reinterpret_cast<const bf16x8_t *>(&qa_s[n * (kK + 8) + 32 * m + 8 * grp]);
                const bf16x8_t b_kq = *reinterpret_cast<const bf16x8_t *>(&kq_s[n * (kK + 8) + 32 * m + 8 * grp]);
                d = mfma_k32(a_qa, b_kq, d);
            }
            b_p = uint2{pack_bf16x2(n <= 4 * grp ? d[0] : 0.f, n <= 4 * grp + 1 ? d[1] : 0.f),
                        pack_bf16x2(n <= 4 * grp + 2 ? d[2] : 0.f, n <= 4 * grp + 3 ? d[3] : 0.f)};
        } else {
            // pair by pair on the vector ALUs (thread = (t, i), fp32), through LDS; dP for the dk phase as well
            const int t = (tid & 255) >> 4, i = tid & 15;
            float p = 0.f;
            if (tid < 256 && i <= t) {
                for (int cr = 0; cr < kK; ++cr) {
                    const int c = (cr + i) & (kK - 1);     // rotated per key row: the 16 rows of a wavefront hit 16 different banks
                    p = fmaf(cur.qs[t * kK + c] * cur.ks[i * kK + c], __expf(lt_cur[t * kK + c] - lt_cur[i * kK + c]), p);
                }
            }
            if (tid < 256) pt_s[i * kTile + t] = (bf16_t)p;
            if (wave == 0) {
#pragma unroll
                for (int r = 0; r < 4; ++r) dp_s[(4 * grp + r) * (kTile + 1) + n] = dp[r];
            }
            __syncthreads();                               // uniform: the flag is the same for the whole workgroup
            b_p = *reinterpret_cast<const uint2 *>(&pt_s[n * kTile + 4 * grp]);
        }

        // du^T[column][i] = G^T khat^T + do^T P  for this wavefront's columns; result to LDS as du[i][column]
        {
            bf16x8_t b_kh[2];
#pragma unroll
            for (int m = 0; m < 2; ++m) {
                // channels 32m + {4grp..4grp+3} (tile 2m) and 32m + 16 + {4grp..} (tile 2m+1): the slots of the packed accumulators
                const uint2 lo = *reinterpret_cast<const uint2 *>(&kh_s[n * (kK + 8) + 32 * m + 4 * grp]);
                const uint2 hi = *reinterpret_cast<const uint2 *>(&kh_s[n * (kK + 8) + 32 * m + 16 + 4 * grp]);
                const uint4 w = {lo.x, lo.y, hi.x, hi.y};
                b_kh[m] = __builtin_bit_cast(bf16x8_t, w);
            }
#pragma unroll
            for (int ct = 0; ct < kCt; ++ct) {
                floatx4_t d = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int m = 0; m < 2; ++m) {
                    const floatx4_t lo = acc[2 * m][ct], hi = acc[2 * m + 1][ct];
                    const uint4 w = {pack_bf16x2(lo[0], lo[1]), pack_bf16x2(lo[2], lo[3]), pack_bf16x2(hi[0], hi[1]), pack_bf16x2(hi[2], hi[3])};
                    d = mfma_k32(__builtin_bit_cast(bf16x8_t, w), b_kh[m], d);
                }
                // do^T tile: lane = column col0 + 16ct + n, 4 tokens 4grp ..; transposing read from the token-major rows
                const int pos = col_position(col0 + 16 * ct + 4 * cc);
                const uint2 a_do = lds_read_transposed(cur.ds + (4 * grp + j) * L::kRowBytes + pos * 2);
                d = mfma_k16(a_do, b_p, d);
                // lane (token i = n, group grp) holds columns col0 + 16ct + 4grp + r
                *reinterpret_cast<floatx4_t *>(&du_s[n * kDuRow + col0 + 16 * ct + 4 * grp]) = d;
            }
        }
        // partial (u G^T)[i][channel] over this wavefront's columns
        {
            floatx4_t d[4];
#pragma unroll
            for (int kt = 0; kt < 4; ++kt) d[kt] = floatx4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int s = 0; s < kSlab / 32; ++s) {
                // A operand: u rows, columns col0 + 32s + 8grp .. +7 in natural order = two 8-byte units at permuted positions
                const int c_lo = col0 + 32 * s + 8 * grp;
                const uint2 u_lo = *reinterpret_cast<const uint2 *>(cur.us + n * L::kRowBytes + col_position(c_lo) * 2);
                const uint2 u_hi = *reinterpret_cast<const uint2 *>(cur.us + n * L::kRowBytes + col_position(c_lo + 4) * 2);
                const uint4 wa = {u_lo.x, u_lo.y, u_hi.x, u_hi.y};
#pragma unroll
                for (int kt = 0; kt < 4; ++kt) {
                    // B operand [column][channel]: lane = channel 16kt + n, slots = columns 32s + 8grp + 0..7 (slab-relative)
                    const bf16_t *base = &gt_s[(32 * s + 8 * grp + j) * (kK + 8) + 16 * kt + 4 * cc];
                    const uint2 g_lo = lds_read_transposed(reinterpret_cast<const unsigned char *>(base));
                    const uint2 g_hi = lds_read_transposed(reinterpret_cast<const unsigned char *>(base + 4 * (kK + 8)));
                    const uint4 wb = {g_lo.x, g_lo.y, g_hi.x, g_hi.y};
                    d[kt] = mfma_k32(__builtin_bit_cast(bf16x8_t, wa), __builtin_bit_cast(bf16x8_t, wb), d[kt]);
                }
            }
            // lane (channel n of tile kt, group grp) holds tokens i = 4grp + r; the partial replaces the slab it was made from
#pragma unroll
            for (int kt = 0; kt < 4; ++kt)
#pragma unroll
                for (int r = 0; r < 4; ++r) red_own[(4 * grp + r) * M::kRedRow + 16 * kt + n] = d[kt][r];
        }
        // G <- diag(A_16) G + (q .* A)^T do;  on the quotient route also the tile-local part of dk before its 1 / A_i factor
        {
            uint2 a_q[4], b_do[kCt];
            floatx4_t dec[4];
#pragma unroll
            for (int kt = 0; kt < 4; ++kt) {
                a_q[kt] = lds_read_transposed(reinterpret_cast<const unsigned char *>(&qa_s[(4 * grp + j) * (kK + 8) + 16 * kt + 4 * cc]));
                dec[kt] = *reinterpret_cast<const floatx4_t *>(&a16_s[16 * kt + 4 * grp]);
            }
            if (!pairwise && wave < 4) {
                // (dP^T (q .* A))[i][channel], channel tile = wavefront (the first four); split-bf16 operands
                float hi[4], lo[4];
#pragma unroll
                for (int r = 0; r < 4; ++r) split_bf16(dp[r], hi[r], lo[r]);
                const uint2 a_hi = {pack_bf16x2(hi[0], hi[1]), pack_bf16x2(hi[2], hi[3])};
                const uint2 a_lo = {pack_bf16x2(lo[0], lo[1]), pack_bf16x2(lo[2], lo[3])};
                uint2 b_hi = a_q[0];
#pragma unroll
                for (int kt = 1; kt < 4; ++kt) b_hi = (wave == kt) ? a_q[kt] : b_hi;
                const uint2 b_lo = lds_read_transposed(reinterpret_cast<const unsigned char *>(&qa_lo_s[(4 * grp + j) * (kK + 8) + 16 * wave + 4 * cc]));
                floatx4_t d = mfma_k16(a_lo, b_hi, floatx4_t{0.f, 0.f, 0.f, 0.f});
                d = mfma_k16(a_hi, b_lo, d);
                d = mfma_k16(a_hi, b_hi, d);
#pragma unroll
                for (int r = 0; r < 4; ++r) intra_s[(4 * grp + r) * M::kRedRow + 16 * wave + n] = d[r];
            }
#pragma unroll
            for (int ct = 0; ct < kCt; ++ct)
                b_do[ct] = lds_read_transposed(cur.ds + (4 * grp + j) * L::kRowBytes + col_position(col0 + 16 * ct + 4 * cc) * 2);
#pragma unroll
            for (int kt = 0; kt < 4; ++kt)
#pragma unroll
                for (int ct = 0; ct < kCt; ++ct) {
                    floatx4_t x = acc[kt][ct];
                    x[0] *= dec[kt][0]; x[1] *= dec[kt][1]; x[2] *= dec[kt][2]; x[3] *= dec[kt][3];
                    acc[kt][ct] = mfma_k16(a_q[kt], b_do[ct], x);
                }
        }
        __syncthreads();

        // =============================== phase Y ===============================
        // ---- dk, and k .* dk in fp32 for the gate cotangent (thread = channel vc, tokens kTok * vg ..)
        {
#pragma unroll
            for (int r = kTok - 1; r >= 0; --r) {
                const int i = kTok * vg + r;
                const float l_i = l_cur[r];
                float khat_term = 0.f;
#pragma unroll
                for (int w = 0; w < kWaves; ++w)
                    khat_term += reinterpret_cast<const float *>(lds_raw + M::kGt + w * M::kGtWave)[i * M::kRedRow + vc];
                khat_term *= __expf(l_cur_tile - l_i);
                float intra = 0.f;
                if (pairwise) {
#pragma unroll
                    for (int t = 0; t < kTile; ++t) {
                        const float wgt = (t >= i) ? __expf(lt_cur[t * kK + vc] - l_i) : 0.f;
                        intra = fmaf(dp_s[t * (kTile + 1) + i] * cur.qs[t * kK + vc], wgt, intra);
                    }
                } else {
                    intra = intra_s[i * M::kRedRow + vc] * __expf(-l_i);
                }
                const float dk_val = khat_term + intra;
                const float kd = cur.ks[i * kK + vc] * dk_val;  // zero for rows beyond the sequence (k is staged as zero)
                kpart += kd;
                if (t0 + i < T) {                           // a wavefront writes whole rows
                    const size_t e = (row0 + (size_t)((unsigned)(t0 + i) * (unsigned)H)) * kK + vc;
                    dk[e] = (bf16_t)dk_val;
                    kdk[e] = kd;
                }
            }
            if (it == run_first) {                          // the run's first tile is its last in this direction
                ktot[((unit * kGateParts + run_index) * kWaves + vg) * kK + vc] = kpart;
                kpart = 0.f;
                --run_index;
                run_first -= part_tiles;
            }
        }
        // ---- tile it-1: running sums, decayed operands, share of dP
        gate_phase(nxt, lt_nxt, flag_s + (par ^ 1), l_cur, l_cur_tile);
        __syncthreads();
    }

    if (dS0 != nullptr) {
#pragma unroll
        for (int kt = 0; kt < 4; ++kt)
#pragma unroll
            for (int ct = 0; ct < kCt; ++ct)
#pragma unroll
                for (int r = 0; r < 4; ++r)
                    dS0[state_base + (size_t)(16 * kt + 4 * grp + r) * DV + col0 + 16 * ct + n] = acc[kt][ct][r];
    }
}

}  // namespace

// When 2 * B * H workgroups would leave much of the chip idle, a dense batch is cut into segments of whole 64-token
// chunks so that about 512 workgroups exist (the two sweeps differ in length, two rounds even them out), each segment
// keeping at least 256 tokens.  A packed batch is not cut here: its lengths live in device memory (choose_bwd_packed_cut).
struct BwdSplit { int nseg, seg_tokens; };
static BwdSplit choose_bwd_split(int B, int T, int H, bool packed)
{
    const int nchunks = (T + 63) / 64;
    const BwdSplit whole{1, nchunks * 64};
    const long long wgs = 2ll * B * H;
    if (packed || wgs == 0 || wgs >= 192 || nchunks < 8) return whole;
    long long want = (512 + wgs - 1) / wgs;
    if (want > nchunks / 4) want = nchunks / 4;
    if (want > 64) want = 64;
    if (want < 2) return whole;
    const int seg_chunks = (int)((nchunks + want - 1) / want);
    const int nseg = (nchunks + seg_chunks - 1) / seg_chunks;
    return nseg < 2 ? whole : BwdSplit{nseg, seg_chunks * 64};
}

// A packed batch cut by the kernels (the caller asks for it): a fixed segment length from the token total, such that about
// 512 workgroups exist when every sequence is cut evenly, at least 256 tokens; and the largest number of segments the batch
// can then have (every sequence adds at most one partial segment, an empty one holds one slot).
static BwdSplit choose_bwd_packed_cut(int N, int total_tokens, int H)
{
    const BwdSplit whole{1, ((total_tokens + 63) / 64) * 64};
    // every workgroup finds its slot by walking the length table: kept to batches where that walk is short
    if (N <= 0 || N > kMaxCutSequences || H <= 0 || total_tokens < 512) return whole;
    // (segments twice and half as long measured 1.32 and 1.28 ms against 1.29 ms on eight sequences of 32768 tokens in all,
    // 1.52 and 1.36 against 1.32 ms on another mix)
    long long seg = ((long long)total_tokens * H / 256 + 63) / 64 * 64;
    if (seg < 256) seg = 256;
    const long long slots = total_tokens / seg + N;
    if (slots < 2 || slots > 65535) return whole;          // the slots are a grid dimension
    return BwdSplit{(int)slots, (int)seg};
}

size_t scan_bwd_packed_cut_workspace_bytes(int N, int total_tokens, int H, int dv)
{
    const BwdSplit sp = choose_bwd_packed_cut(N, total_tokens, H);
    if (sp.nseg <= 1) return 0;
    const size_t units = (size_t)sp.nseg * H;
    const size_t floats = 2 * (size_t)total_tokens * H * kK + units * kK * (1 + kGateParts + 8 * kGateParts) + 2 * units * kK * dv +
                          2 * units * kK;
    return floats * sizeof(float);
}

// Workspace: q .* dq and k .* dk in fp32 for every (token, head, channel); per unit (segment, batch, head) and channel
// rowsum(S .* dS) at the unit's end and the totals of both products over kGateParts runs of tiles (the reverse sweep
// leaves one per wavefront, at most 8); for a call cut into segments also the two sets of state slots and the segment
// decays of both directions.
size_t scan_bwd_workspace_bytes(size_t token_rows, int B, int T, int H, int dv, bool packed)
{
    const BwdSplit sp = choose_bwd_split(B, T, H, packed);
    const size_t units = (size_t)B * H * sp.nseg;
    size_t floats = 2 * token_rows * H * kK + units * kK * (1 + kGateParts + 8 * kGateParts);
    if (sp.nseg > 1) floats += 2 * units * kK * dv + 2 * (size_t)(sp.nseg - 1) * B * H * kK;
    return floats * sizeof(float);
}

bool scan_bwd_supports(int dk, int dv, int io_dtype)
{
    return io_dtype == RODIMUS_BF16 && dk == kK && (dv == 128 || dv == 256);
}

namespace {

// Both sweeps in one launch: blockIdx.z = 0 runs the reverse sweep of (batch, head) blockIdx.x, segment blockIdx.y,
// blockIdx.z = 1 the forward sweep.  They share nothing, so with B * H workgroups each they occupy twice as many compute
// units.  The reverse sweeps take almost twice as long and come first in dispatch order, so that when there are more
// workgroups than compute units the short ones fill the gaps at the end (the other order measured 1058 us against the
// 988 us of an uncut call on the layer workload cut in two).
// kZBeta: `beta` holds the bf16 pre-activations of the value gate and `dbeta` receives the cotangent of those, in bf16.
template <int DV, bool kZBeta>
__global__ __launch_bounds__(BwdShape<DV>::kSweepThreads) void scan_bwd_sweeps_kernel(
    const bf16_t *__restrict__ q, const bf16_t *__restrict__ k, const bf16_t *__restrict__ v,
    const float *__restrict__ log_alpha, const void *__restrict__ beta, const float *__restrict__ S0,
    const bf16_t *__restrict__ d_o, const float *__restrict__ dS_T, bf16_t *__restrict__ dq, bf16_t *__restrict__ dk,
    bf16_t *__restrict__ dv, void *__restrict__ dbeta, float *__restrict__ dS0, float *__restrict__ qdq,
    float *__restrict__ kdk, float *__restrict__ gate_const, float *__restrict__ qtot, float *__restrict__ ktot, int T, int H,
    const int *__restrict__ cu_seqlens, BwdSegments segs)
{
    if (blockIdx.z == 1)
        sweep_dq<DV, kZBeta>(q, k, v, log_alpha, beta, S0, d_o, dS_T, dq, qdq, gate_const, qtot, T, H, cu_seqlens, segs);
    else
        sweep_dkv<DV, kZBeta>(q, k, v, log_alpha, beta, d_o, dS_T, dk, dv, kdk, dbeta, dS0, ktot, T, H, cu_seqlens, segs);
}

// The G recurrence alone over one segment (blockIdx.y + 1; the first segment's result would be dS0 and is left to the
// sweep), from a zero cotangent: G <- diag(A_16) G + (q .* A)^T do over the segment's tiles, last to first, one wavefront
// per 32 value columns as in the reverse sweep.  Leaves the result in slot seg-1 (the segment that receives it) and the
// segment's total decay in decay[seg-1].
template <int DV>
__global__ __launch_bounds__(BwdShape<DV>::kThreads) void scan_bwd_cotangent_summary_kernel(
    const bf16_t *__restrict__ q, const float *__restrict__ log_alpha, const bf16_t *__restrict__ d_o,
    float *__restrict__ G_slots, float *__restrict__ decay, int T, int H, int seg_tokens, const int *__restrict__ cu_seqlens, int nseq)
{
    using L = BwdLayout<DV>;
    constexpr int kWaves = BwdShape<DV>::kWaves, kSlab = 32, kCt = kSlab / 16, kTok = kTile / kWaves;
    constexpr bool kWide = BwdShape<DV>::kThreads == 512;
    __shared__ __align__(16) float qs[kTile * kK], ls[kTile * kK], a16_s[kK];
    __shared__ __align__(16) unsigned char ds[kTile * L::kRowBytes];
    __shared__ __align__(16) bf16_t qa_s[kTile * (kK + 8)];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int n = lane & 15, grp = lane >> 4;
    int bh = blockIdx.x, seg = blockIdx.y + 1;
    int t_begin = seg * seg_tokens;
    int len = min(seg_tokens, T - t_begin);                       // > 0: the host cuts T into ceil(T / seg_tokens) segments
    size_t row0 = ((size_t)(bh / H) * T + t_begin) * H + bh % H;
    size_t unit = (size_t)(seg - 1) * gridDim.x + bh;             // the slot that receives the result: the segment before
    if (cu_seqlens != nullptr) {
        // packed batch cut by the kernels: grid (head, slot); a sequence's first segment has no segment before it
        PackedSlot ps;
        if (!locate_packed_slot(cu_seqlens, nseq, T, seg_tokens, blockIdx.y, ps) || ps.j == 0) return;
        t_begin = ps.j * seg_tokens;
        len = min(seg_tokens, ps.len - t_begin);
        row0 = ((size_t)ps.first + t_begin) * H + blockIdx.x;
        unit = (size_t)(blockIdx.y - 1) * H + blockIdx.x;
    }
    q += row0 * kK; log_alpha += row0 * kK; d_o += row0 * DV;
    const int col0 = wave * kSlab;
    const int vc = tid & 63, vg = __builtin_amdgcn_readfirstlane(tid >> 6);

    floatx4_t acc[4][kCt];
#pragma unroll
    for (int kt = 0; kt < 4; ++kt)
#pragma unroll
        for (int ct = 0; ct < kCt; ++ct) acc[kt][ct] = floatx4_t{0.f, 0.f, 0.f, 0.f};
    float log_decay = 0.f;

    uint4 pq = {0u, 0u, 0u, 0u}, pdo;
    floatx4_t pla = {0.f, 0.f, 0.f, 0.f};
    auto prefetch = [&](int t0) {
        if (tid < 128) pq = *reinterpret_cast<const uint4 *>(q + (size_t)((unsigned)min(t0 + (tid >> 3), len - 1) * (unsigned)H) * kK + 8 * (tid & 7));
        if (!kWide || tid >= 256)
            pla = *reinterpret_cast<const floatx4_t *>(log_alpha + (size_t)((unsigned)min(t0 + ((tid & 255) >> 4), len - 1) * (unsigned)H) * kK + 4 * (tid & 15));
        pdo = *reinterpret_cast<const uint4 *>(d_o + (size_t)((unsigned)min(t0 + tid / L::kPieces, len - 1) * (unsigned)H) * DV + 8 * (tid % L::kPieces));
    };
    const int ntiles = (len + kTile - 1) / kTile;
    prefetch((ntiles - 1) * kTile);
    for (int it = ntiles - 1; it >= 0; --it) {
        const int t0 = it * kTile;
        __syncthreads();                                   // the previous tile is consumed
        if (tid < 128) {
            const int tok = tid >> 3;
            float x[8];
            unpack8(pq, x);
#pragma unroll
            for (int e = 0; e < 8; ++e) qs[tok * kK + 8 * (tid & 7) + e] = (t0 + tok < len) ? x[e] : 0.f;
        }
        if (!kWide || tid >= 256) {
            const int tok = (tid & 255) >> 4;
#pragma unroll
            for (int e = 0; e < 4; ++e) ls[tok * kK + 4 * (tid & 15) + e] = (t0 + tok < len) ? fmaxf(pla[e], kMinLogAlpha) : 0.f;
        }
        {
            const int tok = tid / L::kPieces, piece = tid % L::kPieces;
            float d[8];
            unpack8(pdo, d);
#pragma unroll
            for (int e = 0; e < 8; ++e) d[e] = (t0 + tok < len) ? d[e] : 0.f;
#pragma unroll
            for (int half = 0; half < 2; ++half) {
                const uint2 wd = {pack_bf16x2(d[4 * half], d[4 * half + 1]), pack_bf16x2(d[4 * half + 2], d[4 * half + 3])};
                *reinterpret_cast<uint2 *>(ds + tok * L::kRowBytes + col_position(8 * piece + 4 * half) * 2) = wd;
            }
        }
        prefetch(max(t0 - kTile, 0));
        __syncthreads();
        // thread = (channel vc, tokens kTok * vg ..): running sums of log_alpha, q .* A
        {
            float lsum[kTile], run = 0.f;
#pragma unroll
            for (int i = 0; i < kTile; ++i) {
                run += ls[i * kK + vc];
                lsum[i] = run;
            }
            if (vg == 0) {
                a16_s[vc] = __expf(run);
                log_decay += run;
            }
#pragma unroll
            for (int r = 0; r < kTok; ++r) {
                float l_own = lsum[r];
#pragma unroll
                for (int gsel = 1; gsel < kWaves; ++gsel) l_own = (vg == gsel) ? lsum[kTok * gsel + r] : l_own;
                const int t = kTok * vg + r;
                qa_s[t * (kK + 8) + vc] = (bf16_t)(qs[t * kK + vc] * __expf(l_own));
            }
        }
        __syncthreads();
        {
            const int j = n >> 2, cc = n & 3;              // transposing reads: this lane addresses row 4grp + j, unit cc
            uint2 a_q[4], b_do[kCt];
            floatx4_t dec[4];
#pragma unroll
            for (int kt = 0; kt < 4; ++kt) {
                a_q[kt] = lds_read_transposed(reinterpret_cast<const unsigned char *>(&qa_s[(4 * grp + j) * (kK + 8) + 16 * kt + 4 * cc]));
                dec[kt] = *reinterpret_cast<const floatx4_t *>(&a16_s[16 * kt + 4 * grp]);
            }
#pragma unroll
            for (int ct = 0; ct < kCt; ++ct)
                b_do[ct] = lds_read_transposed(ds + (4 * grp + j) * L::kRowBytes + col_position(col0 + 16 * ct + 4 * cc) * 2);
#pragma unroll
            for (int kt = 0; kt < 4; ++kt)
#pragma unroll
                for (int ct = 0; ct < kCt; ++ct) {
                    floatx4_t x = acc[kt][ct];
                    x[0] *= dec[kt][0]; x[1] *= dec[kt][1]; x[2] *= dec[kt][2]; x[3] *= dec[kt][3];
                    acc[kt][ct] = mfma_k16(a_q[kt], b_do[ct], x);
                }
        }
    }
    float *out = G_slots + unit * kK * DV;
#pragma unroll
    for (int kt = 0; kt < 4; ++kt)
#pragma unroll
        for (int ct = 0; ct < kCt; ++ct)
#pragma unroll
            for (int r = 0; r < 4; ++r) out[(size_t)(16 * kt + 4 * grp + r) * DV + col0 + 16 * ct + n] = acc[kt][ct][r];
    if (vg == 0) decay[unit * kK + vc] = __expf(log_decay);
}

// Cotangent of the state leaving every segment, from the summary pass: the last slot = dS_T (or zero), and for
// s < nseg-1  slot s <- decay[s] .* slot[s+1] + slot[s]  (decay[s] is the total decay of segment s+1, slot[s] held the
// summary of segment s+1).  One thread per four adjacent state elements; the segments are walked from the last one back.
__global__ __launch_bounds__(256) void scan_bwd_cotangent_chain_kernel(const float *__restrict__ dS_T, float *__restrict__ G_slots,
                                                                      const float *__restrict__ decay, int nseg, int dv,
                                                                      size_t quads_per_slot, const int *__restrict__ cu_seqlens,
                                                                      int nseq, int total_tokens, int seg_tokens)
{
    const size_t e4 = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const size_t slot_elems = quads_per_slot * 4;
    size_t elem = e4 * 4;
    if (cu_seqlens != nullptr) {
        // packed batch cut by the kernels: a slot holds the H heads of one sequence, e4 runs over [sequence][slot element],
        // and the chain walks the slots of that sequence
        const int b = (int)(e4 / quads_per_slot);
        if (b >= nseq) return;
        elem = (e4 % quads_per_slot) * 4;
        int first_slot, count;
        packed_sequence_slots(cu_seqlens, b, total_tokens, seg_tokens, first_slot, count);
        if (first_slot >= nseg) return;                    // only with a corrupt table: stay inside the slots
        count = min(count, nseg - first_slot);
        dS_T = dS_T != nullptr ? dS_T + (size_t)b * slot_elems : nullptr;
        G_slots += (size_t)first_slot * slot_elems;
        decay += (size_t)first_slot * (slot_elems / dv);
        nseg = count;
    } else if (e4 >= quads_per_slot) {
        return;
    }
    const size_t row = elem / dv;                          // (batch, head) * 64 + channel
    floatx4_t g = dS_T != nullptr ? *reinterpret_cast<const floatx4_t *>(dS_T + elem) : floatx4_t{0.f, 0.f, 0.f, 0.f};
    *reinterpret_cast<floatx4_t *>(G_slots + (size_t)(nseg - 1) * slot_elems + elem) = g;
    for (int sg = nseg - 2; sg >= 0; --sg) {
        const float a = decay[(size_t)sg * (slot_elems / dv) + row];
        floatx4_t *p = reinterpret_cast<floatx4_t *>(G_slots + (size_t)sg * slot_elems + elem);
        const floatx4_t loc = *p;
        g[0] = fmaf(a, g[0], loc[0]); g[1] = fmaf(a, g[1], loc[1]);
        g[2] = fmaf(a, g[2], loc[2]); g[3] = fmaf(a, g[3], loc[3]);
        *p = g;
    }
}

// dlog_alpha_t = gate_const + sum_{s >= t} (q_s .* dq_s - k_s .* dk_s), zero for a closed gate.  One workgroup per
// (batch, head, half of the channels, segment); thread = (channel, one of the kGateParts runs of tiles): the runs' totals come from
// the sweeps (the reverse sweep leaves one per wavefront), then one pass over the run on top of the totals of the later
// runs.
__global__ __launch_bounds__(1024) void scan_bwd_gate_kernel(const float *__restrict__ qdq, const float *__restrict__ kdk,
                                                             const float *__restrict__ gate_const,
                                                             const float *__restrict__ qtot, const float *__restrict__ ktot,
                                                             int ktot_waves, const float *__restrict__ log_alpha,
                                                             float *__restrict__ dla, int T, int H,
                                                             const int *__restrict__ cu_seqlens, BwdSegments segs)
{
    __shared__ float tot_s[kGateParts][32];
    const int tid = threadIdx.x, c = tid & 31, part = tid >> 5;
    const int bh = blockIdx.x, ch = 32 * blockIdx.y + c;
    BwdUnit u{bh, (size_t)blockIdx.z * gridDim.x + bh, SeqSpan{0, 0}, blockIdx.z == 0};
    if (segs.packed_cut) {
        if (!packed_cut_unit(blockIdx.x, blockIdx.z, T, H, cu_seqlens, segs, u)) return;      // the whole workgroup, before the barrier
    } else {
        u.span = segment_span(seq_span(bh / H, T, cu_seqlens), segs, blockIdx.z);
    }
    const size_t unit = u.unit;
    const SeqSpan span = u.span;
    T = span.length;
    const size_t tok0 = span.first;
    const int h = u.bh % H;
    const int ntiles = (T + kTile - 1) / kTile, part_tiles = gate_part_tiles(T);
    const int t_lo = min(part * part_tiles * kTile, T), t_hi = min(t_lo + part_tiles * kTile, T);
    float total = 0.f;
    if (part * part_tiles < ntiles) {                  // runs beyond the sequence were never written
        const size_t slot = unit * kGateParts + part;
        total = qtot[slot * kK + ch];
        for (int w = 0; w < ktot_waves; ++w) total -= ktot[(slot * ktot_waves + w) * kK + ch];
    }
    tot_s[part][c] = total;
    __syncthreads();
    float run = gate_const[unit * kK + ch];
    for (int p = kGateParts - 1; p > part; --p) run += tot_s[p][c];
#pragma unroll 8
    for (int t = t_hi - 1; t >= t_lo; --t) {
        const size_t e = ((tok0 + t) * H + h) * kK + ch;
        run += __builtin_nontemporal_load(qdq + e) - __builtin_nontemporal_load(kdk + e);      // read once, never again
        dla[e] = __builtin_nontemporal_load(log_alpha + e) <= kMinLogAlpha ? 0.f : run;
    }
}

template <int DV, bool kZBeta>
hipError_t launch_scan_bwd_typed(const ScanBwdArgs &a)
{
    const unsigned bh = (unsigned)(a.B * a.H);
    const bool packed = a.cu_seqlens != nullptr;
    const bool packed_cut = packed && a.packed_cut && choose_bwd_packed_cut(a.B, a.T, a.H).nseg > 1;
    const BwdSplit sp = packed_cut ? choose_bwd_packed_cut(a.B, a.T, a.H) : choose_bwd_split(a.B, a.T, a.H, packed);
    // a packed batch cut by the kernels: the grids run over (head, slot), the per-unit arrays and the slots over slot x head
    const size_t units = packed_cut ? (size_t)sp.nseg * a.H : (size_t)bh * sp.nseg;
    const unsigned grid_x = packed_cut ? (unsigned)a.H : bh;
    const size_t rows = a.token_rows() * a.H * kK;
    float *qdq = static_cast<float *>(a.workspace);
    float *kdk = qdq + rows;
    float *gate_const = kdk + rows;
    float *qtot = gate_const + units * kK;                              // [units][kGateParts][64]
    float *ktot = qtot + units * kGateParts * kK;                       // [units][kGateParts][wavefronts][64]
    BwdSegments segs{sp.nseg, sp.seg_tokens, nullptr, nullptr, packed_cut, a.B};
    if (sp.nseg > 1) {
        const size_t slot_elems = (size_t)grid_x * kK * DV;
        float *S_slots = ktot + units * kGateParts * 8 * kK;
        float *G_slots = S_slots + sp.nseg * slot_elems;
        float *s_decay = G_slots + sp.nseg * slot_elems;                // [nseg-1][B*H][64] ([nseg][H][64] packed), forward direction
        float *g_decay = s_decay + (size_t)(packed_cut ? sp.nseg : sp.nseg - 1) * grid_x * kK;     // the same for the cotangent chain
        hipError_t e = launch_scan_segment_states(a.k, a.v, a.log_alpha, a.beta, kZBeta, a.S0, a.B, a.T, a.H, DV, sp.nseg,
                                                  sp.seg_tokens, S_slots, s_decay, a.stream, packed_cut ? a.cu_seqlens : nullptr);
        if (e != hipSuccess) return e;
        hipLaunchKernelGGL(scan_bwd_cotangent_summary_kernel<DV>, dim3(grid_x, (unsigned)(packed_cut ? sp.nseg : sp.nseg - 1)),
                           dim3(BwdShape<DV>::kThreads), 0,
                           a.stream, (const bf16_t *)a.q, a.log_alpha, (const bf16_t *)a.d_o, G_slots, g_decay, a.T, a.H,
                           sp.seg_tokens, packed_cut ? a.cu_seqlens : (const int *)nullptr, a.B);
        const size_t quads = slot_elems / 4;
        const size_t threads = packed_cut ? quads * a.B : quads;
        hipLaunchKernelGGL(scan_bwd_cotangent_chain_kernel, dim3((unsigned)((threads + 255) / 256)), dim3(256), 0, a.stream, a.dS_T,
                           G_slots, g_decay, sp.nseg, DV, quads, packed_cut ? a.cu_seqlens : (const int *)nullptr, a.B, a.T,
                           sp.seg_tokens);
        segs.S_slots = S_slots;
        segs.G_slots = G_slots;
    }
    // more than the default 64 KB of dynamic LDS: the limit is raised once per kernel instance and device
    static std::atomic<bool> lds_allowed[64];
    int device = 0;
    hipError_t attr = hipGetDevice(&device);
    if (attr != hipSuccess) return attr;
    if (device < 0 || device >= 64) return hipErrorInvalidDevice;
    if (!lds_allowed[device].load(std::memory_order_acquire)) {
        attr = hipFuncSetAttribute(reinterpret_cast<const void *>(&scan_bwd_sweeps_kernel<DV, kZBeta>),
                                   hipFuncAttributeMaxDynamicSharedMemorySize, DkvLds<DV>::kBytes);
        if (attr != hipSuccess) return attr;
        lds_allowed[device].store(true, std::memory_order_release);
    }
    hipLaunchKernelGGL((scan_bwd_sweeps_kernel<DV, kZBeta>), dim3(grid_x, (unsigned)sp.nseg, 2), dim3(BwdShape<DV>::kSweepThreads), DkvLds<DV>::kBytes,
                       a.stream, (const bf16_t *)a.q, (const bf16_t *)a.k, (const bf16_t *)a.v, a.log_alpha, a.beta, a.S0,
                       (const bf16_t *)a.d_o, a.dS_T, (bf16_t *)a.dq, (bf16_t *)a.dk, (bf16_t *)a.dv, a.dbeta, a.dS0, qdq, kdk,
                       gate_const, qtot, ktot, a.T, a.H, a.cu_seqlens, segs);
    if (a.T > 0)
        hipLaunchKernelGGL(scan_bwd_gate_kernel, dim3(grid_x, 2, (unsigned)sp.nseg), dim3(1024), 0, a.stream, qdq, kdk, gate_const, qtot,
                           ktot, BwdShape<DV>::kWaves, a.log_alpha, a.dlog_alpha, a.T, a.H, a.cu_seqlens, segs);
    return hipGetLastError();
}

}  // namespace

// T == 0: nothing flows through any token; dS0 = dS_T (or zero) is produced by the reverse kernel all the same.
hipError_t launch_scan_bwd(const ScanBwdArgs &a)
{
    if ((long long)a.B * a.H == 0) return hipSuccess;
    if (a.beta_preact) return a.dv_width == 256 ? launch_scan_bwd_typed<256, true>(a) : launch_scan_bwd_typed<128, true>(a);
    return a.dv_width == 256 ? launch_scan_bwd_typed<256, false>(a) : launch_scan_bwd_typed<128, false>(a);
}

}  // namespace rodimus
