// Chunkwise forward scan of the Rodimus recurrence on the matrix cores (bf16 MFMA, fp32 accumulate).
// Shape: dk = 64, chunk = 64, value columns in tiles of 128.  gfx950 only.
//
// Per (batch, head), with A_t the product of the decay gates from the chunk start through row t and G_i
// the product over the rows after i to the chunk end (paper appendix "Chunkwise Parallel Representation
// of the Rodimus Block"):
//     o_t   = (q_t .* A_t) S_prev + sum_{i<=t} P[t,i] (beta_i .* v_i)
//     P[t,i]= sum_n q_t[n] k_i[n] prod_{j=i+1..t} alpha_j[n]
//     S_new = diag(A_C) S_prev + sum_i (k_i .* G_i)^T (beta_i .* v_i)
// The appendix's quotient A_t / A_i is never formed: the pairwise decay is built from products of gates
// by binary splitting of the chunk (see the comment on build_versions), so alpha = 0 and decays beyond
// the fp32 range are exact.
//
// One workgroup of 8 wavefronts owns one (batch, head), one tile of 128 value columns and walks the
// chunks of its token range in order.  The fp32 state tile (64 x 128) lives in MFMA accumulators for the
// whole walk: wavefront (rh, cs) holds rows 32rh..32rh+31, columns 32cs..32cs+31.  Per chunk:
//   A  the prefetched q, k, log_alpha tiles go to LDS; beta .* v goes to LDS transposed (token-contiguous)
//   B  every thread owns 4 consecutive rows x 2 key channels: gate products inside the thread, a 16-lane
//      segmented scan across threads, then the decayed copies of q and k ("versions") are written as bf16
//   C  o += (q .* A) S_prev on MFMA; the score tiles on MFMA (Gram matrices of the version arrays, masked)
//   D  o += P (beta .* v), store o;  S = diag(A_C) S + (k .* G)^T (beta .* v);  bf16 copy of S for step C
// The next chunk's global loads are issued in step A and land in registers while B-D run.
//
// LDS arrays holding bf16 rows of 128 bytes are stored unpadded with the 16-byte unit index XOR-swizzled by
// the row, which keeps both the MFMA operand reads (16 B per lane, consecutive rows) and the scan threads'
// 4-byte accesses (rows 4 apart) spread over all banks.
#include "internal.h"

namespace rodimus {

namespace {

constexpr int kC = 64;          // chunk length
constexpr int kK = 64;          // key width
constexpr int kColTile = 128;   // value columns per workgroup
constexpr int kThreads = 512;

// ---- LDS map (bytes) ------------------------------------------------------------------------------------
constexpr int kRowBytes = 128;                        // 64 bf16
constexpr int kTile64 = 64 * kRowBytes;               // a [64][64] bf16 array
constexpr int kOffX = 0;                              // 6 version arrays, one per split level h = 1..32
constexpr int kOffQraw = kOffX + 6 * kTile64;
constexpr int kOffKraw = kOffQraw + kTile64;
constexpr int kOffQin = kOffKraw + kTile64;           // q .* A          [t][n]
constexpr int kOffKstT = kOffQin + kTile64;           // (k .* G)^T      [n][token]
constexpr int kOffGVt = kOffKstT + kTile64;           // (beta .* v)^T   [column][token], 128 rows
constexpr int kOffSt = kOffGVt + 2 * kTile64;         // bf16 state^T    [column][n],     128 rows
constexpr int kOffPm = kOffSt + 2 * kTile64;          // scores [t][i]; the same bytes stage log_alpha (fp32) in step A
constexpr int kOffGam = kOffPm + 2 * kTile64;         // A_C, 64 floats
constexpr int kLdsBytes = kOffGam + 64 * 4;

__device__ __forceinline__ int swz(int row) { return (row ^ (row >> 3)) & 7; }
// byte offset of 16-byte unit `unit` (0..7) of row `row` in a bf16 array with 128-byte rows
__device__ __forceinline__ int boff(int row, int unit) { return row * kRowBytes + ((unit ^ swz(row)) << 4); }
// same for the fp32 log_alpha staging tile (256-byte rows, 16 units)
__device__ __forceinline__ int loff(int row, int unit) { return row * 256 + ((unit ^ ((row >> 2) & 15)) << 4); }

__device__ __forceinline__ bf16x8_t lds_operand(const unsigned char *base, int row, int unit)
{
    return *reinterpret_cast<const bf16x8_t *>(base + boff(row, unit));
}

__device__ __forceinline__ floatx16_t mfma32(bf16x8_t a, bf16x8_t b, floatx16_t c)
{
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}
__device__ __forceinline__ floatx4_t mfma16(bf16x8_t a, bf16x8_t b, floatx4_t c)
{
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0);
}

struct Prefetch {          // one chunk's global data for this thread, in flight while the previous chunk computes
    uint4 q, k;            // 8 bf16 of one row
    floatx4_t la[2];       // 4 log_alpha of two rows
    uint4 v[2];            // 8 bf16 of two rows
    floatx4_t beta[2][2];  // the matching 8 gate values
};

struct Geometry {
    const bf16_t *q, *k, *v;
    const float *la, *beta;
    int T, H, dv;
    int b, h, j0;          // batch, head, first value column of this workgroup
};

// Issue the global loads of the chunk starting at token s.  Rows at or beyond T read as q = k = v = 0,
// log_alpha = 0 (alpha = 1): a padded row changes neither the state nor any stored output.
__device__ __forceinline__ void prefetch_chunk(const Geometry &g, int s, int tid, Prefetch &p)
{
    const uint4 zero4 = {0u, 0u, 0u, 0u};
    const floatx4_t zerof = {0.f, 0.f, 0.f, 0.f};
    {
        const int row = tid >> 3, unit = tid & 7;
        const bool ok = s + row < g.T;
        const size_t off = (((size_t)g.b * g.T + s + row) * g.H + g.h) * kK + unit * 8;
        p.q = ok ? *reinterpret_cast<const uint4 *>(g.q + off) : zero4;
        p.k = ok ? *reinterpret_cast<const uint4 *>(g.k + off) : zero4;
    }
#pragma unroll
    for (int u = 0; u < 2; ++u) {
        const int row = (tid >> 4) + 32 * u, unit = tid & 15;
        const bool ok = s + row < g.T;
        const size_t tok = ((size_t)g.b * g.T + s + row) * g.H + g.h;
        p.la[u] = ok ? *reinterpret_cast<const floatx4_t *>(g.la + tok * kK + unit * 4) : zerof;
        const size_t voff = tok * g.dv + g.j0 + unit * 8;
        p.v[u] = ok ? *reinterpret_cast<const uint4 *>(g.v + voff) : zero4;
        if (g.beta != nullptr) {
            p.beta[u][0] = ok ? *reinterpret_cast<const floatx4_t *>(g.beta + voff) : zerof;
            p.beta[u][1] = ok ? *reinterpret_cast<const floatx4_t *>(g.beta + voff + 4) : zerof;
        }
    }
}

// Step A: registers -> LDS.  beta .* v is rounded to bf16 and stored transposed (one column per LDS row).
__device__ __forceinline__ void stage_chunk(unsigned char *lds, int tid, const Prefetch &p, bool has_beta)
{
    {
        const int row = tid >> 3, unit = tid & 7;
        *reinterpret_cast<uint4 *>(lds + kOffQraw + boff(row, unit)) = p.q;
        *reinterpret_cast<uint4 *>(lds + kOffKraw + boff(row, unit)) = p.k;
    }
#pragma unroll
    for (int u = 0; u < 2; ++u) {
        const int row = (tid >> 4) + 32 * u, unit = tid & 15;
        *reinterpret_cast<floatx4_t *>(lds + kOffPm + loff(row, unit)) = p.la[u];
        const uint32_t w[4] = {p.v[u].x, p.v[u].y, p.v[u].z, p.v[u].w};
        float gv[8];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            gv[2 * j] = bf16_lo(w[j]);
            gv[2 * j + 1] = bf16_hi(w[j]);
        }
        if (has_beta) {
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                gv[j] *= p.beta[u][0][j];
                gv[4 + j] *= p.beta[u][1][j];
            }
        }
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const int col = unit * 8 + j;
            *reinterpret_cast<bf16_t *>(lds + kOffGVt + boff(col, row >> 3) + 2 * (row & 7)) = (bf16_t)gv[j];
        }
    }
}

// Step B.  Binary splitting of the pairwise decay: for a power of two h, a row t with bit h set pairs with the
// rows i of the first half of its aligned 2h-block, and
//     prod_{j=i+1..t} alpha_j = (prod of alpha over t's h-block from its start through t)
//                             * (prod of alpha over the rows after i to the end of i's h-block).
// Version array X_h holds q .* (that prefix product) in rows with bit h set and k .* (that suffix product) in
// the others, so the level-h scores are entries of the Gram matrix X_h X_h^T.  This thread owns rows
// 4rg..4rg+3 and channels n0, n0+1: levels 1 and 2 stay inside the thread; for h >= 4 the in-thread products
// are extended by E (product of the whole threads before it in its aligned group) and F (threads after it),
// obtained by a segmented scan over the 16 lanes that share the channels.  After the last level the prefix is
// A_t and the suffix is G_i.
__device__ __forceinline__ void build_versions(unsigned char *lds, int lane, int wave)
{
    const int rg = lane & 15, cpl = lane >> 4;
    const int n0 = 2 * (4 * wave + cpl);              // first of this thread's two key channels
    const int unit = n0 >> 3, inunit = (n0 & 7) * 2;  // 16-byte unit and byte offset inside it
    const int lane_base = lane & ~15;

    float a[4][2], q[4][2], k[4][2];
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        const int row = 4 * rg + r;
        const floatx2_t la = *reinterpret_cast<const floatx2_t *>(lds + kOffPm + loff(row, n0 >> 2) + (n0 & 3) * 4);
        a[r][0] = __expf(la[0]);
        a[r][1] = __expf(la[1]);
        const uint32_t qw = *reinterpret_cast<const uint32_t *>(lds + kOffQraw + boff(row, unit) + inunit);
        const uint32_t kw = *reinterpret_cast<const uint32_t *>(lds + kOffKraw + boff(row, unit) + inunit);
        q[r][0] = bf16_lo(qw); q[r][1] = bf16_hi(qw);
        k[r][0] = bf16_lo(kw); k[r][1] = bf16_hi(kw);
    }

    float qp[4][2], ks[4][2];     // q .* (prefix inside the thread's 4 rows), k .* (suffix inside them)
    float p2[4][2], s2[4][2];
    float E[5][2], F[5][2];
#pragma unroll
    for (int c = 0; c < 2; ++c) {
        const float a01 = a[0][c] * a[1][c], a23 = a[2][c] * a[3][c];
        p2[0][c] = a[0][c]; p2[1][c] = a01; p2[2][c] = a[2][c]; p2[3][c] = a23;
        s2[0][c] = a[1][c]; s2[1][c] = 1.f; s2[2][c] = a[3][c]; s2[3][c] = 1.f;
        const float p4[4] = {a[0][c], a01, a[2][c] * a01, a23 * a01};
        const float s4[4] = {a[1][c] * a23, a23, a[3][c], 1.f};
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            qp[r][c] = q[r][c] * p4[r];
            ks[r][c] = k[r][c] * s4[r];
        }
        const float total = p4[3];            // product over this thread's 4 rows
        E[0][c] = 1.f; F[0][c] = 1.f;
        float incl_pre = total, incl_suf = total;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int m = 1 << j;
            const int last_first = (rg & ~(2 * m - 1)) + m - 1;      // last thread of the first half of the group
            const float first_half = __shfl(incl_pre, lane_base + last_first);
            const float second_half = __shfl(incl_suf, lane_base + last_first + 1);
            const bool upper = (rg & m) != 0;
            E[j + 1][c] = upper ? E[j][c] * first_half : E[j][c];
            F[j + 1][c] = upper ? F[j][c] : F[j][c] * second_half;
            incl_pre = E[j + 1][c] * total;
            incl_suf = F[j + 1][c] * total;
        }
    }

    unsigned char *X = lds + kOffX;
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        const int row = 4 * rg + r;
        const int off = boff(row, unit) + inunit;
        float x0, x1;
        // h = 1 and h = 2: the split bit is a bit of r
        x0 = (r & 1) ? q[r][0] * a[r][0] : k[r][0];
        x1 = (r & 1) ? q[r][1] * a[r][1] : k[r][1];
        *reinterpret_cast<uint32_t *>(X + 0 * kTile64 + off) = pack_bf16x2(x0, x1);
        x0 = (r & 2) ? q[r][0] * p2[r][0] : k[r][0] * s2[r][0];
        x1 = (r & 2) ? q[r][1] * p2[r][1] : k[r][1] * s2[r][1];
        *reinterpret_cast<uint32_t *>(X + 1 * kTile64 + off) = pack_bf16x2(x0, x1);
        // h = 4, 8, 16, 32: the split bit is bit j of rg
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const bool upper = (rg & (1 << j)) != 0;
            x0 = upper ? qp[r][0] * E[j][0] : ks[r][0] * F[j][0];
            x1 = upper ? qp[r][1] * E[j][1] : ks[r][1] * F[j][1];
            *reinterpret_cast<uint32_t *>(X + (2 + j) * kTile64 + off) = pack_bf16x2(x0, x1);
        }
        *reinterpret_cast<uint32_t *>(lds + kOffQin + off) = pack_bf16x2(qp[r][0] * E[4][0], qp[r][1] * E[4][1]);
    }
    // (k .* G)^T: four consecutive tokens of one channel are 8 contiguous bytes
#pragma unroll
    for (int c = 0; c < 2; ++c) {
        uint2 w;
        w.x = pack_bf16x2(ks[0][c] * F[4][c], ks[1][c] * F[4][c]);
        w.y = pack_bf16x2(ks[2][c] * F[4][c], ks[3][c] * F[4][c]);
        *reinterpret_cast<uint2 *>(lds + kOffKstT + boff(n0 + c, rg >> 1) + 8 * (rg & 1)) = w;
    }
    if (rg == 15) {               // decay of the whole chunk, A_C
        float *gam = reinterpret_cast<float *>(lds + kOffGam);
        gam[n0] = a[0][0] * a[1][0] * a[2][0] * a[3][0] * E[4][0];
        gam[n0 + 1] = a[0][1] * a[1][1] * a[2][1] * a[3][1] * E[4][1];
    }
}

__device__ __forceinline__ void store_score_quad(unsigned char *lds, int t, int i0, float x0, float x1, float x2, float x3)
{
    uint2 w = {pack_bf16x2(x0, x1), pack_bf16x2(x2, x3)};
    *reinterpret_cast<uint2 *>(lds + kOffPm + boff(t, i0 >> 3) + (i0 & 7) * 2) = w;
}

// Step C, score tiles.  D[m][n] = sum_n' Arow_m . Brow_n with m the key row i and n the query row t, so a lane
// ends up with four consecutive i for one t: 8 contiguous bytes of the row-major score matrix.
__device__ __forceinline__ void score_tiles(unsigned char *lds, int lane, int wave)
{
    const unsigned char *X = lds + kOffX;
    if (wave == 0) {
        // h = 32: queries 32..63 against keys 0..31, one 32x32 tile
        floatx16_t d = {0.f};
        const int n = lane & 31, half = lane >> 5;
#pragma unroll
        for (int step = 0; step < 4; ++step)
            d = mfma32(lds_operand(X + 5 * kTile64, n, 2 * step + half),
                       lds_operand(X + 5 * kTile64, 32 + n, 2 * step + half), d);
#pragma unroll
        for (int g = 0; g < 4; ++g)
            store_score_quad(lds, 32 + n, 8 * g + 4 * half, d[4 * g], d[4 * g + 1], d[4 * g + 2], d[4 * g + 3]);
    } else if (wave == 1 || wave == 2) {
        // h = 16: tile (queries 16..31, keys 0..15) or (queries 48..63, keys 32..47); plus one all-zero tile
        // above the diagonal that the 32-row operand reads of step D cover
        const int i0 = (wave == 1) ? 0 : 32, t0 = i0 + 16;
        const int n = lane & 15, g = lane >> 4;
        floatx4_t d = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int kh = 0; kh < 2; ++kh)
            d = mfma16(lds_operand(X + 4 * kTile64, i0 + n, 4 * kh + g),
                       lds_operand(X + 4 * kTile64, t0 + n, 4 * kh + g), d);
        store_score_quad(lds, t0 + n, i0 + 4 * g, d[0], d[1], d[2], d[3]);
        store_score_quad(lds, i0 + n, t0 + 4 * g, 0.f, 0.f, 0.f, 0.f);
    } else if (wave >= 4) {
        // diagonal 16x16 tile: levels h = 1, 2, 4, 8 as masked Gram matrices, plus the undecayed diagonal
        const int t0 = 16 * (wave - 4);
        const int n = lane & 15, g = lane >> 4;
        floatx4_t acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int lvl = 0; lvl < 4; ++lvl) {
            const int h = 1 << lvl;
            floatx4_t d = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int kh = 0; kh < 2; ++kh) {
                const bf16x8_t x = lds_operand(X + lvl * kTile64, t0 + n, 4 * kh + g);
                d = mfma16(x, x, d);
            }
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int m = 4 * g + r;      // key row inside the tile
                const bool keep = (n & h) && !(m & h) && ((n >> (lvl + 1)) == (m >> (lvl + 1)));
                acc[r] += keep ? d[r] : 0.f;
            }
        }
        floatx4_t d = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int kh = 0; kh < 2; ++kh)
            d = mfma16(lds_operand(lds + kOffKraw, t0 + n, 4 * kh + g), lds_operand(lds + kOffQraw, t0 + n, 4 * kh + g), d);
#pragma unroll
        for (int r = 0; r < 4; ++r) acc[r] += (4 * g + r == n) ? d[r] : 0.f;
        store_score_quad(lds, t0 + n, t0 + 4 * g, acc[0], acc[1], acc[2], acc[3]);
    }
}

__global__ __launch_bounds__(kThreads) void scan_mfma_kernel(
    const bf16_t *__restrict__ q, const bf16_t *__restrict__ k, const bf16_t *__restrict__ v,
    const float *__restrict__ log_alpha, const float *__restrict__ beta, const float *S0,
    bf16_t *__restrict__ o, float *S_T, int T, int H, int dv)
{
    extern __shared__ __align__(16) unsigned char lds[];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int rh = wave >> 2, cs = wave & 3;          // this wavefront's 32-row half and 32-column slab
    const int n = lane & 31, half = lane >> 5;
    const int bh = blockIdx.x;

    Geometry g;
    g.q = q; g.k = k; g.v = v; g.la = log_alpha; g.beta = beta;
    g.T = T; g.H = H; g.dv = dv;
    g.b = bh / H; g.h = bh % H; g.j0 = blockIdx.y * kColTile;
    const bool has_beta = beta != nullptr;

    // state tile in accumulators: register r holds row 32rh + 8(r/4) + 4half + r%4, column 32cs + n
    const size_t state_base = (size_t)bh * kK * dv + g.j0 + 32 * cs + n;
    floatx16_t S;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        const int row = 32 * rh + 8 * (r >> 2) + 4 * half + (r & 3);
        S[r] = (S0 != nullptr) ? S0[state_base + (size_t)row * dv] : 0.f;
    }
    auto publish_state = [&]() {      // bf16 copy of the state, transposed, for the next chunk's step C
#pragma unroll
        for (int gq = 0; gq < 4; ++gq) {
            const int n0 = 32 * rh + 8 * gq + 4 * half;
            uint2 w = {pack_bf16x2(S[4 * gq], S[4 * gq + 1]), pack_bf16x2(S[4 * gq + 2], S[4 * gq + 3])};
            *reinterpret_cast<uint2 *>(lds + kOffSt + boff(32 * cs + n, n0 >> 3) + (n0 & 7) * 2) = w;
        }
    };
    publish_state();

    Prefetch pf;
    if (T > 0) prefetch_chunk(g, 0, tid, pf);

    for (int s = 0; s < T; s += kC) {
        // ---- A
        stage_chunk(lds, tid, pf, has_beta);
        if (s + kC < T) prefetch_chunk(g, s + kC, tid, pf);
        __syncthreads();

        // ---- B
        build_versions(lds, lane, wave);
        __syncthreads();

        // ---- C
        floatx16_t O = {0.f};
#pragma unroll
        for (int step = 0; step < 4; ++step)
            O = mfma32(lds_operand(lds + kOffQin, 32 * rh + n, 2 * step + half),
                       lds_operand(lds + kOffSt, 32 * cs + n, 2 * step + half), O);
        score_tiles(lds, lane, wave);
        __syncthreads();

        // ---- D
        bf16x8_t gv[4];
#pragma unroll
        for (int step = 0; step < 4; ++step) gv[step] = lds_operand(lds + kOffGVt, 32 * cs + n, 2 * step + half);
#pragma unroll
        for (int step = 0; step < 4; ++step)
            if (step < 2 * (rh + 1))          // causal: rows 0..31 only see keys 0..31
                O = mfma32(lds_operand(lds + kOffPm, 32 * rh + n, 2 * step + half), gv[step], O);
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int t = s + 32 * rh + 8 * (r >> 2) + 4 * half + (r & 3);
            if (t < T) o[(((size_t)g.b * T + t) * H + g.h) * dv + g.j0 + 32 * cs + n] = (bf16_t)O[r];
        }
        const float *gam = reinterpret_cast<const float *>(lds + kOffGam);
#pragma unroll
        for (int gq = 0; gq < 4; ++gq) {
            const floatx4_t dec = *reinterpret_cast<const floatx4_t *>(gam + 32 * rh + 8 * gq + 4 * half);
#pragma unroll
            for (int e = 0; e < 4; ++e) S[4 * gq + e] *= dec[e];
        }
#pragma unroll
        for (int step = 0; step < 4; ++step)
            S = mfma32(lds_operand(lds + kOffKstT, 32 * rh + n, 2 * step + half), gv[step], S);
        publish_state();
        __syncthreads();
    }

    if (S_T != nullptr) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int row = 32 * rh + 8 * (r >> 2) + 4 * half + (r & 3);
            S_T[state_base + (size_t)row * dv] = S[r];
        }
    }
}

}  // namespace

bool scan_mfma_supports(int dk, int dv, int chunk, int io_dtype)
{
    return io_dtype == RODIMUS_BF16 && dk == kK && chunk == kC && dv >= kColTile && dv % kColTile == 0;
}

hipError_t launch_scan_mfma(const ScanArgs &a)
{
    if ((long long)a.B * a.H == 0) return hipSuccess;
    if (a.T == 0 && (a.S_T == nullptr || a.S_T == a.S0)) return hipSuccess;
    hipError_t err = hipFuncSetAttribute(reinterpret_cast<const void *>(&scan_mfma_kernel),
                                         hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBytes);
    if (err != hipSuccess) return err;
    dim3 grid((unsigned)(a.B * a.H), (unsigned)(a.dv / kColTile)), block(kThreads);
    hipLaunchKernelGGL(scan_mfma_kernel, grid, block, kLdsBytes, a.stream, (const bf16_t *)a.q, (const bf16_t *)a.k,
                       (const bf16_t *)a.v, a.log_alpha, a.beta, a.S0, (bf16_t *)a.o, a.S_T, a.T, a.H, a.dv);
    return hipGetLastError();
}

}  // namespace rodimus
