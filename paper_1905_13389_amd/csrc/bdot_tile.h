// Register-blocked xor + bitcount tile engine shared by the binary GEMM and the implicit-im2col
// binary convolution (paper: Eq. 9 with the {-1,+1} code of Eq. 10; "xnor and bitcount").
//
// A workgroup of 256 lanes (4 wave64) owns a BM x BN block of outputs, BM = 16*TM rows,
// BN = 16*TN columns.  Lane (ty, tx) owns rows ty + 16*i and columns tx + 16*n, so that within
// a wave the activation reads are 4 broadcast addresses and the weight reads are 16 distinct
// LDS rows whose stride (an odd multiple of 4 words) spreads them over all banks.
//
// For every 32-bit word of the reduction axis and every (weight plane i, activation plane j)
// the lane issues one v_xor_b32 and one v_bcnt_u32_b32 whose add operand is the running count,
// so the inner loop holds nothing but those two instructions and the LDS reads feeding them.
// Counts of plane pairs with equal i + j share one accumulator P_s (s = i + j): the
// recombination sum_ij 2^(i+j) y_ij, y_ij = n - 2 P_ij, becomes
//     acc = n (2^WB - 1)(2^AB - 1) - 2 sum_s 2^s P_s
// applied once in the epilogue, with WB + AB - 1 accumulators per output instead of WB * AB.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace qnn {

constexpr int kTileThreads = 256;
constexpr int kBK = 16; // default number of reduction words staged per step (64 bytes per row and plane)

// KV = reduction words fetched from LDS per read (4: ds_read_b128, 2: ds_read_b64); the lane keeps
// KV * (TM*AB + TN*WB) operand registers next to its TM*TN*(WB+AB-1) counters.
// KB = reduction words an LDS stage can hold (a multiple of 4).  The LDS row stride BKP (words) is
// chosen so that the 16 rows a wave reads together fall into different banks (32 banks of 4
// bytes, one pass serves 128 bytes): for 16-byte reads (KV = 4, 8 lanes per pass) an odd multiple
// of 4 words; for 8-byte reads (KV = 2, 16 lanes per pass) twice an odd number, which leaves the
// rows 8-byte aligned only, so stages are then written with 8-byte stores.
// NT = lanes of the workgroup (256 or 512): NT / 16 row groups of 16 lanes, lane (ty, tx) owns rows ty + (NT/16) i.
template <int WB, int AB, int TM, int TN, int KV = 4, int KB = kBK, int NT = kTileThreads> struct Tile {
    static_assert(KV == 2 || KV == 4, "KV is 2 or 4 words");
    static_assert(KB % 4 == 0, "stages are loaded in 16-byte units");
    static_assert(NT % 64 == 0, "whole waves");
    static constexpr int RG = NT / 16; // row groups
    static constexpr int UQ = KB / 4;  // 16-byte units per row and plane
    static constexpr int BKP = KV == 4 ? ((UQ % 2 == 1) ? KB : KB + 4) : KB + 2;
    static constexpr int BM = RG * TM;
    static constexpr int BN = 16 * TN;
    static constexpr int S = WB + AB - 1;
    static constexpr int A_ROWPLANES = AB * BM;
    static constexpr int W_ROWPLANES = WB * BN;
    static constexpr int A_UNITS = A_ROWPLANES * UQ; // one unit = 4 words of one row-plane
    static constexpr int W_UNITS = W_ROWPLANES * UQ;
    static constexpr int A_PER_THREAD = (A_UNITS + NT - 1) / NT;
    static constexpr int W_PER_THREAD = (W_UNITS + NT - 1) / NT;
    static constexpr int A_WORDS = A_ROWPLANES * BKP;
    static constexpr int STAGE_WORDS = (A_ROWPLANES + W_ROWPLANES) * BKP;
};

// Lane tile, LDS read width and occupancy per (w_bits, a_bits), chosen by measurement at 4096^3 (every candidate
// below was timed against the others on one device).  What decides: a wave issues at most one instruction every
// four to five cycles, so one xor / count pair (plus the s_nop that keeps the pairs from stalling each other)
// costs a wave about 13 cycles and a SIMD needs two waves that are ready to issue at every moment to reach its
// 6.5 cycles per pair.  With two resident waves per SIMD every LDS wait, barrier or store of one wave idles half
// the SIMD; with four (at most 128 registers per lane) two may wait while two issue.  So the tiles are small:
// TM*TN*(WB+AB-1) counters plus KV*(TM*AB + TN*WB) operand registers stay near 100, the short side of a
// rectangular tile is on the operand with more planes (a k group reads TM*AB + TN*WB operand words for its
// TM*TN*WB*AB pairs), and only 4 x 4 bits, whose 2 x 2 lane tile would fit even more waves, gains nothing from
// a larger tile at lower occupancy.  Fractions of the VALU peak at 4096^3, before -> after this choice:
// 1x1 0.62 -> 0.74, 1x2 0.62 -> 0.77, 2x2 0.75 -> 0.83, 3x3 0.82 -> 0.86, 4x4 0.84 -> 0.87.
template <int WB, int AB> struct TilePick;
template <> struct TilePick<1, 1> { static constexpr int TM = 8, TN = 4, KV = 4, WPE = 4; };
template <> struct TilePick<1, 2> { static constexpr int TM = 4, TN = 4, KV = 4, WPE = 4; };
template <> struct TilePick<2, 1> { static constexpr int TM = 4, TN = 4, KV = 4, WPE = 4; };
template <> struct TilePick<1, 3> { static constexpr int TM = 2, TN = 4, KV = 4, WPE = 4; };
template <> struct TilePick<3, 1> { static constexpr int TM = 4, TN = 2, KV = 4, WPE = 4; };
template <> struct TilePick<1, 4> { static constexpr int TM = 2, TN = 4, KV = 4, WPE = 4; };
template <> struct TilePick<4, 1> { static constexpr int TM = 4, TN = 2, KV = 4, WPE = 4; };
template <> struct TilePick<2, 2> { static constexpr int TM = 4, TN = 4, KV = 2, WPE = 4; };
template <> struct TilePick<2, 3> { static constexpr int TM = 2, TN = 4, KV = 4, WPE = 4; };
template <> struct TilePick<3, 2> { static constexpr int TM = 4, TN = 2, KV = 4, WPE = 4; };
template <> struct TilePick<2, 4> { static constexpr int TM = 2, TN = 4, KV = 2, WPE = 4; };
template <> struct TilePick<4, 2> { static constexpr int TM = 4, TN = 2, KV = 2, WPE = 4; };
template <> struct TilePick<3, 3> { static constexpr int TM = 4, TN = 2, KV = 4, WPE = 4; };
template <> struct TilePick<3, 4> { static constexpr int TM = 2, TN = 4, KV = 2, WPE = 4; };
template <> struct TilePick<4, 3> { static constexpr int TM = 4, TN = 2, KV = 2, WPE = 4; };
template <> struct TilePick<4, 4> { static constexpr int TM = 2, TN = 2, KV = 2, WPE = 4; };

// Workgroup id -> tile id so that the workgroups an XCD receives (ids congruent mod 8 under
// round-robin dispatch) cover one contiguous band of tiles and share operands in that XCD's L2.
__device__ __forceinline__ int64_t xcd_band_remap(int64_t pid, int64_t nblocks)
{
    constexpr int64_t kXcds = 8;
    if (nblocks < 2 * kXcds) return pid;
    const int64_t xcd = pid % kXcds, local = pid / kXcds;
    const int64_t per = (nblocks + kXcds - 1) / kXcds;
    const int64_t rem = nblocks % kXcds;
    const int64_t tall = rem == 0 ? kXcds : rem; // XCDs that receive `per` workgroups
    if (xcd < tall) return xcd * per + local;
    return tall * per + (xcd - tall) * (per - 1) + local;
}

// Linear tile id -> (tile row, tile column), walking kGroupRows tile rows down before moving one
// tile column right.  The workgroups resident on an XCD at one time then cover a few tile rows
// (their activation planes stay in that XCD's L2) and every weight tile they stream is shared by
// kGroupRows workgroups instead of being fetched again for every tile row.
constexpr int kGroupRows = 4;
__device__ __forceinline__ void grouped_tile(int64_t tile, int64_t tiles_m, int64_t tiles_n, int64_t &tm,
                                             int64_t &tn)
{
    const int64_t per_group = kGroupRows * tiles_n;
    const int64_t group = tile / per_group, in_group = tile % per_group;
    const int64_t first = group * kGroupRows;
    const int64_t rows = tiles_m - first < kGroupRows ? tiles_m - first : kGroupRows;
    tm = first + in_group % rows;
    tn = in_group / rows;
}

// 4 reduction words of one row of a [plane][R][nw] row-major plane tensor; words past nw and
// rows past R read as 0 (a zero word xors to the other operand's zero word: no contribution).
__device__ __forceinline__ uint4 load_rowmajor4(const uint32_t *__restrict__ base, int64_t R,
                                                int64_t nw, int plane, int64_t row, int64_t kword,
                                                bool vec)
{
    uint4 v = make_uint4(0u, 0u, 0u, 0u);
    if (row < R && kword < nw) {
        const uint32_t *p = base + ((int64_t)plane * R + row) * nw + kword;
        if (vec) {
            v = *reinterpret_cast<const uint4 *>(p);
        } else {
            v.x = p[0];
            if (kword + 1 < nw) v.y = p[1];
            if (kword + 2 < nw) v.z = p[2];
            if (kword + 3 < nw) v.w = p[3];
        }
    }
    return v;
}

// All WB x AB plane pairs of one weight word column and one activation word column:
// count[i + j] += bitcount(w[i] xor a[j]), exactly one v_xor_b32 and one v_bcnt_u32_b32 (whose
// third operand is the running count) per pair.  One asm statement per call, so the compiler can
// neither re-associate the count chains into extra adds nor keep hundreds of xor results alive.
//
// Issue order.  On gfx950 a wave64 v_xor_b32 occupies its SIMD for about 2.4 cycles and a
// v_bcnt_u32_b32 for about 4.4 (measured with register-only loops, 2 or 4 waves per SIMD), but
// only when something that is not a VALU instruction follows each xor/count pair: back-to-back
// pairs cost about 10 cycles per pair instead of 6.7.  Hence the s_nop 0 after every pair (the
// compiler puts one between asm statements on its own, which covers the single-pair cases).
#define QNN_XB1(w, a, p) "v_xor_b32 %[t], %[" #w "], %[" #a "]\n\tv_bcnt_u32_b32 %[" #p "], %[t], %[" #p "]\n\t"
#define QNN_XB(w, a, p) QNN_XB1(w, a, p) "s_nop 0\n\t"
#define QNN_ROW1(w, p0) QNN_XB(w, a0, p0)
#define QNN_ROW2(w, p0, p1) QNN_XB(w, a0, p0) QNN_XB(w, a1, p1)
#define QNN_ROW3(w, p0, p1, p2) QNN_XB(w, a0, p0) QNN_XB(w, a1, p1) QNN_XB(w, a2, p2)
#define QNN_ROW4(w, p0, p1, p2, p3) QNN_XB(w, a0, p0) QNN_XB(w, a1, p1) QNN_XB(w, a2, p2) QNN_XB(w, a3, p3)
#define QNN_P1 [p0] "+v"(c[0])
#define QNN_P2 QNN_P1, [p1] "+v"(c[1])
#define QNN_P3 QNN_P2, [p2] "+v"(c[2])
#define QNN_P4 QNN_P3, [p3] "+v"(c[3])
#define QNN_P5 QNN_P4, [p4] "+v"(c[4])
#define QNN_P6 QNN_P5, [p5] "+v"(c[5])
#define QNN_P7 QNN_P6, [p6] "+v"(c[6])
#define QNN_W1 [w0] "v"(w[0])
#define QNN_W2 QNN_W1, [w1] "v"(w[1])
#define QNN_W3 QNN_W2, [w2] "v"(w[2])
#define QNN_W4 QNN_W3, [w3] "v"(w[3])
#define QNN_A1 [a0] "v"(a[0])
#define QNN_A2 QNN_A1, [a1] "v"(a[1])
#define QNN_A3 QNN_A2, [a2] "v"(a[2])
#define QNN_A4 QNN_A3, [a3] "v"(a[3])
#define QNN_PAIRS(body, P, W, A) asm(body : [t] "=&v"(t), P : W, A)

template <int WB, int AB>
__device__ __forceinline__ void xor_bcnt_pairs(const uint32_t (&w)[WB], const uint32_t (&a)[AB],
                                               uint32_t (&c)[WB + AB - 1])
{
    uint32_t t;
    if constexpr (WB == 1 && AB == 1) QNN_PAIRS(QNN_XB1(w0, a0, p0), QNN_P1, QNN_W1, QNN_A1);
    else if constexpr (WB == 1 && AB == 2) QNN_PAIRS(QNN_ROW2(w0, p0, p1), QNN_P2, QNN_W1, QNN_A2);
    else if constexpr (WB == 1 && AB == 3) QNN_PAIRS(QNN_ROW3(w0, p0, p1, p2), QNN_P3, QNN_W1, QNN_A3);
    else if constexpr (WB == 1 && AB == 4) QNN_PAIRS(QNN_ROW4(w0, p0, p1, p2, p3), QNN_P4, QNN_W1, QNN_A4);
    else if constexpr (WB == 2 && AB == 1) QNN_PAIRS(QNN_ROW1(w0, p0) QNN_ROW1(w1, p1), QNN_P2, QNN_W2, QNN_A1);
    else if constexpr (WB == 2 && AB == 2)
        QNN_PAIRS(QNN_ROW2(w0, p0, p1) QNN_ROW2(w1, p1, p2), QNN_P3, QNN_W2, QNN_A2);
    else if constexpr (WB == 2 && AB == 3)
        QNN_PAIRS(QNN_ROW3(w0, p0, p1, p2) QNN_ROW3(w1, p1, p2, p3), QNN_P4, QNN_W2, QNN_A3);
    else if constexpr (WB == 2 && AB == 4)
        QNN_PAIRS(QNN_ROW4(w0, p0, p1, p2, p3) QNN_ROW4(w1, p1, p2, p3, p4), QNN_P5, QNN_W2, QNN_A4);
    else if constexpr (WB == 3 && AB == 1)
        QNN_PAIRS(QNN_ROW1(w0, p0) QNN_ROW1(w1, p1) QNN_ROW1(w2, p2), QNN_P3, QNN_W3, QNN_A1);
    else if constexpr (WB == 3 && AB == 2)
        QNN_PAIRS(QNN_ROW2(w0, p0, p1) QNN_ROW2(w1, p1, p2) QNN_ROW2(w2, p2, p3), QNN_P4, QNN_W3, QNN_A2);
    else if constexpr (WB == 3 && AB == 3)
        QNN_PAIRS(QNN_ROW3(w0, p0, p1, p2) QNN_ROW3(w1, p1, p2, p3) QNN_ROW3(w2, p2, p3, p4), QNN_P5, QNN_W3,
                  QNN_A3);
    else if constexpr (WB == 3 && AB == 4)
        QNN_PAIRS(QNN_ROW4(w0, p0, p1, p2, p3) QNN_ROW4(w1, p1, p2, p3, p4) QNN_ROW4(w2, p2, p3, p4, p5), QNN_P6,
                  QNN_W3, QNN_A4);
    else if constexpr (WB == 4 && AB == 1)
        QNN_PAIRS(QNN_ROW1(w0, p0) QNN_ROW1(w1, p1) QNN_ROW1(w2, p2) QNN_ROW1(w3, p3), QNN_P4, QNN_W4, QNN_A1);
    else if constexpr (WB == 4 && AB == 2)
        QNN_PAIRS(QNN_ROW2(w0, p0, p1) QNN_ROW2(w1, p1, p2) QNN_ROW2(w2, p2, p3) QNN_ROW2(w3, p3, p4), QNN_P5,
                  QNN_W4, QNN_A2);
    else if constexpr (WB == 4 && AB == 3)
        QNN_PAIRS(QNN_ROW3(w0, p0, p1, p2) QNN_ROW3(w1, p1, p2, p3) QNN_ROW3(w2, p2, p3, p4)
                      QNN_ROW3(w3, p3, p4, p5),
                  QNN_P6, QNN_W4, QNN_A3);
    else {
        static_assert(WB == 4 && AB == 4, "plane pairs are built for 1..4 x 1..4 bits");
        QNN_PAIRS(QNN_ROW4(w0, p0, p1, p2, p3) QNN_ROW4(w1, p1, p2, p3, p4) QNN_ROW4(w2, p2, p3, p4, p5)
                      QNN_ROW4(w3, p3, p4, p5, p6),
                  QNN_P7, QNN_W4, QNN_A4);
    }
}

// Store one 4-word unit of a stage row (16-byte store when the row stride keeps that alignment).
template <int KV> __device__ __forceinline__ void lds_write_unit(uint32_t *dst, const uint4 &v)
{
    if constexpr (KV == 4) {
        *reinterpret_cast<uint4 *>(dst) = v;
    } else {
        *reinterpret_cast<uint2 *>(dst) = make_uint2(v.x, v.y);
        *reinterpret_cast<uint2 *>(dst + 2) = make_uint2(v.z, v.w);
    }
}

// The xor + bitcount block: one stage out of LDS into the P_s accumulators.
template <int KV> __device__ __forceinline__ void lds_read_words(const uint32_t *p, uint32_t (&dst)[KV])
{
    if constexpr (KV == 4) {
        const uint4 v = *reinterpret_cast<const uint4 *>(p);
        dst[0] = v.x, dst[1] = v.y, dst[2] = v.z, dst[3] = v.w;
    } else {
        const uint2 v = *reinterpret_cast<const uint2 *>(p);
        dst[0] = v.x, dst[1] = v.y;
    }
}

// `nkq` = number of KV-word groups of this stage that hold reduction words (fewer for the last
// stage of a reduction: nothing is spent on the zero tail).  The activation stage holds APR rows per
// plane and the lane's row i sits at row ty + ASTEP * i of it (the whole tile: BM rows, step 16; a
// wave's private quarter of the tile: BM / 4 rows, step 4, ty = the lane's row group inside the wave).
// One group of G reduction words starting at word `word0` of the stage (G = 4: 16-byte reads, G = 2: 8-byte reads).
template <int WB, int AB, int TM, int TN, int KV, int KB, int APR, int ASTEP, int G>
__device__ __forceinline__ void tile_mac_group(const uint32_t *__restrict__ As, const uint32_t *__restrict__ Ws,
                                               int ty, int tx, int word0, uint32_t (&P)[TM][TN][WB + AB - 1])
{
    using T = Tile<WB, AB, TM, TN, KV, KB>;
    uint32_t a[TM][G][AB]; // [row][word][plane]
    uint32_t w[TN][G][WB];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < AB; ++j) {
            uint32_t v[G];
            lds_read_words<G>(As + (j * APR + ty + ASTEP * i) * T::BKP + word0, v);
#pragma unroll
            for (int kk = 0; kk < G; ++kk) a[i][kk][j] = v[kk];
        }
#pragma unroll
    for (int n = 0; n < TN; ++n)
#pragma unroll
        for (int j = 0; j < WB; ++j) {
            uint32_t v[G];
            lds_read_words<G>(Ws + (j * T::BN + tx + 16 * n) * T::BKP + word0, v);
#pragma unroll
            for (int kk = 0; kk < G; ++kk) w[n][kk][j] = v[kk];
        }
#pragma unroll
    for (int kk = 0; kk < G; ++kk)
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int n = 0; n < TN; ++n) xor_bcnt_pairs<WB, AB>(w[n][kk], a[i][kk], P[i][n]);
}

// HALF (KV = 4 only): `half_tail` asks for one more group of 2 words behind the nkq groups of 4 -- a stage
// that ends 1 or 2 words into a group spends nothing on the other two (zero) words.
template <int WB, int AB, int TM, int TN, int KV, int KB, int APR = 16 * TM, int ASTEP = 16, bool HALF = false>
__device__ __forceinline__ void tile_mac(const uint32_t *__restrict__ As,
                                         const uint32_t *__restrict__ Ws, int ty, int tx, int nkq,
                                         uint32_t (&P)[TM][TN][WB + AB - 1], bool half_tail = false)
{
#pragma unroll 1
    for (int kq = 0; kq < nkq; ++kq) tile_mac_group<WB, AB, TM, TN, KV, KB, APR, ASTEP, KV>(As, Ws, ty, tx, KV * kq, P);
    if constexpr (HALF && KV == 4) {
        if (half_tail) tile_mac_group<WB, AB, TM, TN, KV, KB, APR, ASTEP, 2>(As, Ws, ty, tx, KV * nkq, P);
    }
}

// acc = n_times_top - 2 sum_s 2^s P_s, in wrap-around 32-bit arithmetic (the true value fits
// int32, checked on the host, so the wrapped result is exact).
template <int S> __device__ __forceinline__ int32_t recombine(const uint32_t (&P)[S], uint32_t n_times_top)
{
    uint32_t sum = 0;
#pragma unroll
    for (int s = 0; s < S; ++s) sum += P[s] << s;
    return (int32_t)(n_times_top - 2u * sum);
}

} // namespace qnn
