// qnn_binary_gemm: M x K multi-branch binary GEMM on packed {-1,+1} planes (paper: Eq. 7-9 with
// Eq. 10, Fig. 1), recombined in the epilogue and optionally scaled per output channel (Eq. 18).
#include "bdot_tile.h"
#include "qnn_host.h"

namespace qnn {

struct GemmParams {
    const uint32_t *a; // [AB][rows][nw]
    const uint32_t *w; // [WB][cols][nw]
    int64_t rows, cols, nw;
    uint32_t n_times_top; // n (2^WB - 1)(2^AB - 1)
    int32_t *acc;         // or nullptr
    const float *scale;   // or nullptr
    float *out;           // or nullptr
    int vec;              // nw % 4 == 0: 16-byte loads of the planes are aligned
    int64_t tiles_n, nblocks;
    // Bit widths above 4 run as up to four launches over chunks of at most 4 planes per operand:
    // Eq. 9's double sum splits into chunk pairs, each an ordinary (<= 4) x (<= 4) product whose
    // result enters with the weight 2^shift of its lowest planes.
    int shift;                  // weight of this chunk pair
    const int32_t *partial_in;  // sum of the chunk pairs done so far, or nullptr
    int32_t *partial_out;       // where to leave the running sum (not the last chunk pair), or nullptr
};

// WPE = waves per SIMD the kernel is compiled for (2: up to 256 registers per lane, 4: up to 128).
template <int WB, int AB, int TM, int TN, int KV, int WPE>
__global__ __launch_bounds__(kTileThreads) __attribute__((amdgpu_waves_per_eu(WPE, WPE))) void bgemm_tile_kernel(GemmParams p)
{
    using T = Tile<WB, AB, TM, TN, KV>;
    __shared__ __attribute__((aligned(16))) uint32_t smem[2][T::STAGE_WORDS];

    const int tid = threadIdx.x;
    const int tx = tid & 15, ty = tid >> 4;
    const int64_t tile = xcd_band_remap(blockIdx.x, p.nblocks);
    int64_t tm, tn;
    grouped_tile(tile, p.nblocks / p.tiles_n, p.tiles_n, tm, tn);
    const int64_t row0 = tm * T::BM;
    const int64_t col0 = tn * T::BN;
    const bool vec = p.vec != 0;

    uint32_t P[TM][TN][T::S];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int n = 0; n < TN; ++n)
#pragma unroll
            for (int s = 0; s < T::S; ++s) P[i][n][s] = 0u;

    uint4 ra[T::A_PER_THREAD], rw[T::W_PER_THREAD];

    auto fetch = [&](int64_t k0) {
#pragma unroll
        for (int u = 0; u < T::A_PER_THREAD; ++u) {
            const int idx = tid + u * kTileThreads;
            const int rp = idx >> 2, q = idx & 3;
            ra[u] = make_uint4(0u, 0u, 0u, 0u);
            if (T::A_UNITS % kTileThreads == 0 || idx < T::A_UNITS)
                ra[u] = load_rowmajor4(p.a, p.rows, p.nw, rp / T::BM, row0 + rp % T::BM,
                                       k0 + 4 * q, vec);
        }
#pragma unroll
        for (int u = 0; u < T::W_PER_THREAD; ++u) {
            const int idx = tid + u * kTileThreads;
            const int rp = idx >> 2, q = idx & 3;
            rw[u] = make_uint4(0u, 0u, 0u, 0u);
            if (T::W_UNITS % kTileThreads == 0 || idx < T::W_UNITS)
                rw[u] = load_rowmajor4(p.w, p.cols, p.nw, rp / T::BN, col0 + rp % T::BN,
                                       k0 + 4 * q, vec);
        }
    };
    auto stash = [&](int buf) {
        uint32_t *As = smem[buf], *Ws = smem[buf] + T::A_WORDS;
#pragma unroll
        for (int u = 0; u < T::A_PER_THREAD; ++u) {
            const int idx = tid + u * kTileThreads;
            if (T::A_UNITS % kTileThreads == 0 || idx < T::A_UNITS)
                lds_write_unit<KV>(As + (idx >> 2) * T::BKP + 4 * (idx & 3), ra[u]);
        }
#pragma unroll
        for (int u = 0; u < T::W_PER_THREAD; ++u) {
            const int idx = tid + u * kTileThreads;
            if (T::W_UNITS % kTileThreads == 0 || idx < T::W_UNITS)
                lds_write_unit<KV>(Ws + (idx >> 2) * T::BKP + 4 * (idx & 3), rw[u]);
        }
    };

    const int64_t nchunks = (p.nw + kBK - 1) / kBK;
    fetch(0);
    stash(0);
    __syncthreads();
    for (int64_t c = 0; c < nchunks; ++c) {
        const int buf = (int)(c & 1);
        const bool more = c + 1 < nchunks;
        if (more) fetch((c + 1) * kBK);
        const int64_t left = p.nw - c * kBK; // reduction words still to do
        const int nkq = left >= kBK ? kBK / KV : (int)((left + KV - 1) / KV);
        tile_mac<WB, AB, TM, TN, KV, kBK>(smem[buf], smem[buf] + T::A_WORDS, ty, tx, nkq, P);
        if (more) stash(buf ^ 1);
        __syncthreads();
    }

    // Epilogue.  The recombined accumulators go through LDS once so that the stores run row-major:
    // a lane owns 4 consecutive columns of one row (16-byte acc / out stores, 16 B x BN / 4 lanes =
    // whole 256- or 512-byte row pieces per wave) instead of 64-byte pieces of 4 rows.  The stage
    // buffers are free (the loop ends with a barrier); when they cannot hold the whole block the rows
    // go through in rounds of 16 IPR.
    constexpr int EPI_STRIDE = T::BN + 16;
    constexpr int IPR = (2 * T::STAGE_WORDS) / (16 * EPI_STRIDE) < TM ? (2 * T::STAGE_WORDS) / (16 * EPI_STRIDE) : TM;
    static_assert(IPR >= 1, "the stage buffers hold at least 16 rows of the block");
    constexpr int LPR = T::BN / 4;            // lanes per row
    constexpr int RPP = kTileThreads / LPR;   // rows per pass
    static_assert((16 * IPR) % RPP == 0 || RPP > 16 * IPR, "passes cover whole rounds");
    int32_t *V = reinterpret_cast<int32_t *>(&smem[0][0]);
    const int c4 = (tid % LPR) * 4;
    const int64_t cidx = col0 + c4;
    const bool cols4 = cidx + 3 < p.cols && (p.cols & 3) == 0; // 16-byte accesses are whole and aligned
    float sc[4] = {0.f, 0.f, 0.f, 0.f};
    if (p.out && !p.partial_out) {
#pragma unroll
        for (int e = 0; e < 4; ++e)
            if (cidx + e < p.cols) sc[e] = p.scale[cidx + e];
    }
#pragma unroll
    for (int i0 = 0; i0 < TM; i0 += IPR) {
        if (i0 > 0) __syncthreads(); // the previous round's rows have been read
#pragma unroll
        for (int i = i0; i < i0 + IPR && i < TM; ++i)
#pragma unroll
            for (int n = 0; n < TN; ++n)
                V[((i - i0) * 16 + ty) * EPI_STRIDE + tx + 16 * n] = recombine<T::S>(P[i][n], p.n_times_top);
        __syncthreads();
        constexpr int kRoundRows = 16 * IPR;
#pragma unroll 1
        for (int rl = tid / LPR; rl < kRoundRows && i0 + rl / 16 < TM; rl += RPP) {
            const int64_t r = row0 + (rl % 16) + 16 * (i0 + rl / 16);
            if (r >= p.rows || cidx >= p.cols) continue;
            const int4 vv = *reinterpret_cast<const int4 *>(V + rl * EPI_STRIDE + c4);
            int32_t v[4] = {vv.x, vv.y, vv.z, vv.w};
            const int64_t o = r * p.cols + cidx;
#pragma unroll
            for (int e = 0; e < 4; ++e) v[e] = (int32_t)((uint32_t)v[e] << p.shift);
            if (cols4) {
                if (p.partial_in) {
                    const int4 q = *reinterpret_cast<const int4 *>(p.partial_in + o);
                    v[0] += q.x, v[1] += q.y, v[2] += q.z, v[3] += q.w;
                }
                if (p.partial_out) {
                    *reinterpret_cast<int4 *>(p.partial_out + o) = make_int4(v[0], v[1], v[2], v[3]);
                    continue;
                }
                if (p.acc) *reinterpret_cast<int4 *>(p.acc + o) = make_int4(v[0], v[1], v[2], v[3]);
                if (p.out)
                    *reinterpret_cast<float4 *>(p.out + o) =
                        make_float4((float)v[0] * sc[0], (float)v[1] * sc[1], (float)v[2] * sc[2], (float)v[3] * sc[3]);
            } else {
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    if (cidx + e >= p.cols) continue;
                    if (p.partial_in) v[e] += p.partial_in[o + e];
                    if (p.partial_out) {
                        p.partial_out[o + e] = v[e];
                        continue;
                    }
                    if (p.acc) p.acc[o + e] = v[e];
                    if (p.out) p.out[o + e] = (float)v[e] * sc[e];
                }
            }
        }
    }
}

template <int WB, int AB, int TM, int TN, int KV, int WPE> static void launch_tile(GemmParams p, hipStream_t st)
{
    using T = Tile<WB, AB, TM, TN, KV>;
    const int64_t tiles_m = ceil_div(p.rows, T::BM);
    p.tiles_n = ceil_div(p.cols, T::BN);
    p.nblocks = tiles_m * p.tiles_n;
    hipLaunchKernelGGL((bgemm_tile_kernel<WB, AB, TM, TN, KV, WPE>), dim3((unsigned)p.nblocks),
                       dim3(kTileThreads), 0, st, p);
}

template <int WB, int AB> static void launch_pick(const GemmParams &p, hipStream_t st)
{
    using G = TilePick<WB, AB>;
    launch_tile<WB, AB, G::TM, G::TN, G::KV, G::WPE>(p, st);
}

template <int WB> static bool dispatch_a(int a_bits, const GemmParams &p, hipStream_t st)
{
    switch (a_bits) {
    case 1: launch_pick<WB, 1>(p, st); return true;
    case 2: launch_pick<WB, 2>(p, st); return true;
    case 3: launch_pick<WB, 3>(p, st); return true;
    case 4: launch_pick<WB, 4>(p, st); return true;
    default: return false;
    }
}

} // namespace qnn

using namespace qnn;

extern "C" int qnn_binary_gemm(const uint32_t *a_planes, int a_bits, const uint32_t *w_planes,
                               int w_bits, int64_t rows, int64_t cols, int64_t n, int32_t *acc,
                               const float *scale, float *out, void *stream)
{
    if (a_bits < 1 || a_bits > 8 || w_bits < 1 || w_bits > 8)
        return fail(QNN_ERR_INVALID_ARG, "qnn_binary_gemm: bits must be in [1,8] (a_bits=%d, w_bits=%d)",
                    a_bits, w_bits);
    if (rows < 0 || cols < 0 || n < 0)
        return fail(QNN_ERR_INVALID_ARG, "qnn_binary_gemm: negative size (rows=%lld cols=%lld n=%lld)",
                    (long long)rows, (long long)cols, (long long)n);
    if (!acc && !out) return fail(QNN_ERR_INVALID_ARG, "qnn_binary_gemm: acc and out are both NULL");
    if (out && !scale) return fail(QNN_ERR_INVALID_ARG, "qnn_binary_gemm: out given without scale");
    if (rows == 0 || cols == 0) return QNN_OK;
    if (n > 0 && (!a_planes || !w_planes))
        return fail(QNN_ERR_INVALID_ARG, "qnn_binary_gemm: NULL plane pointer");
    if (!aligned16(a_planes) || !aligned16(w_planes) || !aligned16(acc) || !aligned16(out))
        return fail(QNN_ERR_ALIGNMENT, "qnn_binary_gemm: pointers must be 16-byte aligned");
    if (!acc_fits_int32(n, w_bits, a_bits))
        return fail(QNN_ERR_RANGE, "qnn_binary_gemm: n=%lld with %dx%d bits overflows int32",
                    (long long)n, w_bits, a_bits);
    if (rows * cols / cols != rows || rows > (INT64_MAX >> 8) / cols)
        return fail(QNN_ERR_RANGE, "qnn_binary_gemm: rows*cols too large");

    GemmParams p;
    p.a = a_planes;
    p.w = w_planes;
    p.rows = rows;
    p.cols = cols;
    p.nw = ceil_div(n, 32);
    p.acc = acc;
    p.scale = scale;
    p.out = out;
    p.vec = (p.nw % 4 == 0) ? 1 : 0;
    p.tiles_n = p.nblocks = 0;
    hipStream_t st = static_cast<hipStream_t>(stream);

    // chunk pairs of at most 4 x 4 planes; the running int32 sum lives in acc, or (bit for bit) in
    // the memory of out when no acc was asked for -- the last launch turns it into the results
    int32_t *running = acc ? acc : reinterpret_cast<int32_t *>(out);
    const int w_chunks = (w_bits + 3) / 4, a_chunks = (a_bits + 3) / 4;
    int launch = 0;
    for (int cw = 0; cw < w_chunks; ++cw)
        for (int ca = 0; ca < a_chunks; ++ca, ++launch) {
            const int wb = w_bits - 4 * cw < 4 ? w_bits - 4 * cw : 4;
            const int ab = a_bits - 4 * ca < 4 ? a_bits - 4 * ca : 4;
            GemmParams q = p;
            q.w = w_planes + (int64_t)4 * cw * cols * p.nw;
            q.a = a_planes + (int64_t)4 * ca * rows * p.nw;
            q.n_times_top = (uint32_t)(n * ((1 << wb) - 1) * ((1 << ab) - 1));
            q.shift = 4 * (cw + ca);
            q.partial_in = launch > 0 ? running : nullptr;
            q.partial_out = launch + 1 < w_chunks * a_chunks ? running : nullptr;
            bool done = false;
            switch (wb) {
            case 1: done = dispatch_a<1>(ab, q, st); break;
            case 2: done = dispatch_a<2>(ab, q, st); break;
            case 3: done = dispatch_a<3>(ab, q, st); break;
            default: done = dispatch_a<4>(ab, q, st); break;
            }
            if (!done) return fail(QNN_ERR_UNSUPPORTED, "qnn_binary_gemm: no kernel for %d x %d planes", wb, ab);
            const int rc = check_launch("qnn_binary_gemm");
            if (rc != QNN_OK) return rc;
        }
    return QNN_OK;
}
