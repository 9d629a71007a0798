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
};

template <int WB, int AB, int TM, int TN, int KV>
__global__ __launch_bounds__(kTileThreads) __attribute__((amdgpu_waves_per_eu(2, 2))) void bgemm_tile_kernel(GemmParams p)
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

#pragma unroll
    for (int i = 0; i < TM; ++i) {
        const int64_t r = row0 + ty + 16 * i;
        if (r >= p.rows) continue;
#pragma unroll
        for (int n = 0; n < TN; ++n) {
            const int64_t cidx = col0 + tx + 16 * n;
            if (cidx >= p.cols) continue;
            const int32_t v = recombine<T::S>(P[i][n], p.n_times_top);
            if (p.acc) p.acc[r * p.cols + cidx] = v;
            if (p.out) p.out[r * p.cols + cidx] = (float)v * p.scale[cidx];
        }
    }
}

// Any bit widths 1..8: one lane per output, plane pairs looped at run time.  Slow and plain; it
// serves the widths the register-blocked kernels are not instantiated for.
__global__ __launch_bounds__(256) void bgemm_plain_kernel(GemmParams p, int w_bits, int a_bits)
{
    const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= p.rows * p.cols) return;
    const int64_t r = idx / p.cols, c = idx % p.cols;
    uint32_t sum = 0;
    for (int i = 0; i < w_bits; ++i) {
        const uint32_t *wp = p.w + ((int64_t)i * p.cols + c) * p.nw;
        for (int j = 0; j < a_bits; ++j) {
            const uint32_t *ap = p.a + ((int64_t)j * p.rows + r) * p.nw;
            uint32_t cnt = 0;
            for (int64_t k = 0; k < p.nw; ++k) cnt += __builtin_popcount(wp[k] ^ ap[k]);
            sum += cnt << (i + j);
        }
    }
    const int32_t v = (int32_t)(p.n_times_top - 2u * sum);
    if (p.acc) p.acc[idx] = v;
    if (p.out) p.out[idx] = (float)v * p.scale[c];
}

template <int WB, int AB, int TM, int TN, int KV> static void launch_tile(GemmParams p, hipStream_t st)
{
    using T = Tile<WB, AB, TM, TN, KV>;
    const int64_t tiles_m = ceil_div(p.rows, T::BM);
    p.tiles_n = ceil_div(p.cols, T::BN);
    p.nblocks = tiles_m * p.tiles_n;
    hipLaunchKernelGGL((bgemm_tile_kernel<WB, AB, TM, TN, KV>), dim3((unsigned)p.nblocks),
                       dim3(kTileThreads), 0, st, p);
}

template <int WB, int AB> static void launch_pick(const GemmParams &p, hipStream_t st)
{
    using G = TilePick<WB, AB>;
    launch_tile<WB, AB, G::TM, G::TN, G::KV>(p, st);
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
    p.n_times_top = (uint32_t)(n * ((1 << w_bits) - 1) * ((1 << a_bits) - 1));
    p.acc = acc;
    p.scale = scale;
    p.out = out;
    p.vec = (p.nw % 4 == 0) ? 1 : 0;
    p.tiles_n = p.nblocks = 0;
    hipStream_t st = static_cast<hipStream_t>(stream);

    bool done = false;
    switch (w_bits) {
    case 1: done = dispatch_a<1>(a_bits, p, st); break;
    case 2: done = dispatch_a<2>(a_bits, p, st); break;
    case 3: done = dispatch_a<3>(a_bits, p, st); break;
    case 4: done = dispatch_a<4>(a_bits, p, st); break;
    default: break;
    }
    if (!done) {
        const int64_t total = rows * cols;
        if (ceil_div(total, 256) > 0x7fffffffLL)
            return fail(QNN_ERR_UNSUPPORTED, "qnn_binary_gemm: output too large for the wide-bit kernel");
        hipLaunchKernelGGL(bgemm_plain_kernel, dim3((unsigned)ceil_div(total, 256)), dim3(256), 0, st, p,
                           w_bits, a_bits);
    }
    return check_launch("qnn_binary_gemm");
}
