// The unquantized ends of a network around the quantized trunk (the ResNet-18 workload keeps its first
// convolution and its classifier in full precision): a dense fp32 convolution whose epilogue can hand the
// next -- first quantized -- layer its bit planes, global average pooling, and a dense fp32 fully
// connected layer.  fp32 products and sums on the matrix cores (v_mfma_f32_32x32x2_f32); not part of the
// xor + bitcount path.
//
// dense_conv_kernel: implicit GEMM, rows = output pixels, columns = output channels, reduction axis
// k = (ky, kx, ci).  A workgroup of 4 waves owns 64 pixels x 64 channels, one 32 x 32 MFMA tile per wave.
// The reduction runs in chunks of up to kChunk values: the 64 pixel rows and the 64 weight rows of a chunk
// are staged in LDS with an odd row stride, so that the 32 rows a half-wave reads for one MFMA operand
// fall into 32 different banks; two workgroups fit a CU and cover each other's staging phases.  Workgroups
// are persistent: each walks the pixel tiles of one column tile.  A per-chunk table in LDS maps a reduction
// value to its byte offset from the window origin, so the gather is a batch of independent loads.  When the
// reduction fits one chunk (the 7 x 7 x 3 first convolution: 147 values) the table is built once and the
// weights live in registers instead of LDS (see the kernel's ONE parameter): three workgroups per CU.
#include <atomic>

#include "qnn_host.h"
#include "quantize.h"
#include "fastdiv.h"

namespace qnn {

typedef float v16f __attribute__((ext_vector_type(16)));

constexpr int kDenseThreads = 256;
constexpr int kDenseTile = 64;             // pixels and channels per workgroup
constexpr int kChunk = 152;                // reduction values per LDS stage (even)
constexpr int kChunkStride = kChunk + 1;   // odd: conflict-free operand reads
static_assert(kChunk % 8 == 0 && 2 * kDenseTile * kChunkStride * 4 + kChunk * 8 <= 80 * 1024, "two workgroups per CU");

// A zero in device memory: loads whose tap or weight does not exist read it instead of being skipped or masked
// afterwards, so that a batch of loads stays independent and no mask has to live until the data arrives.
static __device__ float dense_zero = 0.0f;

// Progress words of the resident workgroups: (tag << 32) | pixel tiles done.  The workgroups b, b + CUs, b + 2 CUs ...
// share a CU (the dispatcher fills every CU once per round) and a SIMD issues from its older waves first, so the one
// dispatched first would run ahead and the last would finish the kernel alone.  Each publishes its count after
// every tile and raises its wave priority while a partner is ahead of it.  A hint only: no result depends on it.
constexpr int kGroupSlots = 1024, kGroupMax = 4;
static __device__ unsigned long long group_progress[kGroupSlots];

struct DenseConvParams {
    const float *x, *w, *scale, *shift;
    float *out;
    uint32_t *next;
    int8_t *next_lv; // the same codes as int8 levels 2 u - top, [pixels][Cout] (the matrix-core route's layout)
    int H, W, Cin, Cout, kh, kw, stride, pad, Ho, Wo;
    int64_t M, tiles_m; // output pixels, pixel tiles
    int K;     // kh kw Cin
    int relu, next_bits, next_top, cwo;
    int fast_offsets; // the input tensor is smaller than 4 GiB: 32-bit byte offsets reach all of it (wrap-around sums too)
    int group, group_stride; // workgroups per CU that balance their progress (0: off) and the distance between their ids
    uint32_t group_tag;
    float next_inv_clip, next_half_top;
    FastDiv div_howo, div_wo;
};

// ONE: the reduction is one chunk.  Every lane then keeps its weight operands (its channel's values 2 u + lane / 32)
// in registers for all pixel tiles of the workgroup: no weight stage in LDS (three to four workgroups fit a CU
// instead of two) and no weight reads in the MFMA loop.
// KIND: which outputs exist, as bits 1 (fp32 out), 2 (planes), 4 (int8 levels), so that the epilogue carries only
// their code; -1 = decided at run time.
template <bool ONE, int KIND>
__global__ __launch_bounds__(kDenseThreads) __attribute__((amdgpu_waves_per_eu(3))) void dense_conv_kernel(DenseConvParams p)
{
    __shared__ float As[kDenseTile * kChunkStride];
    __shared__ float Ws[ONE ? 4 : kDenseTile * kChunkStride];
    __shared__ int2 taps[kChunk]; // per reduction value of the chunk: byte offset from the window origin, ky << 16 | kx
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int col0 = (int)blockIdx.y * kDenseTile;
    const int nchunks = (p.K + kChunk - 1) / kChunk;

    // staging: thread -> row tid / 4 of the tile (a pixel for A, a channel for W) and the reduction values
    // sub + 4 t of the chunk, t < kSlots: all of them are fetched and stored (the row has room for them);
    // those past the chunk hold 0 or are never read
    const int srow = tid >> 2, sub = tid & 3;
    constexpr int kSlots = kChunk / 4, kPart = 19, kParts = (kSlots + kPart - 1) / kPart; // values in flight per lane
    const bool ch_ok = col0 + srow < p.Cout;
    const float *wb = p.w + (int64_t)(ch_ok ? col0 + srow : 0) * p.K;

    auto stage_taps = [&](int k0, int kc) {
        for (int kk = tid; kk < kChunk; kk += kDenseThreads) {
            const int k = k0 + kk, tap = k / p.Cin, ci = k - tap * p.Cin, ky = tap / p.kw, kx = tap - ky * p.kw;
            taps[kk] = kk < kc ? make_int2(4 * ((ky * p.W + kx) * p.Cin + ci), (ky << 16) | kx) : make_int2(0, 0);
        }
    };
    auto stage_w = [&](int k0, int kc) {
#pragma unroll
        for (int h = 0; h < kParts; ++h) {
            float v[kPart];
#pragma unroll
            for (int t = 0; t < kPart; ++t) {
                if (h * kPart + t >= kSlots) continue; // the last part is shorter
                const int kk = sub + 4 * (h * kPart + t);
                const bool in_w = ch_ok && kk < kc;
                v[t] = *(in_w ? wb + k0 + kk : &dense_zero);
            }
#pragma unroll
            for (int t = 0; t < kPart; ++t)
                if (h * kPart + t < kSlots) Ws[srow * kChunkStride + sub + 4 * (h * kPart + t)] = v[t];
        }
    };

    // this lane's pixel of a tile: window origin and whether the whole window lies inside the image
    struct Pixel {
        bool ok, inside;
        int hi0, wi0;
        const char *origin;
    };
    auto locate = [&](int64_t tile) {
        Pixel q = {false, false, 0, 0, reinterpret_cast<const char *>(p.x)};
        const int64_t m = tile * kDenseTile + srow;
        if (m < p.M) {
            const uint32_t mm = (uint32_t)m;
            const uint32_t b = fdiv(mm, p.div_howo), rem = mm - b * p.div_howo.d;
            const uint32_t ho = fdiv(rem, p.div_wo), wo = rem - ho * p.div_wo.d;
            q.ok = true;
            q.hi0 = (int)ho * p.stride - p.pad, q.wi0 = (int)wo * p.stride - p.pad;
            q.origin = reinterpret_cast<const char *>(p.x + (((int64_t)b * p.H + q.hi0) * p.W + q.wi0) * p.Cin);
            q.inside = q.hi0 >= 0 && q.hi0 + p.kh <= p.H && q.wi0 >= 0 && q.wi0 + p.kw <= p.W;
        }
        return q;
    };
    // The chunk's values of this lane's pixel into registers.  A wave whose 16 pixels all have their whole
    // window inside the image (and whose tensor 32-bit byte offsets reach) gathers with one table read,
    // one add and one load per value; otherwise every tap is tested against the image, and the load goes
    // to the zero word when the test fails.
    // (In kParts parts of up to kPart values each: part h holds the slots t = h kPart ... .)
    auto gather = [&](const Pixel &q, int kc, int h, float (&v)[kPart]) {
        if (p.fast_offsets && __all(q.inside)) {
            const uint32_t origin = (uint32_t)(q.origin - reinterpret_cast<const char *>(p.x));
#pragma unroll
            for (int t = 0; t < kPart; ++t)
                if (h * kPart + t < kSlots)
                    v[t] = *reinterpret_cast<const float *>(reinterpret_cast<const char *>(p.x) +
                                                            (origin + (uint32_t)taps[sub + 4 * (h * kPart + t)].x));
        } else {
#pragma unroll
            for (int t = 0; t < kPart; ++t) {
                if (h * kPart + t >= kSlots) continue;
                const int kk = sub + 4 * (h * kPart + t);
                const int2 e = taps[kk];
                const int y = q.hi0 + (e.y >> 16), xx = q.wi0 + (e.y & 0xffff);
                const bool in_image = q.ok && kk < kc && (unsigned)y < (unsigned)p.H && (unsigned)xx < (unsigned)p.W;
                v[t] = *(in_image ? reinterpret_cast<const float *>(q.origin + e.x) : &dense_zero);
            }
        }
    };
    auto stash = [&](int h, const float (&v)[kPart]) {
#pragma unroll
        for (int t = 0; t < kPart; ++t)
            if (h * kPart + t < kSlots) As[srow * kChunkStride + sub + 4 * (h * kPart + t)] = v[t];
    };
    auto stage_pixels = [&](const Pixel &q, int kc) {
#pragma unroll
        for (int h = 0; h < kParts; ++h) {
            float v[kPart];
            gather(q, kc, h, v);
            stash(h, v);
        }
        // the fast gather leaves the window origin's value in the slots past the chunk; the MFMA loops read up
        // to the next multiple of 8: zeros there (slot kk belongs to the lane with sub = kk % 4, which wrote it)
        for (int kk = kc + ((sub - kc) & 3); kk < ((kc + 7) & ~7); kk += 4) As[srow * kChunkStride + kk] = 0.0f;
    };

    const int arow = 32 * (wave & 1) + (lane & 31), brow = 32 * (wave >> 1) + (lane & 31), khalf = lane >> 5;
    const float *ap = As + arow * kChunkStride + khalf, *bp = Ws + brow * kChunkStride + khalf;
    auto contract = [&](int kc2, v16f &acc) {
        // groups of kGroup MFMA steps: all operand reads of a group are issued before its first MFMA
        constexpr int kGroup = 16;
        int s = 0;
        for (; s + 2 * kGroup <= kc2; s += 2 * kGroup) {
            float a[kGroup], b[kGroup];
#pragma unroll
            for (int u = 0; u < kGroup; ++u) a[u] = ap[s + 2 * u], b[u] = bp[s + 2 * u];
#pragma unroll
            for (int u = 0; u < kGroup; ++u) acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a[u], b[u], acc, 0, 0, 0);
        }
        for (; s < kc2; s += 2) acc = __builtin_amdgcn_mfma_f32_32x32x2f32(ap[s], bp[s], acc, 0, 0, 0);
    };

    const int c = col0 + 32 * (wave >> 1) + (lane & 31);
    const bool c_ok = c < p.Cout;
    const float sc = p.scale && c_ok ? p.scale[c] : 1.0f, sh = p.shift && c_ok ? p.shift[c] : 0.0f;
    const int wword = (col0 >> 5) + (wave >> 1);
    // D layout of the 32 x 32 tile: this lane holds channel lane % 32 of the pixels 8 (r / 4) + 4 (lane / 32) + r % 4
    auto finish = [&](int64_t tile, const v16f &acc) {
        const int64_t row0 = tile * kDenseTile;
        // outputs that the instantiation rules out are compile-time null: their tests and stores disappear
        float *const o_out = KIND < 0 || (KIND & 1) ? p.out : nullptr;
        uint32_t *const o_next = KIND < 0 || (KIND & 2) ? p.next : nullptr;
        int8_t *const o_lv = KIND < 0 || (KIND & 4) ? p.next_lv : nullptr;
        int code[16];
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int64_t pix = row0 + 32 * (wave & 1) + 8 * (r >> 2) + 4 * khalf + (r & 3);
            const bool ok = pix < p.M && c_ok;
            float y = acc[r];
            if (p.scale) y = y * sc;
            if (p.shift) y = y + sh;
            if (p.relu) y = fmaxf(y, 0.0f);
            if (o_out && ok) o_out[pix * p.Cout + c] = y;
            code[r] = (o_next || o_lv) && ok ? quantize_code(y, p.next_inv_clip, p.next_half_top, p.next_top) : 0;
            if (o_lv && ok) o_lv[pix * p.Cout + c] = (int8_t)(2 * code[r] - p.next_top);
        }
        if (o_next) {
            // The 32 lanes of a half-wave hold the 32 channels of one plane word: one ballot per register
            // and bit gives the words of two pixels.  Lane L < 32 collects the word of the wave's pixel L,
            // so that a plane leaves with one store of 32 lanes instead of 16 stores of 2.
            const int64_t pix = row0 + 32 * (wave & 1) + lane;
            for (int j = 0; j < p.next_bits; ++j) {
                uint32_t mine = 0;
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const unsigned long long bits = __ballot((code[r] >> j) & 1);
                    const int slot = 8 * (r >> 2) + (r & 3); // pixel of the lower half-wave; the upper one's is 4 further
                    if (lane == slot) mine = (uint32_t)bits;
                    if (lane == slot + 4) mine = (uint32_t)(bits >> 32);
                }
                if (lane < 32 && pix < p.M && wword < p.cwo) o_next[((int64_t)j * p.M + pix) * p.cwo + wword] = mine;
            }
        }
    };

    unsigned tiles_done = 0;
    unsigned long long seen[kGroupMax] = {0, 0, 0, 0};
    if (p.group && tid == 0)
        __hip_atomic_store(&group_progress[blockIdx.x], (unsigned long long)p.group_tag << 32, __ATOMIC_RELAXED,
                           __HIP_MEMORY_SCOPE_AGENT);
    auto balance = [&]() {
        if (!p.group) return;
        ++tiles_done;
        bool behind = false;
#pragma unroll
        for (int g = 0; g < kGroupMax; ++g) {
            const unsigned tag = (unsigned)__builtin_amdgcn_readfirstlane((int)(seen[g] >> 32));
            const unsigned done = (unsigned)__builtin_amdgcn_readfirstlane((int)(unsigned)seen[g]);
            behind = behind || (g < p.group && tag == p.group_tag && done > tiles_done);
        }
        if (behind)
            __builtin_amdgcn_s_setprio(1);
        else
            __builtin_amdgcn_s_setprio(0);
        if (tid == 0)
            __hip_atomic_store(&group_progress[blockIdx.x], ((unsigned long long)p.group_tag << 32) | tiles_done,
                               __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        const unsigned first = blockIdx.x % (unsigned)p.group_stride;
#pragma unroll
        for (int g = 0; g < kGroupMax; ++g)
            if (g < p.group)
                seen[g] = __hip_atomic_load(&group_progress[first + g * p.group_stride], __ATOMIC_RELAXED,
                                            __HIP_MEMORY_SCOPE_AGENT);
    };

    if constexpr (ONE) {
        // One chunk (the 7 x 7 x 3 first convolution): the table is staged once, the weights go to registers.
        const int kc = p.K;
        stage_taps(0, kc);
        constexpr int kSteps = kChunk / 2, kGroup = 4; // MFMA steps of a full chunk; steps per uniform branch
        static_assert(kSteps % kGroup == 0 && 2 * kSteps <= kChunkStride, "groups of steps stay inside the stage row");
        float breg[kSteps];
        const float *wrow = p.w + (int64_t)(c_ok ? c : 0) * p.K;
#pragma unroll
        for (int u = 0; u < kSteps; ++u) {
            const bool in_w = c_ok && 2 * u + khalf < kc;
            breg[u] = *(in_w ? wrow + 2 * u + khalf : &dense_zero);
        }
        __syncthreads();
        for (int64_t tile = blockIdx.x; tile < p.tiles_m; tile += gridDim.x) {
            stage_pixels(locate(tile), kc);
            __syncthreads();
            v16f acc;
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[r] = 0.0f;
#pragma unroll
            for (int g = 0; g < kSteps / kGroup; ++g) {
                if (2 * kGroup * g < kc) { // same for all lanes; the stage holds zeros up to the next multiple of 8
                    float a[kGroup];
#pragma unroll
                    for (int u = 0; u < kGroup; ++u) a[u] = ap[2 * (kGroup * g + u)];
#pragma unroll
                    for (int u = 0; u < kGroup; ++u)
                        acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a[u], breg[kGroup * g + u], acc, 0, 0, 0);
                }
            }
            __syncthreads(); // every wave is done with the stage
            finish(tile, acc);
            balance();
        }
    } else {
        for (int64_t tile = blockIdx.x; tile < p.tiles_m; tile += gridDim.x) {
            const Pixel q = locate(tile);
            v16f acc;
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[r] = 0.0f;
            for (int ch = 0; ch < nchunks; ++ch) {
                const int k0 = ch * kChunk;
                const int kc = p.K - k0 < kChunk ? p.K - k0 : kChunk;
                stage_taps(k0, kc);
                stage_w(k0, kc);
                __syncthreads();
                stage_pixels(q, kc);
                __syncthreads();
                contract((kc + 1) & ~1, acc);
                __syncthreads(); // the stage may be overwritten
            }
            finish(tile, acc);
            balance();
        }
    }
}

// out[b][c] = (sum over the hw positions of x[b][.][c]) / hw, summed in position order; one lane per (b, c)
__global__ __launch_bounds__(256) void global_avgpool_kernel(const float *__restrict__ x, int64_t B, int64_t hw, int64_t C,
                                                             float inv_hw, float *__restrict__ out)
{
    const int64_t total = B * C, stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; idx < total; idx += stride) {
        const int64_t b = idx / C, c = idx % C;
        const float *src = x + b * hw * C + c;
        float s = 0.0f;
        for (int64_t i = 0; i < hw; ++i) s = s + src[i * C];
        out[idx] = s * inv_hw;
    }
}

static int dense_conv_run(const char *who, const qnn_dense_conv_desc *d, const float *x, const float *w, const float *scale,
                          const float *shift, int relu, float *out, uint32_t *next_planes, int8_t *next_levels,
                          float next_clip, int next_bits, void *stream)
{
    if (!d) return fail(QNN_ERR_INVALID_ARG, "%s: NULL descriptor", who);
    if (d->B < 0 || d->H <= 0 || d->W <= 0 || d->Cin <= 0 || d->Cout <= 0 || d->kh <= 0 || d->kw <= 0 || d->stride <= 0 ||
        d->pad < 0)
        return fail(QNN_ERR_INVALID_ARG, "%s: sizes must be positive (pad >= 0)", who);
    if (d->H + 2 * (int64_t)d->pad < d->kh || d->W + 2 * (int64_t)d->pad < d->kw)
        return fail(QNN_ERR_INVALID_ARG, "%s: kernel larger than the padded image", who);
    if (d->B == 0) return QNN_OK; // nothing to compute: the (empty) buffers may be NULL
    if (!out && !next_planes && !next_levels) return fail(QNN_ERR_INVALID_ARG, "%s: no output given", who);
    if ((next_planes || next_levels) && (next_bits < 1 || next_bits > 8 || !(next_clip > 0.0f) || next_clip > 3.0e38f))
        return fail(QNN_ERR_INVALID_ARG, "%s: next_bits in [1,8] and a finite next_clip > 0 are required with a quantized output", who);
    if (next_levels && next_bits > 7) return fail(QNN_ERR_UNSUPPORTED, "%s: int8 levels hold at most 7 bits", who);
    if (!x || !w) return fail(QNN_ERR_INVALID_ARG, "%s: NULL input pointer", who);
    if (!aligned16(x) || !aligned16(w) || !aligned16(out) || !aligned16(next_planes) || !aligned16(next_levels))
        return fail(QNN_ERR_ALIGNMENT, "%s: pointers must be 16-byte aligned", who);
    const int64_t Ho = (d->H + 2 * d->pad - d->kh) / d->stride + 1, Wo = (d->W + 2 * d->pad - d->kw) / d->stride + 1;
    // extents first, then their products: every product below stays far inside 64 bits
    if (d->H >= (1LL << 24) || d->W >= (1LL << 24) || d->Cin >= (1LL << 24) || d->Cout >= (1LL << 24) || d->kh > 4096 ||
        d->kw > 4096 || d->pad >= (1 << 24) || d->B >= (1LL << 31) || ceil_div(d->Cout, kDenseTile) > 65535)
        return fail(QNN_ERR_RANGE, "%s: tensor too large", who);
    const int64_t K = (int64_t)d->kh * d->kw * d->Cin;
    if (K >= (1LL << 24) || (int64_t)d->kh * d->W * d->Cin >= (1LL << 29) || Ho * Wo >= (1LL << 31) ||
        d->B > ((1LL << 31) - 1) / (Ho * Wo))
        return fail(QNN_ERR_RANGE, "%s: tensor too large", who);
    const int64_t M = d->B * Ho * Wo;
    DenseConvParams p;
    p.x = x, p.w = w, p.scale = scale, p.shift = shift, p.out = out, p.next = next_planes, p.next_lv = next_levels;
    p.H = (int)d->H, p.W = (int)d->W, p.Cin = (int)d->Cin, p.Cout = (int)d->Cout;
    p.kh = d->kh, p.kw = d->kw, p.stride = d->stride, p.pad = d->pad, p.Ho = (int)Ho, p.Wo = (int)Wo;
    p.M = M, p.K = (int)K, p.relu = relu ? 1 : 0;
    p.next_bits = next_planes || next_levels ? next_bits : 0;
    p.next_top = (1 << p.next_bits) - 1;
    p.cwo = (int)ceil_div(d->Cout, 32);
    p.next_inv_clip = next_planes || next_levels ? 1.0f / next_clip : 0.0f;
    p.next_half_top = 0.5f * (float)p.next_top;
    p.div_howo = make_fastdiv((uint32_t)(Ho * Wo)), p.div_wo = make_fastdiv((uint32_t)Wo);
    p.fast_offsets = d->B * d->H * d->W * d->Cin < (1LL << 30) ? 1 : 0;
    // persistent workgroups: as many as are resident at one time share the pixel tiles of their column tile round-robin
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus < 1)
        return fail(QNN_ERR_LAUNCH, "%s: device query failed", who);
    p.tiles_m = ceil_div(M, kDenseTile);
    const int64_t col_tiles = ceil_div(d->Cout, kDenseTile);
    const bool one = K <= kChunk;
    int per_cu = 0;
    const int kind = (out ? 1 : 0) | (next_planes ? 2 : 0) | (next_levels ? 4 : 0);
    void (*kernel)(DenseConvParams) = dense_conv_kernel<false, -1>;
    if (one) {
        switch (kind) {
        case 1: kernel = dense_conv_kernel<true, 1>; break;
        case 2: kernel = dense_conv_kernel<true, 2>; break;
        case 3: kernel = dense_conv_kernel<true, 3>; break;
        case 4: kernel = dense_conv_kernel<true, 4>; break;
        case 5: kernel = dense_conv_kernel<true, 5>; break;
        default: kernel = dense_conv_kernel<true, -1>; break;
        }
    }
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, kernel, kDenseThreads, 0) != hipSuccess || per_cu < 1)
        return fail(QNN_ERR_LAUNCH, "%s: occupancy query failed", who);
    int64_t per_col = ceil_div((int64_t)per_cu * cus, col_tiles);
    if (per_col > p.tiles_m) per_col = p.tiles_m;
    const dim3 grid((unsigned)per_col, (unsigned)col_tiles);
    // one column tile, every CU holds the same number (2 .. 4) of the resident workgroups: they balance their progress
    static std::atomic<uint32_t> launches{0};
    const bool grouped = col_tiles == 1 && per_cu >= 2 && per_cu <= kGroupMax && per_col == (int64_t)per_cu * cus &&
                         per_col <= kGroupSlots;
    p.group = grouped ? per_cu : 0, p.group_stride = cus, p.group_tag = ++launches;
    hipLaunchKernelGGL(kernel, grid, dim3(kDenseThreads), 0, static_cast<hipStream_t>(stream), p);
    return check_launch(who);
}

} // namespace qnn

using namespace qnn;

extern "C" int qnn_dense_conv2d_f32(const qnn_dense_conv_desc *d, const float *x, const float *w, const float *scale,
                                    const float *shift, int relu, float *out, uint32_t *next_planes, float next_clip,
                                    int next_bits, void *stream)
{
    return dense_conv_run("qnn_dense_conv2d_f32", d, x, w, scale, shift, relu, out, next_planes, nullptr, next_clip, next_bits, stream);
}

extern "C" int qnn_dense_conv2d_f32_levels(const qnn_dense_conv_desc *d, const float *x, const float *w, const float *scale,
                                           const float *shift, int relu, float *out, int8_t *next_levels, float next_clip,
                                           int next_bits, void *stream)
{
    return dense_conv_run("qnn_dense_conv2d_f32_levels", d, x, w, scale, shift, relu, out, nullptr, next_levels, next_clip,
                          next_bits, stream);
}

extern "C" int qnn_dense_fc_f32(const float *x, const float *w, const float *bias, int64_t rows, int64_t cols, int64_t n,
                                float *out, void *stream)
{
    if (rows < 0 || cols <= 0 || n <= 0) return fail(QNN_ERR_INVALID_ARG, "qnn_dense_fc_f32: rows >= 0, cols > 0, n > 0");
    if (!out) return fail(QNN_ERR_INVALID_ARG, "qnn_dense_fc_f32: NULL output");
    // a 1 x 1 convolution over 1 x 1 images: pixels = rows, channels = n -> cols
    const qnn_dense_conv_desc d = {rows, 1, 1, n, cols, 1, 1, 1, 0};
    return dense_conv_run("qnn_dense_fc_f32", &d, x, w, nullptr, bias, 0, out, nullptr, nullptr, 0.0f, 0, stream);
}

extern "C" int qnn_global_avgpool_f32(const float *x, int64_t B, int64_t hw, int64_t C, float *out, void *stream)
{
    if (B < 0 || hw <= 0 || C <= 0) return fail(QNN_ERR_INVALID_ARG, "qnn_global_avgpool_f32: B >= 0, hw > 0, C > 0");
    if (B == 0) return QNN_OK;
    if (!x || !out) return fail(QNN_ERR_INVALID_ARG, "qnn_global_avgpool_f32: NULL pointer");
    if (B > (INT64_MAX >> 8) / C / hw) return fail(QNN_ERR_RANGE, "qnn_global_avgpool_f32: tensor too large");
    const int64_t blocks = ceil_div(B * C, 256);
    const dim3 grid((unsigned)(blocks < 65536 ? blocks : 65536));
    hipLaunchKernelGGL(global_avgpool_kernel, grid, dim3(256), 0, static_cast<hipStream_t>(stream), x, B, hw, C,
                       1.0f / (float)hw, out);
    return check_launch("qnn_global_avgpool_f32");
}
