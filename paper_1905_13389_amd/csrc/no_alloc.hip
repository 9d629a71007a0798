// qnn_conv2d_chain_static: the layer-to-layer form of qnn_conv2d (planes in, the next layer's planes out) for
// callers that cannot allocate device memory and therefore have no acc / out buffer to lend: HIP graph capture,
// tight serving loops, harnesses that forbid hipMalloc.  Above 4 bits qnn_conv2d runs as chunk pairs of at most
// 4 x 4 planes and keeps the running int32 sum of the pairs in the caller's acc (or out) buffer; here that sum
// lives in a file-scope device array of fixed size instead.  Nothing is allocated, freed or retained per call.
#include <mutex>

#include "qnn_host.h"

namespace qnn {

// 8 Mi int32 accumulators = 32 MiB per GPU the library runs on, held until the process ends.
constexpr int64_t kStaticAccElems = int64_t(1) << 23;
static __device__ __align__(256) int32_t scratch[kStaticAccElems];

// The array's name is only a host-side handle; its device address differs per GPU and is looked up once per
// device (with that device current) and kept.
constexpr int kMaxDevices = 64;
static int32_t *g_scratch_ptr[kMaxDevices] = {nullptr};
static std::mutex g_scratch_mutex;

static int scratch_on_current_device(int32_t **ptr)
{
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return fail(QNN_ERR_LAUNCH, "qnn_conv2d_chain_static: hipGetDevice: %s", hipGetErrorString(e));
    if (dev < 0 || dev >= kMaxDevices)
        return fail(QNN_ERR_UNSUPPORTED, "qnn_conv2d_chain_static: device index %d beyond %d", dev, kMaxDevices - 1);
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !p)
            return fail(QNN_ERR_LAUNCH, "qnn_conv2d_chain_static: hipGetSymbolAddress: %s", hipGetErrorString(e));
        g_scratch_ptr[dev] = static_cast<int32_t *>(p);
    }
    *ptr = g_scratch_ptr[dev];
    return QNN_OK;
}

} // namespace qnn

using namespace qnn;

extern "C" int64_t qnn_conv2d_chain_static_max_outputs(void) { return kStaticAccElems; }

extern "C" int qnn_conv2d_chain_static(const qnn_conv_desc *d, const uint32_t *a_planes, const uint32_t *w_planes,
                                       const float *scale, uint32_t *next_planes, float next_clip, int next_bits,
                                       void *stream)
{
    if (!d) return fail(QNN_ERR_INVALID_ARG, "qnn_conv2d_chain_static: NULL descriptor");
    if (!next_planes) return fail(QNN_ERR_INVALID_ARG, "qnn_conv2d_chain_static: next_planes is the only output and is NULL");
    const bool wide = d->w_bits > 4 || d->a_bits > 4;
    if (!wide) // one launch, no running sum: the accumulators never leave the chip
        return qnn_conv2d(d, a_planes, w_planes, scale, nullptr, nullptr, next_planes, next_clip, next_bits, stream);
    // sizes first (host only), so that an oversized call is refused before any HIP call is made
    if (d->B < 0 || d->H <= 0 || d->W <= 0 || d->Cin <= 0 || d->Cout <= 0 || d->kh < 1 || d->kw < 1 || d->stride < 1 ||
        d->pad < 0 || d->H + 2 * (int64_t)d->pad < d->kh || d->W + 2 * (int64_t)d->pad < d->kw)
        return fail(QNN_ERR_INVALID_ARG, "qnn_conv2d_chain_static: bad geometry");
    if (d->a_bits < 1 || d->a_bits > 8 || d->w_bits < 1 || d->w_bits > 8 || next_bits < 1 || next_bits > 8)
        return fail(QNN_ERR_INVALID_ARG, "qnn_conv2d_chain_static: bits must be in [1,8]");
    if (!(next_clip > 0.0f && next_clip <= 3.0e38f))
        return fail(QNN_ERR_INVALID_ARG, "qnn_conv2d_chain_static: next_clip must be positive and finite");
    if (d->B == 0) return QNN_OK;
    if (!a_planes || !w_planes || !scale) return fail(QNN_ERR_INVALID_ARG, "qnn_conv2d_chain_static: NULL pointer");
    if (!aligned16(a_planes) || !aligned16(w_planes) || !aligned16(next_planes))
        return fail(QNN_ERR_ALIGNMENT, "qnn_conv2d_chain_static: pointers must be 16-byte aligned");
    if (!acc_fits_int32((int64_t)d->kh * d->kw * d->Cin, d->w_bits, d->a_bits))
        return fail(QNN_ERR_RANGE, "qnn_conv2d_chain_static: the reduction overflows int32 at these bit widths");
    const int64_t Ho = (d->H + 2 * (int64_t)d->pad - d->kh) / d->stride + 1;
    const int64_t Wo = (d->W + 2 * (int64_t)d->pad - d->kw) / d->stride + 1;
    if (d->Cout > kStaticAccElems || Ho * Wo > kStaticAccElems / d->Cout || d->B > kStaticAccElems / (Ho * Wo * d->Cout))
        return fail(QNN_ERR_RANGE,
                    "qnn_conv2d_chain_static: %lld x %lld x %lld x %lld outputs exceed the static accumulator buffer of "
                    "%lld int32 (use qnn_conv2d with an acc buffer of your own)",
                    (long long)d->B, (long long)Ho, (long long)Wo, (long long)d->Cout, (long long)kStaticAccElems);
    int32_t *acc = nullptr;
    const int rc = scratch_on_current_device(&acc);
    if (rc != QNN_OK) return rc;
    // the first chunk pair's launch overwrites the buffer, so it needs no clearing between calls
    return qnn_conv2d(d, a_planes, w_planes, scale, acc, nullptr, next_planes, next_clip, next_bits, stream);
}
