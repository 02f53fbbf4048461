// Host side of the C ABI declared in include/pb.h: argument checks, workspace
// carving and kernel dispatch.  No device memory is allocated or freed here and
// nothing synchronises; every kernel goes to the caller's stream.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "pb.h"
#include "pb_kernels.h"

namespace {

thread_local int g_last_hip_error = 0;

inline bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

int check_desc(const pb_desc *d, pb::Layout *L)
{
    if (!d) return PB_EINVAL;
    if (d->rows < 1 || d->cols < 1 || d->bits < 1 || d->bits > PB_MAX_BITS) return PB_EINVAL;
    if (d->frac_bits < 0 || d->frac_bits > 30) return PB_EINVAL;
    if (d->act_bits < 2 || d->act_bits > 32) return PB_EINVAL;
    if (d->layout != PB_LAYOUT_ROWMAJOR_V1 && !pb::is_tile16(d->layout)) return PB_EINVAL;
    if (d->layout == PB_LAYOUT_TILE16_GATES_V1 && d->rows % 4 != 0) return PB_EINVAL;
    if (d->cols > PB_MAX_COLS) return PB_ESIZE;
    if (!pb::make_layout(d->layout, d->rows, d->cols, d->bits, L)) return PB_ESIZE;
    if (pb::packed_bytes(*L) > 0xFFFFFFFFull) return PB_ESIZE;  // tiles are addressed with 32-bit byte offsets
    return PB_OK;
}

// Scratch memory of the entry point that allocates nothing (pb_matmul_static): the workspace of a pb_matmul call,
// held by the library in a static device array.  Every GPU the library runs on has its own copy; the array's name
// is a host-side stand-in, the device address comes from hipGetSymbolAddress, once per device.
constexpr size_t kScratchBytes = PB_STATIC_SCRATCH_BYTES;
constexpr int kMaxDevices = 64;
static __device__ __align__(256) unsigned char scratch[kScratchBytes];
void *g_scratch_ptr[kMaxDevices];   // device address of `scratch` on device i, null until its first use there

// Device address of `scratch` on the current device (looked up on first use, with that device current).
int scratch_address(void **out)
{
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return (int)e;
    if (dev < 0 || dev >= kMaxDevices) return (int)hipErrorInvalidDevice;
    void *p = __atomic_load_n(&g_scratch_ptr[dev], __ATOMIC_ACQUIRE);
    if (!p) {
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return (int)e;
        if (!p) return (int)hipErrorInvalidSymbol;
        __atomic_store_n(&g_scratch_ptr[dev], p, __ATOMIC_RELEASE);
    }
    *out = p;
    return 0;
}

int hip_status(int err)
{
    if (err == 0) return PB_OK;
    g_last_hip_error = err;
    return PB_EHIP;
}

}  // namespace

extern "C" {

int pb_desc_init_layout(pb_desc *d, int rows, int cols, int bits, uint32_t layout)
{
    if (!d) return PB_EINVAL;
    if (rows < 1 || cols < 1 || bits < 1 || bits > PB_MAX_BITS) return PB_EINVAL;
    if (cols > PB_MAX_COLS) return PB_ESIZE;
    d->rows = rows;
    d->cols = cols;
    d->bits = bits;
    d->frac_bits = 16;
    d->act_bits = 32;
    d->layout = layout;
    pb::Layout L;
    return check_desc(d, &L);
}

int pb_desc_init(pb_desc *d, int rows, int cols, int bits)
{
    return pb_desc_init_layout(d, rows, cols, bits, PB_LAYOUT_TILE16_V1);
}

size_t pb_packed_bytes(const pb_desc *d)
{
    pb::Layout L;
    if (check_desc(d, &L) != PB_OK) return 0;
    return pb::packed_bytes(L);
}

size_t pb_workspace_bytes(const pb_desc *d, int batch)
{
    pb::Layout L;
    if (check_desc(d, &L) != PB_OK || batch < 1 || batch > PB_MAX_BATCH) return 0;
    return pb::workspace_bytes(L, batch);
}

int pb_quantize_pack_mode(const float *W, const pb_desc *d, int quantizer, void *packed, float *scales, void *stream)
{
    pb::Layout L;
    int rc = check_desc(d, &L);
    if (rc != PB_OK) return rc;
    if (!W || !packed || !scales) return PB_EINVAL;
    if (quantizer < PB_QUANT_SYMMETRIC || quantizer > PB_QUANT_CLIP_SEARCH) return PB_EINVAL;
    if (quantizer == PB_QUANT_SIGN && d->bits != 2) return PB_EINVAL;
    if (!aligned16(W) || !aligned16(packed) || !aligned16(scales)) return PB_EALIGN;
    return hip_status(pb::launch_quantize_pack(W, L, quantizer, static_cast<uint32_t *>(packed), scales,
                                               static_cast<hipStream_t>(stream)));
}

int pb_quantize_pack_desc(const float *W, const pb_desc *d, void *packed, float *scales, void *stream)
{
    return pb_quantize_pack_mode(W, d, PB_QUANT_SYMMETRIC, packed, scales, stream);
}

int pb_quantize_pack(const float *W, int rows, int cols, int bits, void *packed, float *scales, void *stream)
{
    pb_desc d;
    int rc = pb_desc_init(&d, rows, cols, bits);
    if (rc != PB_OK) return rc;
    return pb_quantize_pack_desc(W, &d, packed, scales, stream);
}

int pb_unpack(const void *packed, const pb_desc *d, int32_t *q, void *stream)
{
    pb::Layout L;
    int rc = check_desc(d, &L);
    if (rc != PB_OK) return rc;
    if (!packed || !q) return PB_EINVAL;
    if (!aligned16(packed) || !aligned16(q)) return PB_EALIGN;
    return hip_status(pb::launch_unpack(static_cast<const uint32_t *>(packed), L, q, static_cast<hipStream_t>(stream)));
}

static int matmul_common(const void *packed, const float *scales, const pb_desc *d, int bits_used, const float *X0,
                         int cols0, const float *X1, int cols1, int batch, float *Y, int64_t *A, void *workspace,
                         void *stream, const pb::Epilogue &ep = pb::Epilogue(), bool pairs_out = false)
{
    pb::Layout L;
    int rc = check_desc(d, &L);
    if (rc != PB_OK) return rc;
    if (!packed || !X0 || !workspace || (!Y && !A) || (Y && !scales)) return PB_EINVAL;
    if (bits_used < 1 || bits_used > d->bits) return PB_EINVAL;
    if (batch < 1) return PB_EINVAL;
    if (batch > PB_MAX_BATCH) return PB_ESIZE;
    if (!aligned16(packed) || !aligned16(X0) || !aligned16(workspace) || (Y && !aligned16(Y)) ||
        (A && !aligned16(A)) || (scales && !aligned16(scales)) || (X1 && !aligned16(X1)))
        return PB_EALIGN;
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (ep.bias && !aligned16(ep.bias)) return PB_EALIGN;
    if (pairs_out && L.cols > pb::kMaxColsPairs) return PB_ESIZE;
    if (pb::is_tile16(L.layout))   // conversion, bit transpose, product and epilogue in one launch
        return hip_status(pb::launch_mfma(static_cast<const uint32_t *>(packed), scales, L, bits_used, d->frac_bits,
                                          d->act_bits, X0, cols0, X1, cols1, nullptr, batch, Y,
                                          reinterpret_cast<long long *>(A), pairs_out, ep, st));
    if (pairs_out) return PB_EINVAL;   // only the tiled layouts multiply bitlayer pairs
    char *ws = static_cast<char *>(workspace);
    int *meta = reinterpret_cast<int *>(ws + pb::ws_meta_off(L, batch));
    uint32_t *planes = reinterpret_cast<uint32_t *>(ws + pb::ws_planes_off(L, batch));
    int err = pb::launch_prep(X0, cols0, X1, cols1, batch, L, d->frac_bits, d->act_bits, planes, meta, nullptr, st);
    if (err) return hip_status(err);
    err = pb::launch_matvec(static_cast<const uint32_t *>(packed), scales, L, bits_used, d->frac_bits, planes, meta,
                            batch, Y, reinterpret_cast<long long *>(A), st);
    if (!err && Y && (ep.bias || ep.relu)) err = pb::launch_bias_act(Y, ep.bias, ep.relu, L.rows, batch, st);
    return hip_status(err);
}

int pb_matmul(const void *packed, const float *scales, const pb_desc *d, int bits_used, const float *X, int batch,
              float *Y, void *workspace, void *stream)
{
    if (!Y || !d) return PB_EINVAL;
    return matmul_common(packed, scales, d, bits_used, X, d->cols, nullptr, 0, batch, Y, nullptr, workspace, stream);
}

int pb_matmul_static(const void *packed, const float *scales, const pb_desc *d, int bits_used, const float *X, int batch,
                     float *Y, void *stream)
{
    if (!Y || !d) return PB_EINVAL;
    pb::Layout L;
    int rc = check_desc(d, &L);
    if (rc != PB_OK) return rc;
    if (batch < 1) return PB_EINVAL;
    if (batch > PB_MAX_BATCH || pb::workspace_bytes(L, batch) > kScratchBytes) return PB_ESIZE;
    void *ws = nullptr;
    rc = scratch_address(&ws);
    if (rc) return hip_status(rc);
    // (nothing in the scratch has to start at zero: the activation kernel writes every word the product kernel reads)
    return matmul_common(packed, scales, d, bits_used, X, d->cols, nullptr, 0, batch, Y, nullptr, ws, stream);
}

int pb_matmul_bias_act(const void *packed, const float *scales, const pb_desc *d, int bits_used, const float *X,
                       int batch, const float *bias, int act, float *Y, void *workspace, void *stream)
{
    if (!Y || !d) return PB_EINVAL;
    if (act != PB_ACT_NONE && act != PB_ACT_RELU) return PB_EINVAL;
    pb::Epilogue ep;
    ep.bias = bias;
    ep.relu = act == PB_ACT_RELU;
    return matmul_common(packed, scales, d, bits_used, X, d->cols, nullptr, 0, batch, Y, nullptr, workspace, stream,
                         ep);
}

int pb_matmul_acc(const void *packed, const pb_desc *d, int bits_used, const float *X, int batch, int64_t *A,
                  void *workspace, void *stream)
{
    if (!A || !d) return PB_EINVAL;
    return matmul_common(packed, nullptr, d, bits_used, X, d->cols, nullptr, 0, batch, nullptr, A, workspace, stream);
}

int pb_matmul_acc_pairs(const void *packed, const pb_desc *d, int bits_used, const float *X, int batch, int64_t *A,
                        void *workspace, void *stream)
{
    if (!A || !d) return PB_EINVAL;
    return matmul_common(packed, nullptr, d, bits_used, X, d->cols, nullptr, 0, batch, nullptr, A, workspace, stream,
                         pb::Epilogue(), true);
}

int pb_act_prep(const pb_desc *d, const float *X, int batch, void *workspace, void *stream)
{
    pb::Layout L;
    int rc = check_desc(d, &L);
    if (rc != PB_OK) return rc;
    if (!X || !workspace) return PB_EINVAL;
    if (batch < 1) return PB_EINVAL;
    if (batch > PB_MAX_BATCH) return PB_ESIZE;
    if (!aligned16(X) || !aligned16(workspace)) return PB_EALIGN;
    char *ws = static_cast<char *>(workspace);
    int *meta = reinterpret_cast<int *>(ws + pb::ws_meta_off(L, batch));
    uint32_t *planes = reinterpret_cast<uint32_t *>(ws + pb::ws_planes_off(L, batch));
    return hip_status(pb::launch_prep(X, d->cols, nullptr, 0, batch, L, d->frac_bits, d->act_bits, planes, meta,
                                      nullptr, static_cast<hipStream_t>(stream)));
}

int pb_matmul_prepared(const void *packed, const float *scales, const pb_desc *d, int bits_used, int batch, float *Y,
                       void *workspace, void *stream)
{
    pb::Layout L;
    int rc = check_desc(d, &L);
    if (rc != PB_OK) return rc;
    if (!packed || !scales || !Y || !workspace) return PB_EINVAL;
    if (bits_used < 1 || bits_used > d->bits) return PB_EINVAL;
    if (batch < 1) return PB_EINVAL;
    if (batch > PB_MAX_BATCH) return PB_ESIZE;
    if (!aligned16(packed) || !aligned16(scales) || !aligned16(Y) || !aligned16(workspace)) return PB_EALIGN;
    char *ws = static_cast<char *>(workspace);
    const int *meta = reinterpret_cast<const int *>(ws + pb::ws_meta_off(L, batch));
    const uint32_t *planes = reinterpret_cast<const uint32_t *>(ws + pb::ws_planes_off(L, batch));
    if (pb::is_tile16(L.layout))
        return hip_status(pb::launch_mfma(static_cast<const uint32_t *>(packed), scales, L, bits_used, d->frac_bits,
                                          d->act_bits, nullptr, 0, nullptr, 0, planes, batch, Y, nullptr, false,
                                          pb::Epilogue(), static_cast<hipStream_t>(stream)));
    return hip_status(pb::launch_matvec(static_cast<const uint32_t *>(packed), scales, L, bits_used, d->frac_bits,
                                        planes, meta, batch, Y, nullptr, static_cast<hipStream_t>(stream)));
}

int pb_fixed_point(const pb_desc *d, const float *X, int batch, int32_t *xq, void *workspace, void *stream)
{
    pb::Layout L;
    int rc = check_desc(d, &L);
    if (rc != PB_OK) return rc;
    if (!X || !xq || !workspace) return PB_EINVAL;
    if (batch < 1) return PB_EINVAL;
    if (batch > PB_MAX_BATCH) return PB_ESIZE;
    if (!aligned16(X) || !aligned16(xq) || !aligned16(workspace)) return PB_EALIGN;
    char *ws = static_cast<char *>(workspace);
    int *meta = reinterpret_cast<int *>(ws + pb::ws_meta_off(L, batch));
    uint32_t *planes = reinterpret_cast<uint32_t *>(ws + pb::ws_planes_off(L, batch));
    return hip_status(pb::launch_prep(X, d->cols, nullptr, 0, batch, L, d->frac_bits, d->act_bits, planes, meta, xq,
                                      static_cast<hipStream_t>(stream)));
}

int pb_lstm_cell(const void *packed, const float *scales, const pb_desc *d, int bits_used, const float *x_t,
                 int input_size, const float *h_prev, const float *c_prev, const float *bias, float *h_out,
                 float *c_out, int batch, void *workspace, void *stream)
{
    pb::Layout L;
    int rc = check_desc(d, &L);
    if (rc != PB_OK) return rc;
    if (!x_t || !h_prev || !c_prev || !h_out || !c_out || !workspace) return PB_EINVAL;
    if (d->rows % 4 != 0 || input_size < 1 || input_size >= d->cols) return PB_EINVAL;
    const int H = d->rows / 4;
    if (d->cols != input_size + H) return PB_EINVAL;
    if (batch < 1) return PB_EINVAL;
    if (batch > PB_MAX_BATCH) return PB_ESIZE;
    if (!aligned16(h_prev) || !aligned16(c_prev) || !aligned16(h_out) || !aligned16(c_out) ||
        (bias && !aligned16(bias)))
        return PB_EALIGN;
    if (L.layout == PB_LAYOUT_TILE16_GATES_V1) {
        // one launch, unless the new hidden state would overwrite the old one while other workgroups still read it
        const size_t hbytes = (size_t)batch * (size_t)H * sizeof(float);
        const char *ho = reinterpret_cast<const char *>(h_out), *hp = reinterpret_cast<const char *>(h_prev);
        const char *xp = reinterpret_cast<const char *>(x_t);
        const size_t xbytes = (size_t)batch * (size_t)input_size * sizeof(float);
        const bool overlap = (ho < hp + hbytes && hp < ho + hbytes) || (ho < xp + xbytes && xp < ho + hbytes);
        if (!overlap) {
            pb::Epilogue ep;
            ep.bias = bias;
            ep.c_prev = c_prev;
            ep.h_out = h_out;
            ep.c_out = c_out;
            // (Y is not written in this mode; matmul_common wants a non-null output)
            return matmul_common(packed, scales, d, bits_used, x_t, input_size, h_prev, H, batch, h_out, nullptr,
                                 workspace, stream, ep);
        }
    }
    float *gates = reinterpret_cast<float *>(static_cast<char *>(workspace) + pb::ws_gates_off(L, batch));
    rc = matmul_common(packed, scales, d, bits_used, x_t, input_size, h_prev, H, batch, gates, nullptr, workspace,
                       stream);
    if (rc != PB_OK) return rc;
    return hip_status(pb::launch_lstm_pointwise(gates, bias, c_prev, H, batch, h_out, c_out,
                                                static_cast<hipStream_t>(stream)));
}

const char *pb_strerror(int status)
{
    switch (status) {
        case PB_OK: return "ok";
        case PB_EINVAL: return "invalid argument (null pointer, non-positive size, bits/bits_used/batch out of range)";
        case PB_EALIGN: return "device pointer not 16-byte aligned";
        case PB_ESIZE: return "shape beyond the supported maximum";
        case PB_EHIP: return "HIP call failed (see pb_last_hip_error)";
        default: return "unknown status";
    }
}

int pb_last_hip_error(void) { return g_last_hip_error; }

}  // extern "C"
