// C entry points of libqail: argument validation and dispatch.  Every check is
// done on the host before the first HIP call, so that the error paths can be
// exercised on a machine without a GPU.
#include <algorithm>
#include <atomic>

#include "qail_internal.h"

namespace qail {
int device_cu_count() {
    // read-only after the first call; two host threads racing here store the same value
    static std::atomic<int> cached{0};
    int cus = cached.load(std::memory_order_relaxed);
    if (cus == 0) {
        int dev = 0;
        hipDeviceProp_t prop;
        if (hipGetDevice(&dev) == hipSuccess && hipGetDeviceProperties(&prop, dev) == hipSuccess)
            cus = prop.multiProcessorCount;
        if (cus <= 0) cus = 256;
        cached.store(cus, std::memory_order_relaxed);
    }
    return cus;
}
}  // namespace qail

using namespace qail;

namespace {

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

int check_wdesc(const qail_wdesc* d) {
    if (!d) return QAIL_ERR_NULL;
    if (d->scheme != QAIL_W4_ASYM_GROUP && d->scheme != QAIL_W4_SYM_CHANNEL && d->scheme != QAIL_W8_SYM_CHANNEL &&
        d->scheme != QAIL_W8_SYM_GROUP)
        return QAIL_ERR_UNSUPPORTED;
    if (d->N < 1 || d->K < 8 || d->K % 8 != 0) return QAIL_ERR_SHAPE;
    if (d->scheme == QAIL_W4_ASYM_GROUP || d->scheme == QAIL_W8_SYM_GROUP) {
        if (d->group_size < 8 || d->group_size % 8 != 0 || d->K % d->group_size != 0) return QAIL_ERR_SHAPE;
        if (d->K / d->group_size > 32768) return QAIL_ERR_UNSUPPORTED;  // zero-points of a row are staged in LDS
    }
    return QAIL_OK;
}

int check_conv(const qail_conv_desc* d, int bits = 4) {
    if (!d) return QAIL_ERR_NULL;
    const int per_word = 32 / bits;
    if (d->B < 1 || d->H < 1 || d->W < 1 || d->Cin < per_word || d->Cin % per_word != 0 || d->Cout < 1 || d->KH < 1 ||
        d->KW < 1 || d->stride < 1 || d->pad < 0)
        return QAIL_ERR_SHAPE;
    // every product below in 64 bits: the fields are only known to be positive 32-bit values
    const long long ph = (long long)d->H + 2ll * d->pad, pw = (long long)d->W + 2ll * d->pad;
    if (ph < d->KH || pw < d->KW) return QAIL_ERR_SHAPE;
    // 4-bit: 16 * 8 * 15 * K must fit int32; 8-bit: 128 * 128 * K
    const long long kmax = bits == 4 ? 1118480 : 131071;
    const long long taps = (long long)d->KH * d->KW;   // < 2^62
    if (taps > kmax || taps * d->Cin > kmax) return QAIL_ERR_UNSUPPORTED;
    const long long OH = (ph - d->KH) / d->stride + 1, OW = (pw - d->KW) / d->stride + 1;   // each < 2^33
    if (OH * OW > 0x7FFFFFFFll) return QAIL_ERR_UNSUPPORTED;
    const long long M = (long long)d->B * (OH * OW);   // < 2^62
    if (M > 0x7FFFFFFFll / 2 || M / 64 + 1 > 65535) return QAIL_ERR_UNSUPPORTED;
    if ((long long)d->H * d->W > 0x7FFFFFFFll || (long long)d->B * ((long long)d->H * d->W) > 0x7FFFFFFFll)
        return QAIL_ERR_UNSUPPORTED;
    return QAIL_OK;
}

// The argument rules of qail_w4a4_conv_u4.
int check_conv_u4(const qail_conv_desc* d, const uint32_t* a_u4, const uint32_t* w_s4, const float* scale,
                         const float* bias, float s_out, const uint32_t* res_u4, float res_scale,
                         const float* res_f32, const uint32_t* out_u4) {
    const int e = check_conv(d);
    if (e != QAIL_OK) return e;
    if (d->Cout % 8 != 0) return QAIL_ERR_SHAPE;           // codes are packed 8 per word along Cout
    if (!(s_out > 0.f) || !(s_out <= 3.0e38f)) return QAIL_ERR_SHAPE;
    if (res_u4 && res_f32) return QAIL_ERR_SHAPE;          // at most one shortcut
    if (res_u4 && !(res_scale >= 0.f && res_scale <= 3.0e38f)) return QAIL_ERR_SHAPE;
    if (!a_u4 || !w_s4 || !scale || !bias || !out_u4) return QAIL_ERR_NULL;
    if (!aligned16(a_u4) || !aligned16(w_s4) || !aligned16(scale) || !aligned16(bias) || !aligned16(out_u4) ||
        (res_u4 && !aligned16(res_u4)) || (res_f32 && !aligned16(res_f32)))
        return QAIL_ERR_ALIGN;
    return QAIL_OK;
}

// The argument rules of qail_w4a4_gemm.
int check_conv_plain(const qail_conv_desc* d, const uint32_t* a_u4, const uint32_t* w_s4, const int32_t* acc_out,
                            const float* scale, const float* bias, const float* y_out) {
    const int e = check_conv(d);
    if (e != QAIL_OK) return e;
    if (!a_u4 || !w_s4) return QAIL_ERR_NULL;
    if (!acc_out && !y_out) return QAIL_ERR_NULL;
    if (y_out && (!scale || !bias)) return QAIL_ERR_NULL;
    if (!aligned16(a_u4) || !aligned16(w_s4) || (acc_out && !aligned16(acc_out)) ||
        (y_out && !aligned16(y_out)) || (scale && !aligned16(scale)) || (bias && !aligned16(bias)))
        return QAIL_ERR_ALIGN;
    return QAIL_OK;
}

int check_item(const qail_w4a16_item& it, int M) {
    int e = check_wdesc(&it.d);
    if (e != QAIL_OK) return e;
    if (it.d.scheme != QAIL_W4_ASYM_GROUP) return QAIL_ERR_UNSUPPORTED;
    if (!it.qweight || !it.scales || !it.zeros || !it.x || !it.y) return QAIL_ERR_NULL;
    if (!aligned16(it.qweight) || !aligned16(it.scales) || !aligned16(it.zeros) || !aligned16(it.x) ||
        !aligned16(it.y))
        return QAIL_ERR_ALIGN;
    if ((long long)M * it.d.N > 0x7FFFFFFFll || (long long)M * it.d.K > 0x7FFFFFFFll) return QAIL_ERR_UNSUPPORTED;
    return QAIL_OK;
}

inline int hip_status(hipError_t e) { return e == hipSuccess ? QAIL_OK : QAIL_ERR_HIP; }

}  // namespace

extern "C" {

int qail_version(void) { return 100; }

const char* qail_status_string(int status) {
    switch (status) {
        case QAIL_OK: return "ok";
        case QAIL_ERR_NULL: return "required pointer is NULL";
        case QAIL_ERR_SHAPE: return "bad shape";
        case QAIL_ERR_ALIGN: return "device pointer not 16-byte aligned";
        case QAIL_ERR_WORKSPACE: return "workspace missing or too small";
        case QAIL_ERR_UNSUPPORTED: return "unsupported request";
        case QAIL_ERR_HIP: return "HIP launch failed";
        default: return "unknown status";
    }
}

int qail_packed_sizes(const qail_wdesc* d, size_t* qweight_bytes, size_t* scales_bytes, size_t* zeros_bytes) {
    const int e = check_wdesc(d);
    if (e != QAIL_OK) return e;
    const size_t N = (size_t)d->N, K = (size_t)d->K;
    if (d->scheme == QAIL_W8_SYM_CHANNEL || d->scheme == QAIL_W8_SYM_GROUP) {
        if (qweight_bytes) *qweight_bytes = N * K;
        if (scales_bytes) *scales_bytes = d->scheme == QAIL_W8_SYM_GROUP ? N * (K / (size_t)d->group_size) * 2 : N * 4;
        if (zeros_bytes) *zeros_bytes = 0;
        return QAIL_OK;
    }
    if (qweight_bytes) *qweight_bytes = N * (K / 8) * 4;
    if (d->scheme == QAIL_W4_ASYM_GROUP) {
        const size_t G = K / (size_t)d->group_size;
        if (scales_bytes) *scales_bytes = N * G * 2;
        if (zeros_bytes) *zeros_bytes = N * ((G + 7) / 8) * 4;
    } else {
        if (scales_bytes) *scales_bytes = N * 4;
        if (zeros_bytes) *zeros_bytes = 0;
    }
    return QAIL_OK;
}

int qail_quantize_weights(const qail_wdesc* d, const float* w, uint32_t* qweight, void* scales,
                          uint32_t* zeros, uint32_t* range_errors, void* stream) {
    const int e = check_wdesc(d);
    if (e != QAIL_OK) return e;
    const bool asym = d->scheme == QAIL_W4_ASYM_GROUP;
    if (!w || !qweight || !scales || (asym && !zeros)) return QAIL_ERR_NULL;
    if (!aligned16(w) || !aligned16(qweight) || !aligned16(scales) || (asym && !aligned16(zeros)))
        return QAIL_ERR_ALIGN;
    if (range_errors && (reinterpret_cast<uintptr_t>(range_errors) & 3u)) return QAIL_ERR_ALIGN;
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (d->scheme == QAIL_W8_SYM_CHANNEL || d->scheme == QAIL_W8_SYM_GROUP)
        return hip_status(launch_quantize_s8(*d, w, qweight, scales, range_errors, st));
    if (asym)
        return hip_status(launch_quantize_asym(*d, w, qweight, static_cast<uint16_t*>(scales), zeros,
                                               range_errors, st));
    return hip_status(launch_quantize_sym(*d, w, qweight, static_cast<float*>(scales), st));
}

int qail_unpack_weights(const qail_wdesc* d, const uint32_t* qweight, uint8_t* codes, void* stream) {
    const int e = check_wdesc(d);
    if (e != QAIL_OK) return e;
    if (d->scheme == QAIL_W8_SYM_CHANNEL || d->scheme == QAIL_W8_SYM_GROUP)
        return QAIL_ERR_UNSUPPORTED;  // 8-bit codes are bytes already: qweight read as int8 [N][K]
    if (!qweight || !codes) return QAIL_ERR_NULL;
    if (!aligned16(qweight) || !aligned16(codes)) return QAIL_ERR_ALIGN;
    return hip_status(launch_unpack(*d, qweight, codes, static_cast<hipStream_t>(stream)));
}

int qail_act_scale_u4(const float* a, size_t n, float* s_a, void* stream) {
    if (!s_a || (n > 0 && !a)) return QAIL_ERR_NULL;
    if ((n > 0 && !aligned16(a)) || (reinterpret_cast<uintptr_t>(s_a) & 3u)) return QAIL_ERR_ALIGN;
    return hip_status(launch_act_scale(a, n, s_a, static_cast<hipStream_t>(stream)));
}

int qail_quantize_act_u4(const float* a, size_t n, const float* s_a, uint32_t* a_u4, void* stream) {
    if (n % 8 != 0) return QAIL_ERR_SHAPE;
    if (n / 8 > 0xFFFFFFFFull * 64) return QAIL_ERR_UNSUPPORTED;
    if (n == 0) return QAIL_OK;
    if (!a || !s_a || !a_u4) return QAIL_ERR_NULL;
    if (!aligned16(a) || !aligned16(a_u4) || (reinterpret_cast<uintptr_t>(s_a) & 3u)) return QAIL_ERR_ALIGN;
    return hip_status(launch_act_quant(a, n, s_a, a_u4, static_cast<hipStream_t>(stream)));
}

// Workspace one linear needs at batch M: only the matrix-core GEMM (M > 16) uses any.
static size_t item_workspace(const qail_wdesc& d, int M) {
    if (M == 1 || decode4_supports(d, M) || smallm_supports(d, M) || !gemm_f16_supports(d, M)) return 0;
    return gemm_f16_workspace(d, M);
}

// Whether item `it` of a batch at M goes to the matrix-core GEMM.
static bool takes_gemm(const qail_wdesc& d, int M) {
    return M > 1 && !decode4_supports(d, M) && !smallm_supports(d, M) && gemm_f16_supports(d, M);
}

// Workspace of a batch: consecutive linears of the matrix-core GEMM share launches and lie side
// by side in it; runs follow each other on the stream and reuse it.
static size_t batch_need(const qail_w4a16_item* items, int count, int M) {
    size_t need = 0;
    int i = 0;
    while (i < count) {
        int j = i;
        while (j < count && takes_gemm(items[j].d, M)) ++j;
        if (j > i) {
            need = std::max(need, gemm_f16_batch_workspace(items + i, j - i, M));
            i = j;
        } else {
            ++i;
        }
    }
    return need;
}

int qail_w4a16_workspace(const qail_wdesc* d, int32_t M, size_t* bytes) {
    const int e = check_wdesc(d);
    if (e != QAIL_OK) return e;
    if (d->scheme != QAIL_W4_ASYM_GROUP) return QAIL_ERR_UNSUPPORTED;
    if (M < 1) return QAIL_ERR_SHAPE;
    if (!bytes) return QAIL_ERR_NULL;
    *bytes = item_workspace(*d, M);
    return QAIL_OK;
}

int qail_w4a16_batch_workspace(const qail_w4a16_item* items, int32_t count, int32_t M, size_t* bytes) {
    if (count < 0 || M < 1) return QAIL_ERR_SHAPE;
    if (!bytes || (count > 0 && !items)) return QAIL_ERR_NULL;
    for (int i = 0; i < count; ++i) {
        const int e = check_wdesc(&items[i].d);
        if (e != QAIL_OK) return e;
        if (items[i].d.scheme != QAIL_W4_ASYM_GROUP) return QAIL_ERR_UNSUPPORTED;
    }
    *bytes = batch_need(items, count, M);
    return QAIL_OK;
}

int qail_w4a16_linear_batch(const qail_w4a16_item* items, int32_t count, int32_t M, void* workspace,
                            size_t workspace_bytes, void* stream) {
    if (count < 0 || M < 1) return QAIL_ERR_SHAPE;
    if (count == 0) return QAIL_OK;
    if (!items) return QAIL_ERR_NULL;
    for (int i = 0; i < count; ++i) {
        const int e = check_item(items[i], M);
        if (e != QAIL_OK) return e;
    }
    const size_t need = batch_need(items, count, M);
    if (need > 0) {
        if (!workspace || workspace_bytes < need) return QAIL_ERR_WORKSPACE;
        if (reinterpret_cast<uintptr_t>(workspace) & 255u) return QAIL_ERR_ALIGN;
    }
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (M == 1) {
        // runs of items the streaming kernel takes go out together
        int i = 0;
        while (i < count) {
            int j = i;
            while (j < count && gemv_supports(items[j].d)) ++j;
            if (j > i) {
                const hipError_t e = launch_w4a16_gemv(items + i, j - i, st);
                if (e != hipSuccess) return QAIL_ERR_HIP;
                i = j;
            } else {
                const hipError_t e = launch_w4a16_generic(items[i], 1, st);
                if (e != hipSuccess) return QAIL_ERR_HIP;
                ++i;
            }
        }
        return QAIL_OK;
    }
    int i = 0;
    while (i < count) {
        // runs of items one of the streaming kernels takes go out together
        int j = i;
        while (j < count && decode4_supports(items[j].d, M)) ++j;
        if (j > i) {
            if (launch_w4a16_decode4(items + i, j - i, M, st) != hipSuccess) return QAIL_ERR_HIP;
            i = j;
            continue;
        }
        while (j < count && smallm_supports(items[j].d, M) && !decode4_supports(items[j].d, M)) ++j;
        if (j > i) {
            if (launch_w4a16_smallm(items + i, j - i, M, st) != hipSuccess) return QAIL_ERR_HIP;
            i = j;
            continue;
        }
        while (j < count && takes_gemm(items[j].d, M)) ++j;
        if (j > i) {
            if (launch_w4a16_gemm_f16_batch(items + i, j - i, M, workspace, st) != hipSuccess) return QAIL_ERR_HIP;
            i = j;
            continue;
        }
        if (launch_w4a16_generic(items[i], M, st) != hipSuccess) return QAIL_ERR_HIP;
        ++i;
    }
    return QAIL_OK;
}

int qail_w4a16_chain_workspace(const qail_w4a16_item* items, int32_t count, size_t* bytes) {
    if (count < 0) return QAIL_ERR_SHAPE;
    if (!bytes || (count > 0 && !items)) return QAIL_ERR_NULL;
    for (int i = 0; i < count; ++i) {
        const int e = check_wdesc(&items[i].d);
        if (e != QAIL_OK) return e;
        if (items[i].d.scheme != QAIL_W4_ASYM_GROUP || !gemv_chain_supports(items[i].d)) return QAIL_ERR_UNSUPPORTED;
    }
    *bytes = gemv_chain_workspace(count);
    return QAIL_OK;
}

int qail_w4a16_linear_chain(const qail_w4a16_item* items, int32_t count, void* workspace, size_t workspace_bytes,
                            void* stream) {
    if (count < 0) return QAIL_ERR_SHAPE;
    if (count == 0) return QAIL_OK;
    if (!items) return QAIL_ERR_NULL;
    for (int i = 0; i < count; ++i) {
        const int e = check_item(items[i], 1);
        if (e != QAIL_OK) return e;
        if (!gemv_chain_supports(items[i].d)) return QAIL_ERR_UNSUPPORTED;
    }
    if (!workspace || workspace_bytes < gemv_chain_workspace(count)) return QAIL_ERR_WORKSPACE;
    if (reinterpret_cast<uintptr_t>(workspace) & 255u) return QAIL_ERR_ALIGN;
    return hip_status(launch_w4a16_chain(items, count, workspace, static_cast<hipStream_t>(stream)));
}

namespace {
constexpr int kLoraStride = 64;  // floats per row of a down-projection in the workspace (r <= 64)
constexpr int kLoraMaxM = 65535;  // the adapter kernels put the rows of x on the grid's y axis

int check_loras(const qail_w4a16_item* items, const qail_lora* loras, int count) {
    for (int i = 0; i < count; ++i) {
        const qail_lora& l = loras[i];
        if (l.r < 8 || l.r > kLoraStride || l.r % 8 != 0) return QAIL_ERR_SHAPE;
        if (!(l.scaling > -3.0e38f && l.scaling < 3.0e38f)) return QAIL_ERR_SHAPE;
        if (!l.A || !l.B) return QAIL_ERR_NULL;
        if (!aligned16(l.A) || !aligned16(l.B)) return QAIL_ERR_ALIGN;
        if (!lora_supports(items[i].d, l)) return QAIL_ERR_UNSUPPORTED;
    }
    return QAIL_OK;
}

size_t round256(size_t b) { return (b + 255) / 256 * 256; }
}  // namespace

int qail_w4a16_lora_workspace(const qail_w4a16_item* items, const qail_lora* loras, int32_t count, int32_t M,
                              size_t* bytes) {
    size_t base = 0;
    if (!bytes) return QAIL_ERR_NULL;
    const int e = qail_w4a16_batch_workspace(items, count, M, &base);
    if (e != QAIL_OK) return e;
    if (!bytes || (count > 0 && !loras)) return QAIL_ERR_NULL;
    if (M > kLoraMaxM) return QAIL_ERR_UNSUPPORTED;
    *bytes = round256(base) + round256((size_t)count * M * kLoraStride * sizeof(float));
    return QAIL_OK;
}

namespace {

// Validation shared by the two adapter entry points; *need_out = bytes of workspace the call uses.
int check_lora_call(const qail_w4a16_item* items, const qail_lora* loras, int32_t count, int32_t M,
                    size_t* base_out, size_t* need_out) {
    if (!items || !loras) return QAIL_ERR_NULL;
    if (M > kLoraMaxM) return QAIL_ERR_UNSUPPORTED;
    for (int i = 0; i < count; ++i) {
        const int e = check_item(items[i], M);
        if (e != QAIL_OK) return e;
    }
    const size_t base = batch_need(items, count, M);
    const int el = check_loras(items, loras, count);
    if (el != QAIL_OK) return el;
    *base_out = base;
    *need_out = round256(base) + round256((size_t)count * M * kLoraStride * sizeof(float));
    return QAIL_OK;
}

// The launches of the adapter path on a validated call; `workspace` holds at least the bytes
// check_lora_call reported, 256-byte aligned.
int run_lora_batch(const qail_w4a16_item* items, const qail_lora* loras, int32_t count, int32_t M,
                   void* workspace, size_t base, void* stream) {
    hipStream_t st = static_cast<hipStream_t>(stream);
    float* t = reinterpret_cast<float*>(static_cast<char*>(workspace) + round256(base));

    if (launch_lora_down(items, loras, t, kLoraStride, count, M, st) != hipSuccess) return QAIL_ERR_HIP;
    bool fused = (M == 1);
    for (int i = 0; fused && i < count; ++i) fused = gemv_supports(items[i].d);
    if (fused)
        return hip_status(launch_w4a16_gemv_lora(items, loras, t, kLoraStride, count, st));
    const int e = qail_w4a16_linear_batch(items, count, M, workspace, round256(base), stream);
    if (e != QAIL_OK) return e;
    for (int i = 0; i < count; ++i)
        if (launch_lora_up_add(items[i], loras[i], t + (size_t)i * M * kLoraStride, M, st) != hipSuccess)
            return QAIL_ERR_HIP;
    return QAIL_OK;
}

// Scratch of the entry point that takes no workspace: device memory that exists from the
// moment the library is loaded, one copy per GPU, so that nothing has to be allocated for it.
// The name is only a handle in host code; the address on the current device comes from
// hipGetSymbolAddress and is looked up once per device.
constexpr size_t kStaticScratchBytes = (size_t)1 << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];
constexpr int kMaxDevices = 64;
std::atomic<void*> scratch_ptr[kMaxDevices];

int static_scratch(void** out) {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return QAIL_ERR_HIP;
    if (dev < 0 || dev >= kMaxDevices) return QAIL_ERR_UNSUPPORTED;
    void* p = scratch_ptr[dev].load(std::memory_order_acquire);
    if (!p) {
        // two host threads may both get here: they read the same address
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return QAIL_ERR_HIP;
        scratch_ptr[dev].store(p, std::memory_order_release);
    }
    *out = p;
    return QAIL_OK;
}

}  // namespace

int qail_w4a16_linear_lora_batch(const qail_w4a16_item* items, const qail_lora* loras, int32_t count, int32_t M,
                                 void* workspace, size_t workspace_bytes, void* stream) {
    if (count < 0 || M < 1) return QAIL_ERR_SHAPE;
    if (count == 0) return QAIL_OK;
    size_t base = 0, need = 0;
    const int e = check_lora_call(items, loras, count, M, &base, &need);
    if (e != QAIL_OK) return e;
    if (!workspace || workspace_bytes < need) return QAIL_ERR_WORKSPACE;
    if (reinterpret_cast<uintptr_t>(workspace) & 255u) return QAIL_ERR_ALIGN;
    return run_lora_batch(items, loras, count, M, workspace, base, stream);
}

int qail_static_scratch_bytes(size_t* bytes) {
    if (!bytes) return QAIL_ERR_NULL;
    *bytes = kStaticScratchBytes;
    return QAIL_OK;
}

int qail_w4a16_linear_lora_batch_static(const qail_w4a16_item* items, const qail_lora* loras, int32_t count,
                                        int32_t M, void* stream) {
    if (count < 0 || M < 1) return QAIL_ERR_SHAPE;
    if (count == 0) return QAIL_OK;
    size_t base = 0, need = 0;
    const int e = check_lora_call(items, loras, count, M, &base, &need);
    if (e != QAIL_OK) return e;
    if (need > kStaticScratchBytes) return QAIL_ERR_WORKSPACE;   // beyond the built-in scratch: use the call above
    void* ws = nullptr;
    const int es = static_scratch(&ws);
    if (es != QAIL_OK) return es;
    return run_lora_batch(items, loras, count, M, ws, base, stream);
}

int qail_w4a16_linear(const qail_wdesc* d, const uint32_t* qweight, const uint16_t* scales,
                      const uint32_t* zeros, const uint16_t* x, uint16_t* y, int32_t M, void* workspace,
                      size_t workspace_bytes, void* stream) {
    if (!d) return QAIL_ERR_NULL;
    qail_w4a16_item it;
    it.d = *d;
    it.qweight = qweight;
    it.scales = scales;
    it.zeros = zeros;
    it.x = x;
    it.y = y;
    return qail_w4a16_linear_batch(&it, 1, M, workspace, workspace_bytes, stream);
}

int qail_w4a4_workspace(const qail_conv_desc* d, size_t* bytes) {
    const int e = check_conv(d);
    if (e != QAIL_OK) return e;
    if (!bytes) return QAIL_ERR_NULL;
    *bytes = 0;
    return QAIL_OK;
}

int qail_w4a4_gemm(const qail_conv_desc* d, const uint32_t* a_u4, const uint32_t* w_s4, int32_t* acc_out,
                   const float* scale, const float* bias, float* y_out, void* workspace,
                   size_t workspace_bytes, void* stream) {
    (void)workspace;
    (void)workspace_bytes;
    const int e = check_conv_plain(d, a_u4, w_s4, acc_out, scale, bias, y_out);
    if (e != QAIL_OK) return e;
    return hip_status(launch_w4a4_conv(*d, a_u4, w_s4, acc_out, scale, bias, y_out,
                                       static_cast<hipStream_t>(stream)));
}

int qail_w8a8_gemm(const qail_conv_desc* d, const uint32_t* a_s8, const uint32_t* w_s8, int32_t* acc_out,
                   const float* scale, const float* bias, float* y_out, void* workspace, size_t workspace_bytes,
                   void* stream) {
    (void)workspace;
    (void)workspace_bytes;
    const int e = check_conv(d, 8);
    if (e != QAIL_OK) return e;
    if (!a_s8 || !w_s8) return QAIL_ERR_NULL;
    if (!acc_out && !y_out) return QAIL_ERR_NULL;
    if (y_out && (!scale || !bias)) return QAIL_ERR_NULL;
    if (!aligned16(a_s8) || !aligned16(w_s8) || (acc_out && !aligned16(acc_out)) || (y_out && !aligned16(y_out)) ||
        (scale && !aligned16(scale)) || (bias && !aligned16(bias)))
        return QAIL_ERR_ALIGN;
    return hip_status(launch_w8a8_conv(*d, a_s8, w_s8, acc_out, scale, bias, y_out, static_cast<hipStream_t>(stream)));
}

int qail_act_scale_s8(const float* a, size_t n, float* s_a, void* stream) {
    if (!s_a || (n > 0 && !a)) return QAIL_ERR_NULL;
    if ((n > 0 && !aligned16(a)) || (reinterpret_cast<uintptr_t>(s_a) & 3u)) return QAIL_ERR_ALIGN;
    return hip_status(launch_act_scale_s8(a, n, s_a, static_cast<hipStream_t>(stream)));
}

int qail_quantize_act_s8(const float* a, size_t n, const float* s_a, uint32_t* a_s8, void* stream) {
    if (n % 4 != 0) return QAIL_ERR_SHAPE;
    if (n == 0) return QAIL_OK;
    if (!a || !s_a || !a_s8) return QAIL_ERR_NULL;
    if (!aligned16(a) || !aligned16(a_s8) || (reinterpret_cast<uintptr_t>(s_a) & 3u)) return QAIL_ERR_ALIGN;
    return hip_status(launch_act_quant_s8(a, n, s_a, a_s8, static_cast<hipStream_t>(stream)));
}

namespace {

// Whether an 8-bit weight-only linear at batch M goes to the matrix-core GEMM (M > 1 on the shapes
// it takes; M = 1 is the streaming kernel's, 2 <= M <= 16 at group size 128 the small-batch kernel's).
bool w8_takes_gemm(const qail_wdesc& d, int M) { return M > 1 && !smallm_w8_supports(d, M) && gemm_f16_supports(d, M); }

qail_w4a16_item as_gemm_item(const qail_w8a16_item& it) {
    qail_w4a16_item g;
    g.d = it.d;
    g.qweight = it.qweight;
    g.scales = it.scales;
    g.zeros = nullptr;
    g.x = it.x;
    g.y = it.y;
    return g;
}

int check_w8_item(const qail_w8a16_item& it, int M) {
    const int e = check_wdesc(&it.d);
    if (e != QAIL_OK) return e;
    if (it.d.scheme != QAIL_W8_SYM_GROUP) return QAIL_ERR_UNSUPPORTED;
    if ((long long)M * it.d.N > 0x7FFFFFFFll * 64) return QAIL_ERR_UNSUPPORTED;
    if (!it.qweight || !it.scales || !it.x || !it.y) return QAIL_ERR_NULL;
    if (!aligned16(it.qweight) || !aligned16(it.scales) || !aligned16(it.x) || !aligned16(it.y)) return QAIL_ERR_ALIGN;
    return QAIL_OK;
}

// Workspace of a batch: runs of consecutive items that go to the GEMM share launches, eight at a time.
size_t w8_batch_need(const qail_w8a16_item* items, int count, int M) {
    size_t need = 0;
    int i = 0;
    while (i < count) {
        int j = i;
        qail_w4a16_item run[8];
        while (j < count && j - i < 8 && w8_takes_gemm(items[j].d, M)) {
            run[j - i] = as_gemm_item(items[j]);
            ++j;
        }
        if (j > i) {
            need = std::max(need, gemm_f16_batch_workspace(run, j - i, M));
            i = j;
        } else {
            ++i;
        }
    }
    return need;
}

}  // namespace

int qail_w8a16_workspace(const qail_wdesc* d, int32_t M, size_t* bytes) {
    const int e = check_wdesc(d);
    if (e != QAIL_OK) return e;
    if (d->scheme != QAIL_W8_SYM_GROUP) return QAIL_ERR_UNSUPPORTED;
    if (M < 1) return QAIL_ERR_SHAPE;
    if (!bytes) return QAIL_ERR_NULL;
    *bytes = w8_takes_gemm(*d, M) ? gemm_f16_workspace(*d, M) : 0;
    return QAIL_OK;
}

int qail_w8a16_batch_workspace(const qail_w8a16_item* items, int32_t count, int32_t M, size_t* bytes) {
    if (count < 0 || M < 1) return QAIL_ERR_SHAPE;
    if (!bytes || (count > 0 && !items)) return QAIL_ERR_NULL;
    for (int i = 0; i < count; ++i) {
        const int e = check_wdesc(&items[i].d);
        if (e != QAIL_OK) return e;
        if (items[i].d.scheme != QAIL_W8_SYM_GROUP) return QAIL_ERR_UNSUPPORTED;
    }
    *bytes = w8_batch_need(items, count, M);
    return QAIL_OK;
}

int qail_w8a16_linear_batch(const qail_w8a16_item* items, int32_t count, int32_t M, void* workspace,
                            size_t workspace_bytes, void* stream) {
    if (count < 0 || M < 1) return QAIL_ERR_SHAPE;
    if (count == 0) return QAIL_OK;
    if (!items) return QAIL_ERR_NULL;
    for (int i = 0; i < count; ++i) {
        const int e = check_w8_item(items[i], M);
        if (e != QAIL_OK) return e;
    }
    const size_t need = w8_batch_need(items, count, M);
    if (need > 0) {
        if (!workspace || workspace_bytes < need) return QAIL_ERR_WORKSPACE;
        if (reinterpret_cast<uintptr_t>(workspace) & 255u) return QAIL_ERR_ALIGN;
    }
    hipStream_t st = static_cast<hipStream_t>(stream);
    int i = 0;
    while (i < count) {
        int j = i;
        while (j < count && w8a16_stream_supports(items[j].d, M)) ++j;
        if (j > i) {
            if (launch_w8a16_stream_batch(items + i, j - i, st) != hipSuccess) return QAIL_ERR_HIP;
            i = j;
            continue;
        }
        qail_w4a16_item run[8];
        while (j < count && j - i < 8 && smallm_w8_supports(items[j].d, M)) {
            run[j - i] = as_gemm_item(items[j]);
            ++j;
        }
        if (j > i) {
            if (launch_w8a16_smallm(run, j - i, M, st) != hipSuccess) return QAIL_ERR_HIP;
            i = j;
            continue;
        }
        while (j < count && j - i < 8 && w8_takes_gemm(items[j].d, M)) {
            run[j - i] = as_gemm_item(items[j]);
            ++j;
        }
        if (j > i) {
            if (launch_w4a16_gemm_f16_batch(run, j - i, M, workspace, st) != hipSuccess) return QAIL_ERR_HIP;
            i = j;
            continue;
        }
        const qail_w8a16_item& it = items[i];
        if (launch_w8a16_linear(it.d, it.qweight, it.scales, it.x, it.y, M, st) != hipSuccess) return QAIL_ERR_HIP;
        ++i;
    }
    return QAIL_OK;
}

int qail_w8a16_linear(const qail_wdesc* d, const uint32_t* qweight, const uint16_t* scales, const uint16_t* x,
                      uint16_t* y, int32_t M, void* workspace, size_t workspace_bytes, void* stream) {
    if (!d) return QAIL_ERR_NULL;
    qail_w8a16_item it;
    it.d = *d;
    it.qweight = qweight;
    it.scales = scales;
    it.x = x;
    it.y = y;
    return qail_w8a16_linear_batch(&it, 1, M, workspace, workspace_bytes, stream);
}

int qail_fake_quant_w4(const qail_wdesc* d, const float* w, float* w_hat, void* stream) {
    const int e = check_wdesc(d);
    if (e != QAIL_OK) return e;
    if (d->scheme != QAIL_W4_ASYM_GROUP) return QAIL_ERR_UNSUPPORTED;
    if (!w || !w_hat) return QAIL_ERR_NULL;
    if (!aligned16(w) || !aligned16(w_hat)) return QAIL_ERR_ALIGN;
    return hip_status(launch_fake_quant_w4(*d, w, w_hat, static_cast<hipStream_t>(stream)));
}

int qail_lsq_forward(const float* v, size_t n, const float* s, int32_t qn, int32_t qp, float* v_hat, void* stream) {
    if (qn > 0 || qp < 0 || qn < -32768 || qp > 32767) return QAIL_ERR_SHAPE;
    if (n == 0) return QAIL_OK;
    if (!v || !s || !v_hat) return QAIL_ERR_NULL;
    if (!aligned16(v) || !aligned16(v_hat) || (reinterpret_cast<uintptr_t>(s) & 3u)) return QAIL_ERR_ALIGN;
    return hip_status(launch_lsq_fwd(v, n, s, qn, qp, v_hat, static_cast<hipStream_t>(stream)));
}

int qail_lsq_backward_workspace(size_t* bytes) {
    if (!bytes) return QAIL_ERR_NULL;
    *bytes = lsq_bwd_workspace();
    return QAIL_OK;
}

int qail_lsq_backward(const float* v, const float* dout, size_t n, const float* s, int32_t qn, int32_t qp,
                      float grad_scale, float* dv, float* ds, void* workspace, size_t workspace_bytes, void* stream) {
    if (qn > 0 || qp < 0 || qn < -32768 || qp > 32767) return QAIL_ERR_SHAPE;
    if (!s || !ds || (n > 0 && (!v || !dout || !dv))) return QAIL_ERR_NULL;
    if ((n > 0 && (!aligned16(v) || !aligned16(dout) || !aligned16(dv))) || (reinterpret_cast<uintptr_t>(s) & 3u) ||
        (reinterpret_cast<uintptr_t>(ds) & 3u))
        return QAIL_ERR_ALIGN;
    if (!workspace || workspace_bytes < lsq_bwd_workspace()) return QAIL_ERR_WORKSPACE;
    if (!aligned16(workspace)) return QAIL_ERR_ALIGN;
    return hip_status(launch_lsq_bwd(v, dout, n, s, qn, qp, grad_scale, dv, ds, static_cast<float*>(workspace),
                                     static_cast<hipStream_t>(stream)));
}

int qail_qbc_loss(const float* logits_q, const float* logits_fp, int32_t B, int32_t D, float* loss, float* grad_q,
                  void* workspace, size_t workspace_bytes, void* stream) {
    if (B < 1 || D < 1 || B > 65535 * 16) return QAIL_ERR_SHAPE;
    if (!logits_q || !logits_fp || !loss) return QAIL_ERR_NULL;
    if (!aligned16(logits_q) || !aligned16(logits_fp) || (grad_q && !aligned16(grad_q)) ||
        (reinterpret_cast<uintptr_t>(loss) & 3u))
        return QAIL_ERR_ALIGN;
    if (!workspace || workspace_bytes < (size_t)B * sizeof(float)) return QAIL_ERR_WORKSPACE;
    if (!aligned16(workspace)) return QAIL_ERR_ALIGN;
    return hip_status(launch_qbc(logits_q, logits_fp, B, D, loss, grad_q, static_cast<float*>(workspace),
                                 static_cast<hipStream_t>(stream)));
}

int qail_w4a4_conv_u4(const qail_conv_desc* d, const uint32_t* a_u4, const uint32_t* w_s4, const float* scale,
                      const float* bias, float s_out, const uint32_t* res_u4, float res_scale,
                      const float* res_f32, uint32_t* out_u4, void* workspace, size_t workspace_bytes,
                      void* stream) {
    (void)workspace;
    (void)workspace_bytes;
    const int e = check_conv_u4(d, a_u4, w_s4, scale, bias, s_out, res_u4, res_scale, res_f32, out_u4);
    if (e != QAIL_OK) return e;
    return hip_status(launch_w4a4_conv_u4(*d, a_u4, w_s4, scale, bias, s_out, res_u4, res_scale, res_f32, out_u4,
                                          static_cast<hipStream_t>(stream)));
}

int qail_w4a4_conv_batch(const qail_conv_item* items, int32_t count, void* stream) {
    if (!items) return QAIL_ERR_NULL;
    if (count < 1 || count > 64) return QAIL_ERR_SHAPE;
    for (int i = 0; i < count; ++i) {
        const qail_conv_item& it = items[i];
        int e;
        if (it.out_u4) {
            if (it.acc_out || it.y_out) return QAIL_ERR_SHAPE;   // one kind of output per item
            e = check_conv_u4(&it.d, it.a_u4, it.w_s4, it.scale, it.bias, it.s_out, it.res_u4, it.res_scale,
                              it.res_f32, it.out_u4);
        } else {
            if (it.res_u4 || it.res_f32) return QAIL_ERR_SHAPE;  // a shortcut belongs to the fused output
            e = check_conv_plain(&it.d, it.a_u4, it.w_s4, it.acc_out, it.scale, it.bias, it.y_out);
        }
        if (e != QAIL_OK) return e;
    }
    return hip_status(launch_w4a4_conv_batch(items, count, static_cast<hipStream_t>(stream)));
}

}  // extern "C"
