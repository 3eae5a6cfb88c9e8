// Internal declarations shared by the translation units of libqail.
// Nothing here crosses the C ABI; see include/qail.h for the public surface.
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "qail.h"

namespace qail {

typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_t;
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(4))) float f32x4_t;
typedef __attribute__((ext_vector_type(16))) float f32x16_t;
typedef __attribute__((ext_vector_type(4))) int i32x4_t;
typedef __attribute__((ext_vector_type(16))) int i32x16_t;

constexpr int kWave = 64;

// fp32 -> bf16 bit pattern, round to nearest even (finite inputs).
__device__ __forceinline__ uint16_t f32_to_bf16_rne(float f) {
    uint32_t u = __builtin_bit_cast(uint32_t, f);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

// Two fp32 -> packed bf16 pair (a in the low half), round to nearest even: one v_cvt_pk_bf16_f32.
__device__ __forceinline__ uint32_t f32x2_to_bf16x2_rne(float a, float b) {
    typedef __attribute__((ext_vector_type(2))) float f32x2_t;
    const f32x2_t v = {a, b};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_t));
}

__device__ __forceinline__ float bf16_bits_to_f32(uint16_t b) {
    return __builtin_bit_cast(float, (uint32_t)b << 16);
}

__device__ __forceinline__ float f16_bits_to_f32(uint16_t b) {
    return (float)__builtin_bit_cast(_Float16, b);
}

// Launchers (host side).  Each validates nothing: the C entry points do.
hipError_t launch_quantize_asym(const qail_wdesc& d, const float* w, uint32_t* qw, uint16_t* scales,
                                uint32_t* zeros, uint32_t* range_errors, hipStream_t st);
hipError_t launch_quantize_sym(const qail_wdesc& d, const float* w, uint32_t* qw, float* scales,
                               hipStream_t st);
hipError_t launch_unpack(const qail_wdesc& d, const uint32_t* qw, uint8_t* codes, hipStream_t st);
hipError_t launch_act_scale(const float* a, size_t n, float* s_a, hipStream_t st);
hipError_t launch_act_quant(const float* a, size_t n, const float* s_a, uint32_t* out, hipStream_t st);

// W4A16.  `items` lives in host memory; the launcher copies what it needs into
// kernel arguments.
bool gemv_supports(const qail_wdesc& d);
hipError_t launch_w4a16_gemv(const qail_w4a16_item* items, int count, hipStream_t st);
hipError_t launch_w4a16_gemv_lora(const qail_w4a16_item* items, const qail_lora* loras, const float* t,
                                  int t_stride, int count, hipStream_t st);
// Linears that depend on each other (M = 1, every item taken by the streaming kernel), in one
// launch per 32 items; `ws`: gemv_chain_workspace(count) bytes, 256-byte aligned.
bool gemv_chain_supports(const qail_wdesc& d);
size_t gemv_chain_workspace(int count);
hipError_t launch_w4a16_chain(const qail_w4a16_item* items, int count, void* ws, hipStream_t st);
bool lora_supports(const qail_wdesc& d, const qail_lora& l);
hipError_t launch_lora_down(const qail_w4a16_item* items, const qail_lora* loras, float* t, int t_stride,
                            int count, int M, hipStream_t st);
hipError_t launch_lora_up_add(const qail_w4a16_item& it, const qail_lora& l, const float* t, int M, hipStream_t st);
// 2 <= M <= 4: the M = 1 stream with four rows of x (preferred over the small-batch kernel).
bool decode4_supports(const qail_wdesc& d, int M);
hipError_t launch_w4a16_decode4(const qail_w4a16_item* items, int count, int M, hipStream_t st);
bool smallm_supports(const qail_wdesc& d, int M);
hipError_t launch_w4a16_smallm(const qail_w4a16_item* items, int count, int M, hipStream_t st);
// 8-bit weights at 2 <= M <= 16 on the same kernel (group size 128); items in the W4A16 record, zeros unused
bool smallm_w8_supports(const qail_wdesc& d, int M);
hipError_t launch_w8a16_smallm(const qail_w4a16_item* items, int count, int M, hipStream_t st);
// Compute units of the current device (256 when none can be asked); the launchers size their grids by it.
int device_cu_count();

// fp16-MFMA GEMM for M > 16; needs gemm_f16_workspace() bytes of 256-byte aligned device memory.
bool gemm_f16_supports(const qail_wdesc& d, int M);
size_t gemm_f16_workspace(const qail_wdesc& d, int M);
hipError_t launch_w4a16_gemm_f16(const qail_w4a16_item& it, int M, void* ws, hipStream_t st);
// Several such linears (all supported, same M) in shared launches, each on a share of the blocks;
// needs gemm_f16_batch_workspace() bytes.
size_t gemm_f16_batch_workspace(const qail_w4a16_item* items, int count, int M);
hipError_t launch_w4a16_gemm_f16_batch(const qail_w4a16_item* items, int count, int M, void* ws, hipStream_t st);
hipError_t launch_w4a16_generic(const qail_w4a16_item& it, int M, hipStream_t st);

// 8-bit variants.
hipError_t launch_quantize_s8(const qail_wdesc& d, const float* w, uint32_t* qw, void* scales,
                              uint32_t* range_errors, hipStream_t st);
hipError_t launch_act_scale_s8(const float* a, size_t n, float* s_a, hipStream_t st);
hipError_t launch_act_quant_s8(const float* a, size_t n, const float* s_a, uint32_t* out, hipStream_t st);
hipError_t launch_w8a16_linear(const qail_wdesc& d, const uint32_t* qw, const uint16_t* sc, const uint16_t* x,
                               uint16_t* y, int M, hipStream_t st);
// M = 1 on the shapes the streaming kernel takes (w8a16_gemv.hip); launch_w8a16_linear dispatches.
bool w8a16_stream_supports(const qail_wdesc& d, int M);
// `count` linears, all supported at M = 1, in shared launches
hipError_t launch_w8a16_stream_batch(const qail_w8a16_item* items, int count, hipStream_t st);
hipError_t launch_w8a16_stream(const qail_wdesc& d, const uint32_t* qw, const uint16_t* sc, const uint16_t* x,
                               uint16_t* y, hipStream_t st);

// Training-side operators.
hipError_t launch_fake_quant_w4(const qail_wdesc& d, const float* w, float* out, hipStream_t st);
hipError_t launch_lsq_fwd(const float* v, size_t n, const float* s, int qn, int qp, float* out, hipStream_t st);
size_t lsq_bwd_workspace();
hipError_t launch_lsq_bwd(const float* v, const float* dout, size_t n, const float* s, int qn, int qp, float grad_scale,
                          float* dv, float* ds, float* ws, hipStream_t st);
hipError_t launch_qbc(const float* lq, const float* lf, int B, int D, float* loss, float* grad, float* ws, hipStream_t st);

// W4A4.
hipError_t launch_w4a4_conv(const qail_conv_desc& d, const uint32_t* a, const uint32_t* w, int32_t* acc,
                            const float* scale, const float* bias, float* y, hipStream_t st);
hipError_t launch_w8a8_conv(const qail_conv_desc& d, const uint32_t* a, const uint32_t* w, int32_t* acc,
                            const float* scale, const float* bias, float* y, hipStream_t st);
hipError_t launch_w4a4_conv_batch(const qail_conv_item* items, int count, hipStream_t st);
hipError_t launch_w4a4_conv_u4(const qail_conv_desc& d, const uint32_t* a, const uint32_t* w, const float* scale,
                               const float* bias, float s_out, const uint32_t* res_u4, float res_scale,
                               const float* res_f32, uint32_t* out_u4, hipStream_t st);

}  // namespace qail
