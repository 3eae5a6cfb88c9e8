// Training-side operators (Sec. 3.2, Algorithm 1: the quantised policy is trained through its
// quantisers with the straight-through estimator; Sec. 3.3, Eq. 3: the QBC term, which the
// appendix instantiates as the mean L2 distance between the two policies' final logits).
// All are HBM-bound elementwise / reduction kernels.  Reductions are in a fixed order (per-block
// partial sums, then one block adds them): the results do not depend on scheduling.
#include "qail_internal.h"

namespace qail {

namespace {

constexpr int kRedBlocks = 1024;  // partial sums of the step gradient (workspace floats)

__device__ __forceinline__ float block_sum_256(float v, float* red) {
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) v += __shfl_xor(v, o, kWave);
    if (threadIdx.x % kWave == 0) red[threadIdx.x / kWave] = v;
    __syncthreads();
    const float r = (red[0] + red[1]) + (red[2] + red[3]);
    __syncthreads();
    return r;
}

// w_hat = (q - z) * s with (q, s, z) of the 4-bit group quantiser: one wave per (row, group).
__device__ __forceinline__ uint16_t f16_up(float v) {
    _Float16 h = (_Float16)v;
    uint16_t b = __builtin_bit_cast(uint16_t, h);
    if ((float)h < v) b += 1;
    return b;
}
__global__ __launch_bounds__(256) void fake_quant_w4_kernel(const float* __restrict__ w, float* __restrict__ out,
                                                            long long ngroups, int g) {
    const long long gi = (long long)blockIdx.x * 4 + threadIdx.x / kWave;
    if (gi >= ngroups) return;  // wave-uniform
    const int lane = threadIdx.x % kWave;
    const float4* src = reinterpret_cast<const float4*>(w + gi * g);
    float lo = 0.f, hi = 0.f;
    for (int i = lane; i < g / 4; i += kWave) {
        const float4 v = src[i];
        lo = fminf(fminf(lo, fminf(v.x, v.y)), fminf(v.z, v.w));
        hi = fmaxf(fmaxf(hi, fmaxf(v.x, v.y)), fmaxf(v.z, v.w));
    }
#pragma unroll
    for (int o = 1; o < kWave; o <<= 1) {
        lo = fminf(lo, __shfl_xor(lo, o, kWave));
        hi = fmaxf(hi, __shfl_xor(hi, o, kWave));
    }
    float s32 = (hi - lo) / 15.0f;
    if (s32 > 65504.0f) s32 = 65504.0f;
    uint16_t sb = f16_up(s32);
    if (sb < 0x0400) sb = 0x0400;
    if (hi == lo) sb = 0x3C00;
    const float s = f16_bits_to_f32(sb);
    const float z = fminf(fmaxf(rintf(-lo / s), 0.f), 15.f);
    float4* dst = reinterpret_cast<float4*>(out + gi * g);
    for (int i = lane; i < g / 4; i += kWave) {
        const float4 v = src[i];
        float4 r;
        r.x = (fminf(fmaxf(rintf(v.x / s) + z, 0.f), 15.f) - z) * s;
        r.y = (fminf(fmaxf(rintf(v.y / s) + z, 0.f), 15.f) - z) * s;
        r.z = (fminf(fmaxf(rintf(v.z / s) + z, 0.f), 15.f) - z) * s;
        r.w = (fminf(fmaxf(rintf(v.w / s) + z, 0.f), 15.f) - z) * s;
        dst[i] = r;
    }
}

__global__ __launch_bounds__(256) void lsq_fwd_kernel(const float* __restrict__ v, size_t n, const float* __restrict__ sp,
                                                      float qn, float qp, float* __restrict__ out) {
    const float s = *sp;
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256)
        out[i] = fminf(fmaxf(rintf(v[i] / s), qn), qp) * s;
}

__global__ __launch_bounds__(256) void lsq_bwd_kernel(const float* __restrict__ v, const float* __restrict__ dout, size_t n,
                                                      const float* __restrict__ sp, float qn, float qp,
                                                      float* __restrict__ dv, float* __restrict__ partial) {
    __shared__ float red[4];
    const float s = *sp;
    float acc = 0.f;
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256) {
        const float r = v[i] / s, d = dout[i];
        const bool inside = r >= qn && r <= qp;
        dv[i] = inside ? d : 0.f;
        const float t = inside ? rintf(r) - r : (r < qn ? qn : qp);
        acc = fmaf(d, t, acc);
    }
    const float tot = block_sum_256(acc, red);
    if (threadIdx.x == 0) partial[blockIdx.x] = tot;
}

__global__ __launch_bounds__(256) void sum_partials_kernel(const float* __restrict__ partial, int count, float mul,
                                                           float* __restrict__ out) {
    __shared__ float red[4];
    float acc = 0.f;
    for (int i = threadIdx.x; i < count; i += 256) acc += partial[i];
    const float tot = block_sum_256(acc, red);
    if (threadIdx.x == 0) *out = mul * tot;
}

// One block per batch row: distance, then (optionally) the row of the gradient.
__global__ __launch_bounds__(256) void qbc_rows_kernel(const float* __restrict__ lq, const float* __restrict__ lf, int D,
                                                       float inv_b, float* __restrict__ dist, float* __restrict__ grad) {
    __shared__ float red[4];
    const size_t base = (size_t)blockIdx.x * D;
    float acc = 0.f;
    for (int j = threadIdx.x; j < D; j += 256) {
        const float d = lq[base + j] - lf[base + j];
        acc = fmaf(d, d, acc);
    }
    const float nrm = sqrtf(block_sum_256(acc, red));
    if (threadIdx.x == 0) dist[blockIdx.x] = nrm;
    if (grad) {
        const float k = nrm > 0.f ? inv_b / nrm : 0.f;
        for (int j = threadIdx.x; j < D; j += 256) grad[base + j] = (lq[base + j] - lf[base + j]) * k;
    }
}

}  // namespace

hipError_t launch_fake_quant_w4(const qail_wdesc& d, const float* w, float* out, hipStream_t st) {
    const long long ngroups = (long long)d.N * (d.K / d.group_size);
    hipLaunchKernelGGL(fake_quant_w4_kernel, dim3((unsigned)((ngroups + 3) / 4)), dim3(256), 0, st, w, out, ngroups,
                       d.group_size);
    return hipGetLastError();
}

hipError_t launch_lsq_fwd(const float* v, size_t n, const float* s, int qn, int qp, float* out, hipStream_t st) {
    size_t blocks = (n + 255) / 256;
    if (blocks > 16384) blocks = 16384;
    hipLaunchKernelGGL(lsq_fwd_kernel, dim3((unsigned)blocks), dim3(256), 0, st, v, n, s, (float)qn, (float)qp, out);
    return hipGetLastError();
}

size_t lsq_bwd_workspace() { return kRedBlocks * sizeof(float); }

hipError_t launch_lsq_bwd(const float* v, const float* dout, size_t n, const float* s, int qn, int qp, float grad_scale,
                          float* dv, float* ds, float* ws, hipStream_t st) {
    size_t blocks = (n + 255) / 256;
    if (blocks > kRedBlocks) blocks = kRedBlocks;
    hipLaunchKernelGGL(lsq_bwd_kernel, dim3((unsigned)blocks), dim3(256), 0, st, v, dout, n, s, (float)qn, (float)qp, dv, ws);
    hipLaunchKernelGGL(sum_partials_kernel, dim3(1), dim3(256), 0, st, ws, (int)blocks, grad_scale, ds);
    return hipGetLastError();
}

hipError_t launch_qbc(const float* lq, const float* lf, int B, int D, float* loss, float* grad, float* ws, hipStream_t st) {
    hipLaunchKernelGGL(qbc_rows_kernel, dim3(B), dim3(256), 0, st, lq, lf, D, 1.0f / (float)B, ws, grad);
    hipLaunchKernelGGL(sum_partials_kernel, dim3(1), dim3(256), 0, st, ws, B, 1.0f / (float)B, loss);
    return hipGetLastError();
}

}  // namespace qail
