// Low-rank adapter beside the 4-bit linear (Sec. 5.1: the 4-bit policy is fine-tuned with
// rank-32 adapters on the quantised backbone, which then run next to the packed weights):
//   y[m][n] = sum_k x[m][k] w_hat[n][k] + scaling * sum_j t[m][j] B[n][j],   t[m][j] = sum_k x[m][k] A[j][k].
// Two small kernels: the down-projection t = x A^T (fp32, before the linear) and, for the
// batch sizes whose linear kernel does not take the adapter into its own epilogue, the
// up-projection added to the bf16 output afterwards.  Both are bandwidth-trivial next to the
// 4-bit stream (r (K + N) bf16 per linear).
#include "qail_internal.h"

namespace qail {

namespace {

constexpr int kMaxLoraItems = 16;

struct DownItem {
    const uint16_t* x;   // bf16 [M][K]
    const uint16_t* A;   // bf16 [r][K]
    float* t;            // fp32 [M][r]
    int K, r;
};
struct DownArgs {
    DownItem it[kMaxLoraItems];
    int M;
};

// One block per (j, m, item): its 1024 threads split K, 8 elements a piece.  A thread's first two
// pieces (all of K up to 16384) are requested before either is used: one round trip to memory
// instead of one per piece, which is what this kernel's time consists of.
constexpr int kDownThreads = 1024;
__device__ __forceinline__ float dot8(const uint4& xv, const uint4& av, float acc) {
    const uint32_t xw[4] = {xv.x, xv.y, xv.z, xv.w}, aw[4] = {av.x, av.y, av.z, av.w};
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        acc = fmaf(__builtin_bit_cast(float, xw[e] << 16), __builtin_bit_cast(float, aw[e] << 16), acc);
        acc = fmaf(__builtin_bit_cast(float, xw[e] & 0xFFFF0000u), __builtin_bit_cast(float, aw[e] & 0xFFFF0000u), acc);
    }
    return acc;
}
__global__ __launch_bounds__(kDownThreads) void lora_down_kernel(const DownArgs args) {
    __shared__ float red[kDownThreads / kWave];
    const DownItem& it = args.it[blockIdx.z];
    const int j = blockIdx.x, m = blockIdx.y;
    if (j >= it.r) return;  // block-uniform (items of a launch may differ in rank)
    const uint4* xr = reinterpret_cast<const uint4*>(it.x + (size_t)m * it.K);
    const uint4* ar = reinterpret_cast<const uint4*>(it.A + (size_t)j * it.K);
    const int n8 = it.K / 8;
    uint4 xv[2], av[2];
#pragma unroll
    for (int u = 0; u < 2; ++u) {   // every load is issued; a piece past the end re-reads piece 0 and is not used
        const int i = (int)threadIdx.x + u * kDownThreads;
        xv[u] = xr[i < n8 ? i : 0];
        av[u] = ar[i < n8 ? i : 0];
    }
    float acc = 0.f;
#pragma unroll
    for (int u = 0; u < 2; ++u)
        if ((int)threadIdx.x + u * kDownThreads < n8) acc = dot8(xv[u], av[u], acc);
    for (int i = (int)threadIdx.x + 2 * kDownThreads; i < n8; i += kDownThreads) acc = dot8(xr[i], ar[i], acc);
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) acc += __shfl_xor(acc, o);
    if (threadIdx.x % kWave == 0) red[threadIdx.x / kWave] = acc;
    __syncthreads();
    if (threadIdx.x == 0) {
        float sum = 0.f;
#pragma unroll
        for (int w = 0; w < kDownThreads / kWave; ++w) sum += red[w];   // in the order of the waves: deterministic
        it.t[(size_t)m * it.r + j] = sum;
    }
}

// y[m][n] = bf16(float(y[m][n]) + scaling * sum_j t[m][j] B[n][j]); a block covers 256 columns n
// and up to 32 rows m (their t in LDS), a thread keeps its column's row of B in registers.
constexpr int kUpRows = 32;
constexpr int kUpMaxRank = 64;
__global__ __launch_bounds__(256) void lora_up_add_kernel(const uint16_t* __restrict__ B, const float* __restrict__ t,
                                                          uint16_t* __restrict__ y, int M, int N, int r, float scaling) {
    __shared__ float ts[kUpRows * kUpMaxRank];
    const int n = blockIdx.x * 256 + threadIdx.x;
    const int m0 = blockIdx.y * kUpRows;
    const int rows = min(kUpRows, M - m0);
    for (int i = threadIdx.x; i < rows * r; i += 256) ts[i] = t[(size_t)m0 * r + i];
    __syncthreads();
    if (n >= N) return;
    float b[kUpMaxRank];
#pragma unroll
    for (int j = 0; j < kUpMaxRank; j += 8) {
        if (j < r) {
            const uint4 v = *reinterpret_cast<const uint4*>(B + (size_t)n * r + j);
            const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                b[j + 2 * e] = __builtin_bit_cast(float, w[e] << 16);
                b[j + 2 * e + 1] = __builtin_bit_cast(float, w[e] & 0xFFFF0000u);
            }
        } else {
#pragma unroll
            for (int e = 0; e < 8; ++e) b[j + e] = 0.f;
        }
    }
    for (int mi = 0; mi < rows; ++mi) {
        float dot = 0.f;
#pragma unroll
        for (int j = 0; j < kUpMaxRank; ++j)
            if (j < r) dot = fmaf(ts[mi * r + j], b[j], dot);
        uint16_t* yp = y + (size_t)(m0 + mi) * N + n;
        *yp = f32_to_bf16_rne(fmaf(scaling, dot, bf16_bits_to_f32(*yp)));
    }
}

}  // namespace

bool lora_supports(const qail_wdesc& d, const qail_lora& l) {
    return l.r >= 8 && l.r <= kUpMaxRank && l.r % 8 == 0 && d.K % 8 == 0;
}

// t for item i starts at t + i * M * t_stride floats, rows of r floats... laid out [M][r] with
// the item's own r; t_stride >= r is the per-item allotment per row.
hipError_t launch_lora_down(const qail_w4a16_item* items, const qail_lora* loras, float* t, int t_stride,
                            int count, int M, hipStream_t st) {
    for (int i0 = 0; i0 < count; i0 += kMaxLoraItems) {
        const int c = (count - i0 < kMaxLoraItems) ? count - i0 : kMaxLoraItems;
        DownArgs a;
        int rmax = 0;
        for (int i = 0; i < c; ++i) {
            const qail_w4a16_item& s = items[i0 + i];
            const qail_lora& l = loras[i0 + i];
            a.it[i] = DownItem{s.x, l.A, t + (size_t)(i0 + i) * M * t_stride, s.d.K, l.r};
            if (l.r > rmax) rmax = l.r;
        }
        for (int i = c; i < kMaxLoraItems; ++i) a.it[i] = a.it[c - 1];
        a.M = M;
        hipLaunchKernelGGL(lora_down_kernel, dim3(rmax, M, c), dim3(kDownThreads), 0, st, a);
        const hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

hipError_t launch_lora_up_add(const qail_w4a16_item& it, const qail_lora& l, const float* t, int M, hipStream_t st) {
    dim3 grid((it.d.N + 255) / 256, (M + kUpRows - 1) / kUpRows);
    hipLaunchKernelGGL(lora_up_add_kernel, grid, dim3(256), 0, st, l.B, t, it.y, M, it.d.N, l.r, l.scaling);
    return hipGetLastError();
}

}  // namespace qail
