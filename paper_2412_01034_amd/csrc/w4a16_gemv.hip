// W4A16 linear for M = 1 (decode): y[n] = sum_k x[k] * (q[n,k] - z[n,k/g]) * s[n,k/g].
//
// Appendix "Analysis": the decode stage is memory-bound, its time is the time to
// stream the packed weights.  The kernel is therefore organised around the HBM
// stream: each lane fetches 16 bytes (32 codes) of a row per load, a wave covers
// 2048 consecutive k of one row, and the arithmetic per weight is kept to about
// 1.5 vector-ALU operations so that it hides under the loads:
//
//   sum_k x_k (q_k - z) s  =  s * ( sum_k x_k (q_k + 128)  -  (128 + z) * sum_k x_k )
//
//   * (q_k + 128) as bf16 is the bit pattern 0x4300 | q_k, so one AND-OR turns two
//     nibbles of a packed word into a bf16 pair; nibbles j and j+4 come out
//     together, and x is staged in LDS in that pair order once per block.
//   * the pair products go through v_dot2c_f32_bf16 (fp32 accumulate).
//   * sum_k x_k per 32-k chunk is computed once per block; a chunk never straddles
//     a group because group_size is a multiple of 32.
//
// One launch serves a list of independent linears (a work list in the kernel
// arguments), so that a decode layer's four GEMVs ramp up once.
#include "qail_internal.h"

namespace qail {

namespace {

constexpr int kGemvMaxItems = 16;
constexpr int kGemvWaves = 16;                    // waves per block
constexpr int kGemvThreads = kGemvWaves * kWave;  // 1024
constexpr int kChunkK = 32;                       // k per lane per load (16 bytes of codes)
constexpr int kWaveK = kWave * kChunkK;           // 2048 k per wave-wide load
constexpr int kGemvMaxK = 16384;                  // x (32 KB) + chunk sums (2 KB) in LDS

struct GemvItem {
    const uint32_t* qw;
    const uint16_t* sc;
    const uint32_t* zr;
    const uint16_t* x;
    uint16_t* y;
    int N, K, g;
    int pass_begin;  // first pass (of rows_per_pass rows) of this item in the launch
};

struct GemvArgs {
    GemvItem it[kGemvMaxItems];
    int count;
    int total_passes;
};

__device__ __forceinline__ float dot2_bf16(uint32_t a, uint32_t b, float c) {
    return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, a),
                                           __builtin_bit_cast(bf16x2_t, b), c, false);
}

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off, kWave);
    return v;
}

// 32 codes (one uint4) against the matching 32 staged activations.
__device__ __forceinline__ float dot32(const uint4& q, const uint4* __restrict__ xl) {
    float acc = 0.f;
    const uint32_t w[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const uint4 xv = xl[j];
        const uint32_t t0 = (w[j] & 0x000F000Fu) | 0x43004300u;          // codes 0,4
        const uint32_t t1 = ((w[j] >> 4) & 0x000F000Fu) | 0x43004300u;   // codes 1,5
        const uint32_t t2 = ((w[j] >> 8) & 0x000F000Fu) | 0x43004300u;   // codes 2,6
        const uint32_t t3 = ((w[j] >> 12) & 0x000F000Fu) | 0x43004300u;  // codes 3,7
        acc = dot2_bf16(t0, xv.x, acc);
        acc = dot2_bf16(t1, xv.y, acc);
        acc = dot2_bf16(t2, xv.z, acc);
        acc = dot2_bf16(t3, xv.w, acc);
    }
    return acc;
}

// R rows per wave per pass; a pass is kGemvWaves * R consecutive rows of one item.
template <int R>
__global__ __launch_bounds__(kGemvThreads) void w4a16_gemv_kernel(const GemvArgs args) {
    extern __shared__ uint4 lds[];
    // layout: x pairs, K/8 uint4 (8 bf16 each, order x0,x4,x1,x5,x2,x6,x3,x7), then K/32 floats
    const int wave = threadIdx.x / kWave;
    const int lane = threadIdx.x % kWave;

    const int nb = gridDim.x;
    const int p_begin = (int)(((long long)args.total_passes * blockIdx.x) / nb);
    const int p_end = (int)(((long long)args.total_passes * (blockIdx.x + 1)) / nb);

    int cur = -1;
    for (int p = p_begin; p < p_end; ++p) {
        int idx = 0;
        while (idx + 1 < args.count && args.it[idx + 1].pass_begin <= p) ++idx;
        idx = __builtin_amdgcn_readfirstlane(idx);
        const GemvItem& it = args.it[idx];
        const int K = it.K, N = it.N, g = it.g;
        float* xs = reinterpret_cast<float*>(lds + K / 8);

        if (idx != cur) {
            if (cur >= 0) __syncthreads();  // everyone is done with the previous x
            const uint4* xg = reinterpret_cast<const uint4*>(it.x);
            for (int i = threadIdx.x; i < K / 8; i += kGemvThreads) {
                const uint4 v = xg[i];  // (x0,x1) (x2,x3) (x4,x5) (x6,x7)
                uint4 o;
                o.x = (v.x & 0xFFFFu) | (v.z << 16);          // x0,x4
                o.y = (v.x >> 16) | (v.z & 0xFFFF0000u);      // x1,x5
                o.z = (v.y & 0xFFFFu) | (v.w << 16);          // x2,x6
                o.w = (v.y >> 16) | (v.w & 0xFFFF0000u);      // x3,x7
                lds[i] = o;
            }
            __syncthreads();
            for (int c = threadIdx.x; c < K / kChunkK; c += kGemvThreads) {
                float s = 0.f;
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const uint4 v = lds[c * 4 + j];
                    const uint32_t u[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        s += __builtin_bit_cast(float, u[e] << 16) +
                             __builtin_bit_cast(float, u[e] & 0xFFFF0000u);
                }
                xs[c] = s;
            }
            __syncthreads();
            cur = idx;
        }

        const int G = K / g;
        const int zwords = (G + 7) / 8;
        const int kw = K / 8;
        const int row0 = (p - it.pass_begin) * (kGemvWaves * R) + wave * R;

        float acc[R];
        int rown[R];
#pragma unroll
        for (int r = 0; r < R; ++r) {
            acc[r] = 0.f;
            rown[r] = min(row0 + r, N - 1);  // clamp: tail rows are read, not stored
        }

        for (int k0 = lane * kChunkK; k0 < K; k0 += kWaveK) {
            const int grp = k0 / g;
            uint4 q[R];
            uint32_t sb[R], zw[R];
#pragma unroll
            for (int r = 0; r < R; ++r) {
                q[r] = *reinterpret_cast<const uint4*>(it.qw + (size_t)rown[r] * kw + k0 / 8);
                sb[r] = it.sc[(size_t)rown[r] * G + grp];
                zw[r] = it.zr[(size_t)rown[r] * zwords + grp / 8];
            }
            const float xsum = xs[k0 / kChunkK];
            const uint4* xl = lds + k0 / 8;
#pragma unroll
            for (int r = 0; r < R; ++r) {
                const float d = dot32(q[r], xl);
                const float s = f16_bits_to_f32((uint16_t)sb[r]);
                const float zc = (float)(128u + ((zw[r] >> (4 * (grp & 7))) & 0xFu));
                acc[r] = fmaf(s, fmaf(-zc, xsum, d), acc[r]);
            }
        }
#pragma unroll
        for (int r = 0; r < R; ++r) {
            const float v = wave_sum(acc[r]);
            if (lane == 0 && row0 + r < N) it.y[row0 + r] = f32_to_bf16_rne(v);
        }
    }
}

int device_cus() {
    static int cus = 0;
    if (cus == 0) {
        int dev = 0;
        hipDeviceProp_t prop;
        if (hipGetDevice(&dev) == hipSuccess && hipGetDeviceProperties(&prop, dev) == hipSuccess)
            cus = prop.multiProcessorCount;
        if (cus <= 0) cus = 256;
    }
    return cus;
}

template <int R>
hipError_t launch_chunk(const qail_w4a16_item* items, int count, hipStream_t st) {
    GemvArgs a;
    int passes = 0;
    int maxK = 0;
    for (int i = 0; i < count; ++i) {
        const qail_w4a16_item& s = items[i];
        GemvItem& t = a.it[i];
        t.qw = s.qweight; t.sc = s.scales; t.zr = s.zeros; t.x = s.x; t.y = s.y;
        t.N = s.d.N; t.K = s.d.K; t.g = s.d.group_size;
        t.pass_begin = passes;
        passes += (s.d.N + kGemvWaves * R - 1) / (kGemvWaves * R);
        if (s.d.K > maxK) maxK = s.d.K;
    }
    for (int i = count; i < kGemvMaxItems; ++i) a.it[i] = a.it[count - 1];
    a.count = count;
    a.total_passes = passes;
    const size_t lds = (size_t)maxK * 2 + (size_t)(maxK / kChunkK) * 4;
    int grid = device_cus();
    if (grid > passes) grid = passes;
    hipLaunchKernelGGL(w4a16_gemv_kernel<R>, dim3(grid), dim3(kGemvThreads), lds, st, a);
    return hipGetLastError();
}

}  // namespace

bool gemv_supports(const qail_wdesc& d) {
    return d.K % kChunkK == 0 && d.group_size % kChunkK == 0 && d.K <= kGemvMaxK;
}

hipError_t launch_w4a16_gemv(const qail_w4a16_item* items, int count, hipStream_t st) {
    for (int i0 = 0; i0 < count; i0 += kGemvMaxItems) {
        const int c = (count - i0 < kGemvMaxItems) ? count - i0 : kGemvMaxItems;
        long long rows = 0;
        for (int i = 0; i < c; ++i) rows += items[i0 + i].d.N;
        // more rows per wave once every CU has several passes to chew on
        const long long per_cu = rows / device_cus();
        hipError_t e;
        if (per_cu >= 4 * kGemvWaves * 4) e = launch_chunk<4>(items + i0, c, st);
        else if (per_cu >= 2 * kGemvWaves * 2) e = launch_chunk<2>(items + i0, c, st);
        else e = launch_chunk<1>(items + i0, c, st);
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

}  // namespace qail
