// W4A16 linear for a small batch, 2 <= M <= 16: y[m][n] = sum_k x[m][k] (q[n][k] - z[n][k/g]) s[n][k/g].
//
// Appendix "Analysis": decode is bound by streaming the packed weights; with a few
// sequences decoded together the weights are still read once, so the kernel keeps the
// structure of the M = 1 stream and lets the matrix cores serve all M rows of x at once.
//
//   * A tile is 16 weight rows.  For v_mfma_f32_16x16x32_bf16 lane l = 16*kb + i supplies, as
//     B operand, 8 consecutive k of column (weight row) i starting at 8*kb: exactly one packed
//     word.  A lane loads 16 bytes = 4 words = 32 k of its row, so one wave-wide load covers
//     16 rows x 128 k (64 contiguous bytes per row) and feeds 4 MFMAs; 128 k is one
//     quantisation group (group_size is a multiple of 128), so the group's scale and
//     zero-point are applied to the 16 x 16 result of those 4 MFMAs:
//         sum_k x (q - z) s = s * ( sum_k x (q + 128)  -  (128 + z) * sum_k x )
//     with (q + 128) as bf16 = 0x4300 | q (one AND-OR per nibble pair) and sum_k x per
//     (row of x, 128-k step) computed once per wave.
//   * The 16 waves of a block split K among themselves (whole 128-k steps), so a wave's share
//     of x fits in registers as ready-made A operands (16 registers per step) and is never
//     re-read; every wave walks all tiles of the block's slab of rows, keeping about 8
//     wave-wide loads in flight in a register ring, and the 16 partial 16 x 16 results of a
//     tile are summed through LDS in a fixed order (deterministic).
//   * Nothing is stored to global memory while loads are in flight (a store would break the
//     in-order completion the exact load waits rely on): results are collected in LDS and
//     written once at the end.  K beyond 6144 is walked in several passes over the slab, each
//     adding to the collected results.
//   * As for M = 1, one launch serves a list of linears, blocks divided by bytes.
#include "qail_internal.h"

namespace qail {

namespace {

constexpr int kSmMaxItems = 16;
constexpr int kSmWaves = 16;
constexpr int kSmThreads = kSmWaves * kWave;
constexpr int kStepK = 128;         // k per wave-wide load
constexpr int kSmMaxSteps = 3;      // steps per wave and pass (x operands held in registers)
constexpr int kSmMaxPasses = 4;     // passes over K: K <= 4 * 16 * 3 * 128 = 24576
constexpr int kSmMaxTiles = 48;     // tiles per block (LDS result buffer)
constexpr int kRound = 4;           // tiles per LDS reduction round

struct SmItem {
    const uint32_t* qw;
    const uint16_t* sc;
    const uint32_t* zr;
    const uint16_t* x;
    uint16_t* y;
    int N, K, g;
    int block_begin, blocks;
};

struct SmArgs {
    SmItem it[kSmMaxItems];
    int count;
    int M;
};

// LDS: partial sums [kRound][16 waves][4][64] fp32, results [kSmMaxTiles][4][64] fp32, and the
// per-wave table of step sums of x [16 waves][3 steps][16 rows] fp32.
constexpr int kPartialFloats = kRound * kSmWaves * 256;
constexpr size_t kSmLdsBytes = (size_t)kPartialFloats * 4 + (size_t)kSmMaxTiles * 256 * 4 +
                               (size_t)kSmWaves * kSmMaxSteps * 16 * 4;

template <int SPW, int PT>
__device__ __forceinline__ void smallm_tiles(const SmItem& it, int M, int tile0, int nt, int wave, int lane,
                                             int npass, float* __restrict__ partial,
                                             float* __restrict__ result, float* __restrict__ xs_tab) {
    const int K = it.K, N = it.N, g = it.g;
    const int G = K / g, zwords = (G + 7) / 8, kw = K / 8;
    const int Sall = K / kStepK;
  for (int pass = 0; pass < npass; ++pass) {
    // one pass: the 128-k steps [sb, se) of every tile of the slab, split among the 16 waves
    const int sb = (int)(((long long)Sall * pass) / npass), se = (int)(((long long)Sall * (pass + 1)) / npass);
    const bool first_pass = pass == 0;
    const int S = se - sb;
    const int ks0 = sb + (int)(((long long)S * wave) / kSmWaves), ks1 = sb + (int)(((long long)S * (wave + 1)) / kSmWaves);
    const int li = lane & 15, kb = lane >> 4;

    // ---- register ring of PT tiles x SPW steps of weight loads, issued first: the loads of x
    // below then overlap with them
    uint4 q[PT][SPW];
    _Float16 sh[PT][SPW];  // kept in its loaded type: a widening at the load would wait there
    uint32_t zw[PT][SPW];
    int stepw[SPW], grp[SPW];
#pragma unroll
    for (int i = 0; i < SPW; ++i) {
        const int st = max(sb, min(ks0 + i, max(ks1, sb + 1) - 1));  // steps past the wave's share re-read its last one
        stepw[i] = st * (kStepK / 8) + 4 * kb;
        grp[i] = (st * kStepK) / g;
    }
    auto issue = [&](int p, int i, int tile) {
        const int row = min(tile * 16 + li, N - 1);
        q[p][i] = *reinterpret_cast<const uint4*>(it.qw + (size_t)row * kw + stepw[i]);
        sh[p][i] = reinterpret_cast<const _Float16*>(it.sc)[(size_t)row * G + grp[i]];
        zw[p][i] = it.zr[(size_t)row * zwords + (grp[i] >> 3)];
    };
    const int tlast = tile0 + nt - 1;
#pragma unroll
    for (int p = 0; p < PT; ++p)
#pragma unroll
        for (int i = 0; i < SPW; ++i) {
            issue(p, i, min(tile0 + p, tlast));
            __builtin_amdgcn_sched_barrier(0);  // program order = consumption order
        }

    // ---- this wave's share of x as A operands: row li of x, k = 128*step + 32*kb + 8*j + (0..7),
    // in the pair order x0,x4 | x1,x5 | x2,x6 | x3,x7 that the nibble expansion produces
    uint4 xa[SPW][4];
    // sum of x over each step, per row of x: parked in the wave's LDS table [step][m] and read
    // back four rows at a time (a lane's results are rows m = 4*kb .. 4*kb + 3)
    float* xs_w = xs_tab + wave * (kSmMaxSteps * 16);
#pragma unroll
    for (int i = 0; i < SPW; ++i) {
        const bool live = (ks0 + i < ks1) && (li < M);
        float part = 0.f;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            uint4 v = make_uint4(0, 0, 0, 0);
            if (live)
                v = *reinterpret_cast<const uint4*>(it.x + (size_t)li * K + (size_t)(ks0 + i) * kStepK + 32 * kb + 8 * j);
            const uint32_t u[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
            for (int e = 0; e < 4; ++e)
                part += __builtin_bit_cast(float, u[e] << 16) + __builtin_bit_cast(float, u[e] & 0xFFFF0000u);
            xa[i][j].x = (v.x & 0xFFFFu) | (v.z << 16);      // x0,x4
            xa[i][j].y = (v.x >> 16) | (v.z & 0xFFFF0000u);  // x1,x5
            xa[i][j].z = (v.y & 0xFFFFu) | (v.w << 16);      // x2,x6
            xa[i][j].w = (v.y >> 16) | (v.w & 0xFFFF0000u);  // x3,x7
        }
        part += __shfl_xor(part, 16, kWave);
        part += __shfl_xor(part, 32, kWave);  // every lane with the same li now holds sum_k x[li][step]
        if (kb == 0) xs_w[i * 16 + li] = part;
    }
    __syncthreads();  // makes the table visible to the wave's other lanes (and ends the last pass's reads)
    __builtin_amdgcn_sched_barrier(0);

    uint32_t magic = 0x43004300u;    // bf16 pair (128, 128); in a vector register so that the
    asm volatile("" : "+v"(magic));  // AND-OR needs only one scalar operand

    // The arithmetic of one tile (slot p of the ring); its 16 x 16 partial result goes to LDS.
    auto consume = [&](int p, int slot) {
        f32x4_t acc = {0.f, 0.f, 0.f, 0.f};
        int xo = 4 * kb;  // opaque, so that the table reads below stay in the loop instead of
        asm volatile("" : "+v"(xo));  // being hoisted into (and spilled from) registers
#pragma unroll
        for (int i = 0; i < SPW; ++i) {
            const uint32_t w[4] = {q[p][i].x, q[p][i].y, q[p][i].z, q[p][i].w};
            f32x4_t d = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const uint4 b = make_uint4((w[j] & 0x000F000Fu) | magic, ((w[j] >> 4) & 0x000F000Fu) | magic,
                                           ((w[j] >> 8) & 0x000F000Fu) | magic, ((w[j] >> 12) & 0x000F000Fu) | magic);
                d = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, xa[i][j]),
                                                            __builtin_bit_cast(bf16x8_t, b), d, 0, 0, 0);
            }
            const float s = (float)sh[p][i];
            const float zc = (float)(128u + ((zw[p][i] >> (4 * (grp[i] & 7))) & 0xFu));
            const float4 xs = *reinterpret_cast<const float4*>(xs_w + i * 16 + xo);
            acc[0] = fmaf(s, fmaf(-zc, xs.x, d[0]), acc[0]);
            acc[1] = fmaf(s, fmaf(-zc, xs.y, d[1]), acc[1]);
            acc[2] = fmaf(s, fmaf(-zc, xs.z, d[2]), acc[2]);
            acc[3] = fmaf(s, fmaf(-zc, xs.w, d[3]), acc[3]);
        }
        float* dst = partial + (slot * kSmWaves + wave) * 256 + lane;
#pragma unroll
        for (int r = 0; r < 4; ++r) dst[r * kWave] = acc[r];
    };

    // Sums the 16 partial results of the first `nslots` tiles of a round into the block's
    // result buffer (same (register, lane) layout as the partials).
    auto reduce_round = [&](int first_local_tile, int nslots) {
        __syncthreads();
        const int slot = threadIdx.x >> 8, o = threadIdx.x & 255;
        if (slot < nslots) {
            float sum = 0.f;
#pragma unroll
            for (int wv = 0; wv < kSmWaves; ++wv) sum += partial[(slot * kSmWaves + wv) * 256 + o];
            float* dst = result + (first_local_tile + slot) * 256 + o;
            *dst = first_pass ? sum : *dst + sum;
        }
        __syncthreads();
    };

    int t = 0;
    for (; t + PT < nt; t += PT) {
#pragma unroll
        for (int p = 0; p < PT; ++p) {
            consume(p, p % kRound);
#pragma unroll
            for (int i = 0; i < SPW; ++i) {
                issue(p, i, min(tile0 + t + p + PT, tlast));
                __builtin_amdgcn_sched_barrier(0);
            }
            if (p % kRound == kRound - 1 || p == PT - 1) reduce_round(t + p - (p % kRound), (p % kRound) + 1);
        }
    }
    // drain: the last (up to PT) tiles, no further loads
#pragma unroll
    for (int p = 0; p < PT; ++p) {
        if (t + p < nt) {
            consume(p, p % kRound);
            const bool last = (t + p == nt - 1);
            if (p % kRound == kRound - 1 || p == PT - 1 || last) reduce_round(t + p - (p % kRound), (p % kRound) + 1);
        }
    }
  }  // pass

}

__global__ __launch_bounds__(kSmThreads) void w4a16_smallm_kernel(const SmArgs args) {
    extern __shared__ __attribute__((aligned(16))) float sm_lds[];
    float* partial = sm_lds;
    float* result = sm_lds + kPartialFloats;
    float* xs_tab = result + kSmMaxTiles * 256;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
    const int lane = threadIdx.x % kWave;

    int idx = 0;
    while (idx + 1 < args.count && args.it[idx + 1].block_begin <= (int)blockIdx.x) ++idx;
    idx = __builtin_amdgcn_readfirstlane(idx);
    const SmItem& it = args.it[idx];
    const int ntiles = (it.N + 15) / 16;
    const int b = (int)blockIdx.x - it.block_begin;
    const int tile0 = (int)(((long long)ntiles * b) / it.blocks);
    const int tile1 = (int)(((long long)ntiles * (b + 1)) / it.blocks);
    const int nt = tile1 - tile0;
    if (nt <= 0) return;  // block-uniform

    // K is walked in passes of at most 16 waves x 3 steps, so that a wave's x operands fit in
    // registers; a pass adds its sums to the results of the passes before it.
    const int S = it.K / kStepK;
    const int npass = (S + kSmWaves * kSmMaxSteps - 1) / (kSmWaves * kSmMaxSteps);
    const int spw = ((S + npass - 1) / npass + kSmWaves - 1) / kSmWaves;  // the same in every pass
    switch (spw) {
        case 1: smallm_tiles<1, 6>(it, args.M, tile0, nt, wave, lane, npass, partial, result, xs_tab); break;
        case 2: smallm_tiles<2, 3>(it, args.M, tile0, nt, wave, lane, npass, partial, result, xs_tab); break;
        default: smallm_tiles<3, 2>(it, args.M, tile0, nt, wave, lane, npass, partial, result, xs_tab); break;
    }

    // write the block's results: result[tile][r][l] holds y[m = 4*(l/16) + r][(tile0 + tile)*16 + l%16]
    const int M = args.M, N = it.N;
    for (int idx = threadIdx.x; idx < nt * 256; idx += kSmThreads) {
        const int tile = idx >> 8, rem = idx & 255;
        const int m = rem >> 4, n = rem & 15;           // consecutive threads -> consecutive n
        const int row = (tile0 + tile) * 16 + n;
        if (m < M && row < N)
            it.y[(size_t)m * N + row] = f32_to_bf16_rne(result[tile * 256 + (m & 3) * 64 + (m >> 2) * 16 + n]);
    }
}

int sm_device_cus() {
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

size_t sm_item_bytes(const qail_wdesc& d) {
    const size_t G = (size_t)d.K / d.group_size;
    return (size_t)d.N * (d.K / 2 + G * 2 + ((G + 7) / 8) * 4);
}

hipError_t sm_launch_chunk(const qail_w4a16_item* items, int count, int M, hipStream_t st) {
    static bool attr_done = false;  // more than 64 KB of LDS needs an opt-in, once per process
    if (!attr_done) {
        const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&w4a16_smallm_kernel),
                                                 hipFuncAttributeMaxDynamicSharedMemorySize, (int)kSmLdsBytes);
        if (e != hipSuccess) return e;
        attr_done = true;
    }
    SmArgs a;
    int grid = sm_device_cus();
    if (grid < count) grid = count;
    double total = 0;
    for (int i = 0; i < count; ++i) total += (double)sm_item_bytes(items[i].d);
    int nb[kSmMaxItems], lo[kSmMaxItems], hi[kSmMaxItems];
    double frac[kSmMaxItems];
    int used = 0;
    for (int i = 0; i < count; ++i) {
        const int ntiles = (items[i].d.N + 15) / 16;
        lo[i] = (ntiles + kSmMaxTiles - 1) / kSmMaxTiles;  // the LDS result buffer bounds a block's tiles
        hi[i] = ntiles;
        const double share = (double)sm_item_bytes(items[i].d) / total * grid;
        nb[i] = (int)share;
        if (nb[i] < lo[i]) nb[i] = lo[i];
        if (nb[i] > hi[i]) nb[i] = hi[i];
        frac[i] = share - (int)share;
        used += nb[i];
    }
    while (used < grid) {
        int best = -1;
        for (int i = 0; i < count; ++i)
            if (nb[i] < hi[i] && (best < 0 || frac[i] > frac[best])) best = i;
        if (best < 0) break;
        ++nb[best];
        frac[best] = -1.0;
        ++used;
    }
    int bb = 0;
    for (int i = 0; i < count; ++i) {
        const qail_w4a16_item& s = items[i];
        SmItem& t = a.it[i];
        t.qw = s.qweight; t.sc = s.scales; t.zr = s.zeros; t.x = s.x; t.y = s.y;
        t.N = s.d.N; t.K = s.d.K; t.g = s.d.group_size;
        t.block_begin = bb;
        t.blocks = nb[i];
        bb += nb[i];
    }
    for (int i = count; i < kSmMaxItems; ++i) a.it[i] = a.it[count - 1];
    a.count = count;
    a.M = M;
    hipLaunchKernelGGL(w4a16_smallm_kernel, dim3(bb), dim3(kSmThreads), kSmLdsBytes, st, a);
    return hipGetLastError();
}

}  // namespace

bool smallm_supports(const qail_wdesc& d, int M) {
    return M >= 2 && M <= 16 && d.K % kStepK == 0 && d.group_size % kStepK == 0 &&
           d.K <= kSmMaxPasses * kSmWaves * kSmMaxSteps * kStepK;
}

hipError_t launch_w4a16_smallm(const qail_w4a16_item* items, int count, int M, hipStream_t st) {
    for (int i0 = 0; i0 < count; i0 += kSmMaxItems) {
        const int c = (count - i0 < kSmMaxItems) ? count - i0 : kSmMaxItems;
        const hipError_t e = sm_launch_chunk(items + i0, c, M, st);
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

}  // namespace qail
