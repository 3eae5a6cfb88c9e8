// W4A16 linear for 2 <= M <= 4 (a few sequences decoded together):
//   y[m][n] = sum_k x[m][k] * (q[n,k] - z[n,k/g]) * s[n,k/g].
//
// Appendix "Analysis": decode is bound by streaming the packed weights, and a few rows of x
// do not change that.  The kernel keeps the M = 1 stream (w4a16_gemv.hip) and its arithmetic,
//
//   sum_k x_k (q_k - z) s  =  s * ( sum_k x_k (q_k + 1024)  -  1024 sum_k x_k  -  z sum_k x_k ),
//
// with (q_k + 1024) as fp16 = 0x6400 | q_k, but uses every entry of the small matrix products
// instead of their diagonals.  v_mfma_f32_4x4x4_16b_f16 computes 16 independent 4x4x4 products;
// lane l = 4b + j supplies row j of A and column j of B of product b (4 values each) and
// receives column j of D.  Here product b is a stretch of k, the four rows of A are four
// neighbouring weight rows and the four columns of B are the (up to) four rows of x:
//
//   lane 4b + i loads 16 bytes (32 codes) of weight row n0 + i at k = 512 c + 32 b ...,
//   lane 4b + j reads from LDS the same 32 k of row j of x,
//
// so that after eight chained instructions lane 4b + j holds, for i = 0..3, the dot product of
// weight row n0 + i with row j of x over those 32 k.  A wave-wide load is four rows x 256
// contiguous bytes.  Scale and zero-point belong to a weight row and are loaded by the lane that
// loads the row's codes; the lanes of a quad pass them to each other through DPP operands.
// The sums over the 16 stretches b meet once per four rows (cross-lane adds), results stay in
// registers until the wave has finished its rows.
//
// As in the M = 1 kernel: x is staged once per block in LDS as fp16 with a power of two per
// 32-k stretch, together with the per-stretch sums the offsets need; a block works on rows of
// one linear; one launch serves a list of linears, blocks divided by bytes; every wave keeps a
// ring of wave-wide loads in flight with exact load waits (all loads unconditional, program
// order = consumption order, nothing stored while loads fly); addresses are buffer descriptor
// + scalar offset + a lane offset that never changes.
#include <string.h>

#include <atomic>

#include "qail_internal.h"

namespace qail {

namespace {

constexpr int kD4MaxItems = 16;
constexpr int kD4Waves = 16;
constexpr int kD4Threads = kD4Waves * kWave;
constexpr int kD4Ring = 8;            // wave-wide loads (1 KB each) in flight per wave
constexpr int kD4ChunkK = 512;        // k of a row per wave-wide load
constexpr int kD4MaxChunks = 24;      // K <= 12288: x of four rows and its constants fit in LDS
constexpr int kD4MaxBlocks = 4096;    // blocks of a launch that serves more than one item
constexpr int kD4XRuns = kD4MaxChunks * (kD4ChunkK / 8) * 4 / kD4Threads;  // 8-k runs of x per thread

typedef __attribute__((ext_vector_type(4))) uint32_t u32x4_t;
typedef __attribute__((ext_vector_type(4))) _Float16 f16x4_t;

// 64 bytes, so that a block fetches everything it needs to know with one scalar load.
struct D4Item {
    const uint32_t* qw;
    const uint16_t* sc;
    const uint32_t* zr;
    const uint16_t* x;
    uint16_t* y;
    int N, K, g;
    int block_begin;  // first block of the grid that works on this item
    int quads_base;   // block b of the item owns quads_base groups of four rows, one more if
    int quads_rem;    // b < quads_rem, in the order of the blocks
};

struct D4Args {
    D4Item it[kD4MaxItems];
    uint32_t item_of_block[kD4MaxBlocks / 8];  // 4 bits per block; blocks past the table work on item 0
    int M;
};

template <int kCtrl>
__device__ __forceinline__ float dpp_f(float v) {
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), kCtrl, 0xF, 0xF, true));
}

// acc += (v of lane 4b + i of the caller's quad) * m, in one instruction: the multiply-add reads
// its first operand through the quad permute.  Written as assembly because the compiler emits
// a separate v_mov_b32_dpp per operand instead; the s_nop covers the two wait states a DPP read
// needs after a vector write of the same register, which the compiler cannot see in here.
template <int i>
__device__ __forceinline__ void quad_fmac(float& acc, float v, float m);
#define QAIL_QUAD_FMAC(i)                                                                                   \
    template <>                                                                                             \
    __device__ __forceinline__ void quad_fmac<i>(float& acc, float v, float m) {                            \
        asm("s_nop 1\n\tv_fmac_f32_dpp %0, %1, %2 quad_perm:[" #i "," #i "," #i "," #i                      \
            "] row_mask:0xf bank_mask:0xf bound_ctrl:1"                                                     \
            : "+v"(acc)                                                                                     \
            : "v"(v), "v"(m));                                                                              \
    }
QAIL_QUAD_FMAC(0)
QAIL_QUAD_FMAC(1)
QAIL_QUAD_FMAC(2)
QAIL_QUAD_FMAC(3)
#undef QAIL_QUAD_FMAC

// Sum over the 16 lanes that share lane % 4 (all stretches b of one row of x); every lane gets it.
__device__ __forceinline__ float sum_over_stretches(float v) {
    v += dpp_f<0x124>(v);  // row_ror:4
    v += dpp_f<0x128>(v);  // row_ror:8: the four stretches of this 16-lane row
    v += __shfl_xor(v, 16);
    v += __shfl_xor(v, 32);
    return v;
}

// LDS map of a block (uint4 units), nc = ceil(K / 512) chunks per row:
//   [0, nc*256)        staged activations: word e of lane L in chunk c at (c*4 + e)*64 + L
//   then nc*64 float4  constants of lane L's stretch of chunk c at c*64 + L, with P = 2^e:
//                      (P * 1024 * sum of the staged values, -P * sum of x * 2^-e, P, unused)
// Lane L = 4b + j owns, in chunk c, the 32 k starting at 512 c + 32 b of row j of x (rows past
// M are zero).  Its staged word e holds those k's 8e..8e+7 as fp16 in the order
// x0,x4 | x1/16,x5/16 | x2,x6 | x3/16,x7/16 (all times 2^-e), matching the four registers the
// weight nibbles are expanded into.  Everything past K is zero.
__global__ __launch_bounds__(kD4Threads) void w4a16_decode4_kernel(const D4Args args) {
    extern __shared__ uint4 d4_lds[];
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
    const int lane = threadIdx.x % kWave;
    const int li = lane & 3, lb = lane >> 2;  // row of the quad (or row of x), stretch
    const int M = args.M;

    int idx = 0;
    if (blockIdx.x < (unsigned)kD4MaxBlocks) idx = (args.item_of_block[blockIdx.x / 8] >> (4 * (blockIdx.x % 8))) & 15;
    idx = __builtin_amdgcn_readfirstlane(idx);
    const D4Item it = args.it[idx];
    const int K = it.K, N = it.N, g = it.g;
    const int G = K / g, zwords = (G + 7) / 8, kw = K / 8;
    const int nc = (K + kD4ChunkK - 1) / kD4ChunkK;
    uint4* const xl = d4_lds;
    float4* const consts = reinterpret_cast<float4*>(d4_lds + nc * 4 * kWave);

    // x first: it is needed first and loads return in order.  Run e = 8 consecutive k of one of
    // four rows (rows past M are zeros); the 4 threads of a quad hold the 4 runs of one stretch.
    // Run e of row j at position r is bytes 16 e .. 16 e + 15 of x ([M][K], rows back to back), so the
    // request needs neither j nor r, and runs past row M lie past the end of the buffer and read zeros
    // without a fetch: every load is issued, no condition and no division stands before it.
    const int row_runs = K / 8;
    const __amdgpu_buffer_rsrc_t rx = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t*>(it.x), 0, M * K * 2, 0x00020000);
    uint4 xr[kD4XRuns];
#pragma unroll
    for (int u = 0; u < kD4XRuns; ++u) {
        const u32x4_t v = __builtin_amdgcn_raw_buffer_load_b128(rx, (threadIdx.x + u * kD4Threads) * 16, 0, 0);
        xr[u] = make_uint4(v[0], v[1], v[2], v[3]);
    }
    __builtin_amdgcn_sched_barrier(0);  // the scheduler must not move the x loads behind the weights

    // this block's groups of four rows ("quads"), dealt to its waves in turn
    const int bk = (int)blockIdx.x - it.block_begin;
    const int quad0 = bk * it.quads_base + min(bk, it.quads_rem);
    const int nq = it.quads_base + (bk < it.quads_rem ? 1 : 0);
    const int nqw = max(0, (nq - wave + kD4Waves - 1) / kD4Waves);  // quads of this wave: at most 16
    const int total = nqw * nc;                                     // its stream of (quad, chunk) loads

    // Loads.  Lane offsets never change; quad and chunk go into the scalar offset (which the
    // hardware does not range-check: every address below is inside its tensor; N is a multiple
    // of 4).  Only the last chunk of a row can run past K: a lane whose stretch does reads the
    // first bytes and the first group of that chunk instead (valid data; it meets zeros in x).
    // The host checks that a chunk holds a whole number of groups or a group a whole number of
    // chunks, so a stretch's group is (chunk part) + (lane part).
    const __amdgpu_buffer_rsrc_t rq = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint32_t*>(it.qw), 0, N * kw * 4, 0x00020000);
    const __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t*>(it.sc), 0, N * G * 2, 0x00020000);
    const __amdgpu_buffer_rsrc_t rz = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint32_t*>(it.zr), 0, N * zwords * 4, 0x00020000);
    const int gpc = g < kD4ChunkK ? kD4ChunkK / g : 1;   // groups per chunk
    const int cpg = g < kD4ChunkK ? 1 : g / kD4ChunkK;   // chunks per group
    const int lgrp = g < kD4ChunkK ? (32 * lb) / g : 0;  // lane part of the group index
    const bool tail_out = (nc - 1) * kD4ChunkK + 32 * lb >= K;
    // (a wave without rows asks for offsets past the end of every tensor, all below 2 GB: the range
    // check answers with zeros and fetches nothing.  Its loads are issued all the same: with the
    // ring's first loads behind a condition the compiler can no longer count the loads in flight,
    // and the staging of x below would wait for the weights as well)
    const int past = (int)0x80000000u;
    const int qlane = nqw == 0 ? past : li * kw * 4 + 16 * lb, qlane_last = (tail_out && nqw != 0) ? li * kw * 4 : qlane;
    const int slane = nqw == 0 ? past : li * G * 2 + lgrp * 2, slane_last = (tail_out && nqw != 0) ? li * G * 2 : slane;
    const int zlane = nqw == 0 ? past : li * zwords * 4;
    // the zero-point word of group (chunk part + lane part) is the chunk part's word: the lane
    // part stays below 8 and the chunk part is a multiple of gpc (8 or a divisor of 8)
    // (both counts are powers of two: host check)
    const int cpg_shift = __builtin_ctz(cpg), gpc_shift = __builtin_ctz(gpc);
    auto chunk_group = [&](int c) { return (c >> cpg_shift) << gpc_shift; };

    uint4 q[kD4Ring];
    uint32_t sh[kD4Ring];  // fp16 bits as loaded (zero-extended): a conversion at the load would wait there
    uint32_t zw[kD4Ring];
    int iq = 0, ic = 0;  // quad (of this wave) and chunk of the next load to issue
    auto issue = [&](int p, int iq, int ic) {
        const int n0 = (quad0 + wave + kD4Waves * iq) * 4;
        const int cg = chunk_group(ic);
        const bool last = ic == nc - 1;
        const u32x4_t v = __builtin_amdgcn_raw_buffer_load_b128(rq, last ? qlane_last : qlane,
                                                                n0 * (kw * 4) + ic * (kD4ChunkK / 2), 0);
        q[p] = make_uint4(v[0], v[1], v[2], v[3]);
        sh[p] = __builtin_amdgcn_raw_buffer_load_b16(rs, last ? slane_last : slane, n0 * (G * 2) + cg * 2, 0);
        zw[p] = __builtin_amdgcn_raw_buffer_load_b32(rz, zlane, n0 * (zwords * 4) + (cg >> 3) * 4, 0);
    };
    // next (quad, chunk) of the stream; past its end the last load is repeated (and not consumed)
    auto advance = [&](int& qd, int& ch) {
        const bool last = ch == nc - 1;
        if (!(qd == nqw - 1 && last)) {
            ch = last ? 0 : ch + 1;
            qd += last ? 1 : 0;
        }
    };
#pragma unroll
    for (int p = 0; p < kD4Ring; ++p) {
        issue(p, iq, ic);
        advance(iq, ic);
        __builtin_amdgcn_sched_barrier(0);  // program order = consumption order
    }

    // ---- stage x (whole block; one barrier)
    {
#pragma unroll
        for (int u = 0; u < kD4XRuns; ++u) {
            if (u * kD4Threads >= 4 * row_runs) break;  // block-uniform
            const int e = threadIdx.x + u * kD4Threads;
            // e / row_runs, at most 4 here (the rows past the fourth are skipped below)
            const int j = (e >= row_runs) + (e >= 2 * row_runs) + (e >= 3 * row_runs) + (e >= 4 * row_runs);
            const int r = e - __mul24(j, row_runs);
            const uint32_t w[4] = {xr[u].x, xr[u].y, xr[u].z, xr[u].w};
            float f[8];
            float amax = 0.f;
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                f[2 * t] = __builtin_bit_cast(float, w[t] << 16);
                f[2 * t + 1] = __builtin_bit_cast(float, w[t] & 0xFFFF0000u);
                amax = fmaxf(amax, fmaxf(fabsf(f[2 * t]), fabsf(f[2 * t + 1])));
            }
            amax = fmaxf(amax, dpp_f<0xB1>(amax));  // quad_perm [1,0,3,2]
            amax = fmaxf(amax, dpp_f<0x4E>(amax));  // quad_perm [2,3,0,1]
            // 2^-e with amax * 2^-e in [2^14, 2^15): exponent arithmetic on the bit pattern
            const int ex = (int)((__builtin_bit_cast(uint32_t, amax) >> 23) & 0xFF);
            int down = (amax > 0.f) ? (ex - 141) : 0;  // 141 = 127 + 14
            down = max(-126, min(113, down));           // keeps both exponent fields valid
            const float pre = __builtin_bit_cast(float, (uint32_t)(127 - down) << 23);
            const float pre16 = pre * 0.0625f;
            const bool live = j < M;
            _Float16 h[8];
#pragma unroll
            for (int t = 0; t < 8; ++t) h[t] = live ? (_Float16)(f[t] * ((t & 1) ? pre16 : pre)) : (_Float16)0.f;
            float se = ((float)h[0] + (float)h[4]) + ((float)h[2] + (float)h[6]);
            float so = ((float)h[1] + (float)h[5]) + ((float)h[3] + (float)h[7]);
            se += dpp_f<0xB1>(se);
            se += dpp_f<0x4E>(se);
            so += dpp_f<0xB1>(so);
            so += dpp_f<0x4E>(so);
            if (j < 4) {
                auto pk = [](_Float16 lo, _Float16 hi) {
                    typedef __attribute__((ext_vector_type(2))) _Float16 h2;
                    const h2 v = {lo, hi};
                    return __builtin_bit_cast(uint32_t, v);
                };
                const uint4 o = make_uint4(pk(h[0], h[4]), pk(h[1], h[5]), pk(h[2], h[6]), pk(h[3], h[7]));
                const int c = r / (kD4ChunkK / 8), rr = r % (kD4ChunkK / 8);
                const int L = 4 * (rr >> 2) + j, t = rr & 3;
                xl[(c * 4 + t) * kWave + L] = o;
                if (t == 0)
                {
                    const float P = __builtin_bit_cast(float, (uint32_t)(127 + down) << 23);  // exact factors
                    consts[c * kWave + L] = make_float4(P * (1024.f * (se + so)), -P * (se + 16.f * so), P, 0.f);
                }
            }
        }
        // the part of the last chunk past K, for all four rows
        const int pad = nc * (kD4ChunkK / 8) - row_runs;  // runs per row past K
        for (int e = threadIdx.x; e < pad * 4; e += kD4Threads) {
            const int j = e / pad, r = row_runs + e % pad;
            const int c = r / (kD4ChunkK / 8), rr = r % (kD4ChunkK / 8);
            const int L = 4 * (rr >> 2) + j, t = rr & 3;
            xl[(c * 4 + t) * kWave + L] = make_uint4(0, 0, 0, 0);
            if (t == 0) consts[c * kWave + L] = make_float4(0.f, 0.f, 1.f, 0.f);
        }
    }
    __syncthreads();
    if (total <= 0) return;

    uint32_t magic = 0x64006400u;    // fp16 pair (1024, 1024); held in a vector register so that
    asm volatile("" : "+v"(magic));  // the AND-OR needs only one scalar operand

    // Results stay in registers (the wave's t-th quad in the lanes of stretch t, row j of x in
    // lane 4t + j, the four weight rows in four registers) and are stored once at the end: a store
    // between the loads would break the in-order completion that exact load waits rely on.
    float keep[4] = {0.f, 0.f, 0.f, 0.f};
    float acc[4] = {0.f, 0.f, 0.f, 0.f};
    int cq = 0, cc = 0;  // quad and chunk being consumed

    auto consume = [&](int p, int cq, int cc) {
        int xo = lane;
        asm volatile("" : "+v"(xo));  // keeps the LDS reads inside the loop
        uint4 xv[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) xv[e] = xl[(cc * 4 + e) * kWave + xo];
        const float4 cst = consts[cc * kWave + xo];
        const uint32_t w[4] = {q[p].x, q[p].y, q[p].z, q[p].w};
        f32x4_t d = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            // codes 0,4 | 16*codes 1,5 | codes 2,6 | 16*codes 3,7, each plus 1024, as fp16
            const uint32_t w8 = w[e] >> 8;
            const uint2 a01 = make_uint2((w[e] & 0x000F000Fu) | magic, (w[e] & 0x00F000F0u) | magic);
            const uint2 a23 = make_uint2((w8 & 0x000F000Fu) | magic, (w8 & 0x00F000F0u) | magic);
            d = __builtin_amdgcn_mfma_f32_4x4x4f16(__builtin_bit_cast(f16x4_t, a01),
                                                   __builtin_bit_cast(f16x4_t, make_uint2(xv[e].x, xv[e].y)), d, 0, 0, 0);
            d = __builtin_amdgcn_mfma_f32_4x4x4f16(__builtin_bit_cast(f16x4_t, a23),
                                                   __builtin_bit_cast(f16x4_t, make_uint2(xv[e].z, xv[e].w)), d, 0, 0, 0);
        }
        // this lane's weight row: scale and zero-point of its stretch's group
        const bool last = cc == nc - 1;
        const int grp = chunk_group(cc) + (last && tail_out ? 0 : lgrp);
        const float s = (float)__builtin_bit_cast(_Float16, (uint16_t)sh[p]);
        const float z = (float)((zw[p] >> (4 * (grp & 7))) & 0xFu);
        // register i of d belongs to weight row n0 + i, whose scale and zero-point lane 4b + i holds:
        //   s * P * sum_k x_k (q_k - z) = s * (P D - P xoff) + (s z) * (-P xsum)
        const float sz = s * z;
#define QAIL_D4_ROW(i)                                          \
    {                                                           \
        quad_fmac<i>(acc[i], s, fmaf(cst.z, d[i], -cst.x));     \
        quad_fmac<i>(acc[i], sz, cst.y);                        \
    }
        QAIL_D4_ROW(0) QAIL_D4_ROW(1) QAIL_D4_ROW(2) QAIL_D4_ROW(3)
#undef QAIL_D4_ROW
        asm volatile("" : "+v"(xo));
    };
    // A quad is complete: add up its 16 stretches and park the result.  Kept out of the chunk
    // code and behind a scalar branch: folded into it, the compiler runs the cross-lane adds
    // for every chunk and selects.
    auto finish_quad = [&](int cq) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const float v = sum_over_stretches(acc[i]);
            keep[i] = (lb == cq) ? v : keep[i];
            acc[i] = 0.f;
        }
        asm volatile("" ::: "memory");
    };

    int t = 0;
    for (; t + kD4Ring < total; t += kD4Ring) {
#pragma unroll
        for (int p = 0; p < kD4Ring; ++p) {
            consume(p, cq, cc);
            if (__builtin_amdgcn_readfirstlane(cc == nc - 1)) finish_quad(cq);
            advance(cq, cc);
            issue(p, iq, ic);
            advance(iq, ic);
            __builtin_amdgcn_sched_barrier(0);
        }
    }
#pragma unroll
    for (int p = 0; p < kD4Ring; ++p)
        if (t + p < total) {
            consume(p, cq, cc);
            if (__builtin_amdgcn_readfirstlane(cc == nc - 1)) finish_quad(cq);
            advance(cq, cc);
        }

    // lane 4t + j: y[j][n0 .. n0 + 3] of the wave's t-th quad
    if (lb < nqw && li < M) {
        const int n0 = (quad0 + wave + kD4Waves * lb) * 4;
        uint16_t* dst = it.y + (size_t)li * N + n0;
        uint16_t h[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) h[i] = f32_to_bf16_rne(keep[i]);
        // N is a multiple of 4 (host check), so the four values are one aligned 8-byte piece of row li of y
        *reinterpret_cast<uint2*>(dst) = make_uint2(h[0] | ((uint32_t)h[1] << 16), h[2] | ((uint32_t)h[3] << 16));
    }
}

size_t d4_item_bytes(const qail_wdesc& d) {
    const size_t G = (size_t)d.K / d.group_size;
    return (size_t)d.N * (d.K / 2 + G * 2 + ((G + 7) / 8) * 4);
}

size_t d4_lds_bytes(const qail_wdesc& d) {
    const size_t nc = ((size_t)d.K + kD4ChunkK - 1) / kD4ChunkK;
    return nc * kWave * (4 * 16 + 16);  // staged activations and per-stretch constants
}

hipError_t d4_launch_chunk(const qail_w4a16_item* items, int count, int M, hipStream_t st) {
    // more than 64 KB of LDS needs an opt-in; the call is idempotent, so two host threads that
    // both find the flag clear may both make it
    static std::atomic<bool> attr_done{false};
    if (!attr_done.load(std::memory_order_acquire)) {
        const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&w4a16_decode4_kernel),
                                                 hipFuncAttributeMaxDynamicSharedMemorySize,
                                                 kD4MaxChunks * kWave * (4 * 16 + 16));
        if (e != hipSuccess) return e;
        attr_done.store(true, std::memory_order_release);
    }
    D4Args a;
    memset(a.item_of_block, 0, sizeof(a.item_of_block));
    int grid = device_cu_count();
    if (grid < count) grid = count;
    // blocks per item in proportion to its bytes (largest remainder), at least one each
    double total = 0;
    for (int i = 0; i < count; ++i) total += (double)d4_item_bytes(items[i].d);
    int nb[kD4MaxItems], cap[kD4MaxItems];
    double frac[kD4MaxItems];
    int used = 0;
    for (int i = 0; i < count; ++i) {
        const int quads = (items[i].d.N + 3) / 4;
        const double share = (double)d4_item_bytes(items[i].d) / total * grid;
        nb[i] = (int)share;
        if (nb[i] < 1) nb[i] = 1;
        // a wave parks the results of at most 16 quads: at most 256 quads per block
        const int need = (quads + kD4Waves * 16 - 1) / (kD4Waves * 16);
        if (nb[i] < need) nb[i] = need;
        cap[i] = quads;  // no more blocks than quads
        if (nb[i] > cap[i]) nb[i] = cap[i];
        frac[i] = share - (int)share;
        used += nb[i];
    }
    while (used < grid) {
        int best = -1;
        for (int i = 0; i < count; ++i)
            if (nb[i] < cap[i] && (best < 0 || frac[i] > frac[best])) best = i;
        if (best < 0) break;
        ++nb[best];
        frac[best] = -1.0;
        ++used;
    }
    if (count > 1 && used > kD4MaxBlocks) {
        // the block-to-item table is too short: one launch per item (a lone item needs no table)
        for (int i = 0; i < count; ++i) {
            const hipError_t e = d4_launch_chunk(items + i, 1, M, st);
            if (e != hipSuccess) return e;
        }
        return hipSuccess;
    }
    size_t lds = 0;
    int bb = 0;
    for (int i = 0; i < count; ++i) {
        const qail_w4a16_item& s = items[i];
        D4Item& t = a.it[i];
        const int quads = (s.d.N + 3) / 4;
        t.qw = s.qweight; t.sc = s.scales; t.zr = s.zeros; t.x = s.x; t.y = s.y;
        t.N = s.d.N; t.K = s.d.K; t.g = s.d.group_size;
        t.block_begin = bb;
        t.quads_base = quads / nb[i];
        t.quads_rem = quads % nb[i];
        for (int b = bb; b < bb + nb[i] && b < kD4MaxBlocks; ++b) a.item_of_block[b / 8] |= (uint32_t)i << (4 * (b % 8));
        bb += nb[i];
        if (d4_lds_bytes(s.d) > lds) lds = d4_lds_bytes(s.d);
    }
    for (int i = count; i < kD4MaxItems; ++i) a.it[i] = a.it[count - 1];
    a.M = M;
    hipLaunchKernelGGL(w4a16_decode4_kernel, dim3(bb), dim3(kD4Threads), lds, st, a);
    return hipGetLastError();
}

}  // namespace

bool decode4_supports(const qail_wdesc& d, int M) {
    const int g = d.group_size;
    // a chunk of 512 k holds 1, 2, 4 or 8 whole groups, or a group a power-of-two number of chunks
    const bool groups_ok = g == 64 || g == 128 || g == 256 || (g % kD4ChunkK == 0 && (g & (g - 1)) == 0);
    return M >= 2 && M <= 4 && d.N % 4 == 0 && d.K % 32 == 0 && d.K <= kD4MaxChunks * kD4ChunkK && groups_ok &&
           (unsigned long long)d.N * d.K / 2 < 0x80000000ull;  // 32-bit byte offsets in the kernel
}

hipError_t launch_w4a16_decode4(const qail_w4a16_item* items, int count, int M, hipStream_t st) {
    for (int i0 = 0; i0 < count; i0 += kD4MaxItems) {
        const int c = (count - i0 < kD4MaxItems) ? count - i0 : kD4MaxItems;
        const hipError_t e = d4_launch_chunk(items + i0, c, M, st);
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

}  // namespace qail
