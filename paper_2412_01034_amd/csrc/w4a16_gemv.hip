// W4A16 linear for M = 1 (decode): y[n] = sum_k x[k] * (q[n,k] - z[n,k/g]) * s[n,k/g].
//
// Appendix "Analysis": the decode stage is memory-bound, its time is the time to
// stream the packed weights.  The kernel is organised around that stream:
//
//   * a lane fetches 16 bytes (32 codes) of a row per load, a wave covers 2048
//     consecutive k of one row per load instruction, rows are contiguous, so every
//     wave-wide load is one 1 KB burst;
//   * every wave keeps several rows of loads in flight (a register pipeline), and a
//     block works on rows of ONE linear only, so the activations are staged in LDS
//     once per block and there is no barrier inside the stream;
//   * the multiply-adds run on the matrix cores (see stream_rows), so the vector ALU only
//     expands nibbles.  With
//
//       sum_k x_k (q_k - z) s  =  s * ( sum_k x_k (q_k + 1024)  -  1024 sum_k x_k  -  z sum_k x_k )
//
//     (q_k + 1024) as fp16 is the bit pattern 0x6400 | q_k, and 0x6400 | (q_k << 4) is
//     16 q_k + 1024, so one AND-OR turns two nibbles of a packed word into an fp16 pair at
//     either of two bit positions; the activations that meet the shifted codes are staged
//     divided by 16.  The sums of x over a lane's 32-k chunk are computed once per wave; a
//     chunk never straddles a group because group_size is a multiple of 32.
//
// One launch serves a list of independent linears: the blocks of the grid are
// divided among the linears in proportion to their bytes, so a decoder layer's
// four GEMVs ramp up once and finish together.
#include <string.h>

#include "qail_internal.h"

namespace qail {

namespace {

constexpr int kGemvMaxItems = 16;
constexpr int kGemvWaves = 8;                     // waves per block (two blocks share a CU)
constexpr int kGemvThreads = kGemvWaves * kWave;  // 512
constexpr int kChunkK = 32;                       // k per lane per load (16 bytes of codes)
constexpr int kWaveK = kWave * kChunkK;           // 2048 k per wave-wide load
constexpr int kGemvMaxChunks = 6;                 // K <= 12288 (more chunks would spill registers)
constexpr int kGemvMaxK = kGemvMaxChunks * kWaveK;
constexpr int kGemvMaxBlocks = 4096;              // blocks of a launch that serves more than one item

// 64 bytes, so that a block fetches everything it needs to know with one scalar load.
struct GemvItem {
    const uint32_t* qw;
    const uint16_t* sc;
    const uint32_t* zr;
    const uint16_t* x;
    uint16_t* y;
    int N, K, g;
    int block_begin;  // first block of the grid that works on this item
    int rows_base;    // block b of the item owns rows_base rows, one more if b < rows_rem,
    int rows_rem;     // in the order of the blocks
};

struct GemvArgs {
    GemvItem it[kGemvMaxItems];
    uint32_t item_of_block[kGemvMaxBlocks / 8];  // 4 bits per block; blocks past the table work on item 0
};

// Low-rank adapter of an item (Sec. 5.1: rank-32 adapters beside the 4-bit backbone):
// y[n] += scaling * sum_j t[j] * B[n][j], with t = A x computed beforehand.
struct GemvLora {
    const uint16_t* B;   // bf16 [N][r]
    const float* t;      // fp32 [r]
    int r;               // multiple of 8
    float scaling;
};

struct GemvLoraArgs {
    GemvLora l[kGemvMaxItems];
};

typedef __attribute__((ext_vector_type(8))) _Float16 f16x8_t;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4_t;

// Linears that depend on each other in one launch (see w4a16_chain_kernel).  Every block works on
// every item in turn; between two items all blocks meet through counters in the workspace.
constexpr int kChainMaxItems = 32;   // items per launch (their records travel in the kernel arguments)
constexpr int kChainFlagBase = 64;   // workspace words: [0] status, [16 + i] arrivals at item i, [64 + b] flag of block b
constexpr int kChainMaxPolls = 1 << 16;   // a block gives up waiting after this many looks at its flag

struct ChainCtx {
    const uint32_t* flag;   // this block's flag: holds the number of items every block has finished
    uint32_t need;          // value the flag must reach before this item's x may be read; 0: nothing to wait for
    uint32_t* status;       // one word of the workspace: set to 1 by a block that gave up waiting
};

template <int kCtrl>
__device__ __forceinline__ float dpp_add(float v) {
    const int moved = __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), kCtrl, 0xF, 0xF, true);
    return v + __builtin_bit_cast(float, moved);
}

template <int kCtrl>
__device__ __forceinline__ float dpp_max(float v) {
    const int moved = __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), kCtrl, 0xF, 0xF, true);
    return fmaxf(v, __builtin_bit_cast(float, moved));
}

// Sum over the 64 lanes; the result is wave-uniform.
__device__ __forceinline__ float wave_sum(float v) {
    v = dpp_add<0xB1>(v);   // quad_perm [1,0,3,2]
    v = dpp_add<0x4E>(v);   // quad_perm [2,3,0,1]
    v = dpp_add<0x141>(v);  // row_half_mirror
    v = dpp_add<0x140>(v);  // row_mirror: every lane of a 16-lane row holds the row sum
    const int vi = __builtin_bit_cast(int, v);
    return __builtin_bit_cast(float, __builtin_amdgcn_readlane(vi, 0)) +
           __builtin_bit_cast(float, __builtin_amdgcn_readlane(vi, 16)) +
           (__builtin_bit_cast(float, __builtin_amdgcn_readlane(vi, 32)) +
            __builtin_bit_cast(float, __builtin_amdgcn_readlane(vi, 48)));
}

// A lane owns 32 * kSub consecutive k of every wave-wide unit of a row (kSub = 2 whenever
// the group size and K are multiples of 64, else 1): its codes are kSub 16-byte loads, and
// everything that exists once per lane and unit (scale, zero-point, the constants below, the
// pick of the MFMA diagonal) is shared by 64 instead of 32 codes.
//
// LDS map of a block (uint4 units), nu = ceil(K / (2048 * kSub)) units per row:
//   [0, nu*kSub*256)   staged activations: word j of lane L in unit c at (c*4*kSub + j)*64 + L
//   then nu*64 float4  per-unit constants of lane L's unit c at c*64 + L:
//                      (1024 * sum of the staged values, sum of x * 2^-e, 2^e, unused)
// Lane L of a wave owns, in unit c, the 32*kSub k starting at (c*64 + L)*32*kSub.  Its staged
// word j holds those k's 8j..8j+7 as fp16 in the order x0,x4 | x1/16,x5/16 | x2,x6 | x3/16,x7/16
// (all times 2^-e), matching the four registers the weight nibbles are expanded into.
// Everything past K is zero.

// Stages the activations of one item (whole block; one barrier).
//
// x is bf16; the matrix cores take fp16 here because fp16 has room for a 4-bit code at two
// mantissa positions (see stream_rows).  Every bf16 significand fits fp16, the range does
// not, so each lane's stretch of a unit is scaled by the power of two that brings its largest
// magnitude into [2^14, 2^15); its dot product is multiplied back by 2^e in fp32.
// Elements more than 2^-28 below that maximum lose bits or vanish, which is far
// below the fp32 accumulation noise of the products.
template <int kMaxRuns, int kSub>
__device__ __forceinline__ void stage_x(const GemvItem& it, int nu, uint4* __restrict__ lds,
                                        const uint4 (&xr)[kMaxRuns]) {
    constexpr int kUnitRuns = kWave * 4 * kSub;  // runs of 8 k per unit
    const int K = it.K;
    float4* consts = reinterpret_cast<float4*>(lds + nu * kUnitRuns);
    const int runs = nu * kUnitRuns;
#pragma unroll
    for (int u = 0; u < kMaxRuns; ++u) {
        // run i = 8 consecutive k; 4 * kSub neighbouring threads hold the runs of one lane's stretch
        const int i = threadIdx.x + u * kGemvThreads;
        const uint32_t w[4] = {xr[u].x, xr[u].y, xr[u].z, xr[u].w};
        float f[8];
        float amax = 0.f;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            f[2 * e] = __builtin_bit_cast(float, w[e] << 16);
            f[2 * e + 1] = __builtin_bit_cast(float, w[e] & 0xFFFF0000u);
            amax = fmaxf(amax, fmaxf(fabsf(f[2 * e]), fabsf(f[2 * e + 1])));
        }
        amax = dpp_max<0xB1>(amax);  // quad_perm [1,0,3,2]
        amax = dpp_max<0x4E>(amax);  // quad_perm [2,3,0,1]
        if (kSub == 2) amax = dpp_max<0x141>(amax);  // row_half_mirror: the other quad of the 8
        // 2^-e with amax * 2^-e in [2^14, 2^15): exponent arithmetic on the bit pattern
        const int ex = (int)((__builtin_bit_cast(uint32_t, amax) >> 23) & 0xFF);  // biased exponent
        int down = (amax > 0.f) ? (ex - 141) : 0;                                 // 141 = 127 + 14
        down = max(-126, min(113, down));  // keeps both exponent fields valid
        const float pre = __builtin_bit_cast(float, (uint32_t)(127 - down) << 23);
        // the staged values as the matrix cores will see them (rounded to fp16), and their sums
        // over the stretch: even positions as they are, odd positions carry the factor 1/16
        const float pre16 = pre * 0.0625f;
        const bool live = i < K / 8;
        _Float16 h[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) h[e] = live ? (_Float16)(f[e] * ((e & 1) ? pre16 : pre)) : (_Float16)0.f;
        float se = ((float)h[0] + (float)h[4]) + ((float)h[2] + (float)h[6]);
        float so = ((float)h[1] + (float)h[5]) + ((float)h[3] + (float)h[7]);
        se = dpp_add<0xB1>(se);
        se = dpp_add<0x4E>(se);
        so = dpp_add<0xB1>(so);
        so = dpp_add<0x4E>(so);
        if (kSub == 2) {
            se = dpp_add<0x141>(se);
            so = dpp_add<0x141>(so);
        }
        if (i < runs) {
            auto pk = [](_Float16 lo, _Float16 hi) {
                typedef __attribute__((ext_vector_type(2))) _Float16 h2;
                const h2 v = {lo, hi};
                return __builtin_bit_cast(uint32_t, v);
            };
            const uint4 o = make_uint4(pk(h[0], h[4]), pk(h[1], h[5]), pk(h[2], h[6]), pk(h[3], h[7]));
            const int c = i / kUnitRuns, r = i % kUnitRuns;
            const int L = r / (4 * kSub), j = r % (4 * kSub);
            lds[(c * 4 * kSub + j) * kWave + L] = o;
            if (j == 0)
                consts[c * kWave + L] = make_float4(1024.f * (se + so), se + 16.f * so,
                                                    __builtin_bit_cast(float, (uint32_t)(127 + down) << 23), 0.f);
        }
    }
    __syncthreads();
}

// Rows [r0, r1) of one item, streamed by one wave.  The wave keeps NU * kSub * kPR wave-wide
// loads (1 KB each) in flight: a register slot is refilled with the same unit of a later
// row as soon as its codes have been consumed.  The first loads go out before the
// activations are staged, so the two latencies overlap.
//
// The multiply-adds run on the matrix cores.  v_mfma_f32_4x4x4_16b_f16 computes 16
// independent 4x4x4 products; lane l = 4b + j supplies row j of A and column j of B of
// block b (4 values each) and receives column j of D.  D[j][j], register j of lane l, is
// therefore the dot product of the lane's own four A values with its own four B values:
// eight such instructions, chained through the accumulator, give every lane the dot
// product of its 32 codes with the 32 activations at the same k.  The other entries of D
// are ignored.  The vector ALU only expands nibbles: 5 operations per 8 codes.
//
// kChain: the item's activations may have been written by the previous item of the same launch
// (by other blocks, on other XCDs).  The order then is: a first look at the previous item's
// counters, the first ring of weight loads (they depend on nothing), the wait, and only then
// the loads of x, which carry the agent scope so that they see what the other blocks released.
// Vector loads return in order, so the first look (issued before the ring) is the one poll whose
// answer arrives while the ring is still in flight; later polls queue behind the ring.
template <int NU, int kPR, int kSub, bool kChain>
__device__ __forceinline__ void stream_rows(const GemvItem& it, const GemvLora* lo, const float4* lora_t,
                                            int rbase, int nrows, int lane,
                                            uint4* __restrict__ xlds, int wave, const ChainCtx& cc) {
    typedef __attribute__((ext_vector_type(4))) _Float16 f16x4_t;
    const int K = it.K, g = it.g;
    const int G = K / g, zwords = (G + 7) / 8, kw = K / 8;

    constexpr int kLaneK = kChunkK * kSub;  // k per lane and unit
    constexpr int kUnitK = kWave * kLaneK;  // k per wave-wide unit
    constexpr int kMaxRuns = (NU * (kUnitK / 8) + kGemvThreads - 1) / kGemvThreads;
    uint4 xr[kMaxRuns];
    uint32_t seen = 0;
    if (!kChain) {
        // x first: it is needed first and loads return in order
#pragma unroll
        for (int u = 0; u < kMaxRuns; ++u) {
            const int i = threadIdx.x + u * kGemvThreads;
            xr[u] = (i < K / 8) ? reinterpret_cast<const uint4*>(it.x)[i] : make_uint4(0, 0, 0, 0);
        }
    } else if (cc.need) {
        seen = __hip_atomic_load(cc.flag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    __builtin_amdgcn_sched_barrier(0);  // the scheduler must not move these loads behind the weights

    // Per-unit constants of this lane.  Only the last unit of a row can run past K (a lane's
    // stretch lies entirely inside or outside: K is a multiple of its length); there the lane
    // reads the start of the row instead (valid data) and meets zeros in x.
    const bool tail_out = (NU - 1) * kUnitK + lane * kLaneK >= K;
    int goff[NU];
#pragma unroll
    for (int c = 0; c < NU; ++c) {
        const int kc = c * kUnitK + lane * kLaneK;
        goff[c] = ((c == NU - 1 && tail_out) ? 0 : kc) / g;
    }
    const int lane_b = lane * (kLaneK / 2);  // byte offset of the lane's codes within unit 0
    const int last_b = tail_out ? 0 : (NU - 1) * (kUnitK / 2) + lane_b;

    uint4 q[kPR][NU][kSub];
    uint16_t sh[kPR][NU];  // fp16 bits, kept as loaded: a widening at the load would force a wait there
    uint32_t zw[kPR][NU];

    // Loads go through buffer descriptors (one per tensor, in scalar registers): the address
    // is descriptor base + scalar row offset + a 32-bit lane offset that never changes, so a
    // load costs one scalar multiply and no vector arithmetic.  The host checks that each
    // tensor is shorter than 4 GB.
    const __amdgpu_buffer_rsrc_t rq = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint32_t*>(it.qw), 0, it.N * kw * 4, 0x00020000);
    const __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t*>(it.sc), 0, it.N * G * 2, 0x00020000);
    const __amdgpu_buffer_rsrc_t rz = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint32_t*>(it.zr), 0, it.N * zwords * 4, 0x00020000);
    int soff[NU], zoff[NU];
#pragma unroll
    for (int c = 0; c < NU; ++c) {
        soff[c] = goff[c] * 2;
        zoff[c] = (goff[c] >> 3) * 4;
    }
    auto issue = [&](int p, int c, int row) {
        const int qb = (c == NU - 1) ? last_b : c * (kUnitK / 2) + lane_b;
#pragma unroll
        for (int h = 0; h < kSub; ++h) {
            const u32x4_t v = __builtin_amdgcn_raw_buffer_load_b128(rq, qb + 16 * h, row * (kw * 4), 0);
            q[p][c][h] = make_uint4(v[0], v[1], v[2], v[3]);
        }
        sh[p][c] = __builtin_amdgcn_raw_buffer_load_b16(rs, soff[c], row * (G * 2), 0);
        zw[p][c] = __builtin_amdgcn_raw_buffer_load_b32(rz, zoff[c], row * (zwords * 4), 0);
    };

    // Every load below is issued unconditionally (rows past the end are clamped to the last
    // row and their results dropped), so that the number of loads in flight at each point is
    // known at compile time and the waits can be exact.
    const int ilast = max(nrows - 1, 0);
#pragma unroll
    for (int p = 0; p < kPR; ++p)
#pragma unroll
        for (int c = 0; c < NU; ++c) {
            issue(p, c, min(rbase + min(p, ilast) * kGemvWaves, it.N - 1));
            __builtin_amdgcn_sched_barrier(0);  // program order = consumption order, see above
        }

    if (kChain) {
        if (cc.need && wave == 0) {
            // bounded: a block that never sees the others arrive (the grid was not resident as a
            // whole) says so in the status word and goes on, so every wave ends
            int polls = 0;
            while (__builtin_amdgcn_readfirstlane(seen) < cc.need) {
                if (++polls > kChainMaxPolls) {
                    if (lane == 0) __hip_atomic_store(cc.status, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    break;
                }
                __builtin_amdgcn_s_sleep(8);
                seen = __hip_atomic_load(cc.flag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
        }
        // every wave of the block is through with the previous item's staged x, and the previous
        // item's outputs are visible at agent scope
        __syncthreads();
        const __amdgpu_buffer_rsrc_t rx = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t*>(it.x), 0, K * 2, 0x00020000);
#pragma unroll
        for (int u = 0; u < kMaxRuns; ++u) {
            const int i = threadIdx.x + u * kGemvThreads;
            // aux 16 = sc1: agent scope, the load is served from where the other XCDs' released stores are
            // visible; past the end of x the descriptor returns zeros
            const u32x4_t v = __builtin_amdgcn_raw_buffer_load_b128(rx, i * 16, 0, 16);
            xr[u] = make_uint4(v[0], v[1], v[2], v[3]);
        }
    }
    stage_x<kMaxRuns, kSub>(it, NU, xlds, xr);

    // Per unit, for the lane's own stretch (written by the staging):
    //   xoff = 1024 * (sum of the staged values): what the fp16 offsets add to the MFMA result
    //   xsum = sum of x * 2^-e
    //   post = 2^e
    // kept in registers for short rows, re-read from LDS per row for long ones
    constexpr bool kParked = NU > 4;
    const float4* parked = reinterpret_cast<const float4*>(xlds + NU * kSub * 4 * kWave);
    float xoff[NU], xsum[NU], post[NU];
    if (!kParked) {
#pragma unroll
        for (int c = 0; c < NU; ++c) {
            const float4 t = parked[c * kWave + lane];
            xoff[c] = t.x; xsum[c] = t.y; post[c] = t.z;
        }
    }
    if (nrows <= 0) return;
    uint32_t magic = 0x64006400u;   // fp16 pair (1024, 1024); held in a vector register so that
    asm volatile("" : "+v"(magic)); // the AND-OR needs only one scalar operand

    // Results stay in registers (the wave's i-th row in lane i; the launcher gives a wave at most 64
    // rows) and are stored once at the end: a store between the loads would break the
    // in-order completion that exact load waits rely on.
    float ykeep = 0.f;

    const bool odd = lane & 1, hi = lane & 2;

    // The arithmetic of the wave's i-th row, whose codes sit in slot p.  With `next` >= 0 every
    // chunk's registers are refilled with the same chunk of row `next` as soon as they have
    // been used, so the number of loads in flight stays level instead of dipping once per row.
    auto consume = [&](int p, int i, int next) {
        float acc = 0.f;
        // x is the same for every row, but holding all of it in registers costs 16 per
        // chunk.  It is re-read from LDS per row, one chunk ahead of the arithmetic; the
        // empty asm ties each chunk's reads to the previous chunk's result so that the
        // compiler can neither hoist the reads out of the row loop nor bunch them up.
        int xo = lane;
        asm volatile("" : "+v"(xo));
        constexpr int kXB = kParked ? 1 : 2;  // long rows: no read-ahead, to stay within the registers
        uint4 xv[kXB][4];
        if (kXB == 2) {
#pragma unroll
            for (int j = 0; j < 4; ++j) xv[0][j] = xlds[j * kWave + xo];
        }
#pragma unroll
        for (int c = 0; c < NU; ++c) {
            f32x4_t d0 = {0.f, 0.f, 0.f, 0.f};  // one chain: the expansion between two MFMAs covers their latency
#pragma unroll
            for (int h = 0; h < kSub; ++h) {
                const int sc = c * kSub + h;  // 32-k piece of the row, in k order
                if (kXB == 2 && sc + 1 < NU * kSub) {
#pragma unroll
                    for (int j = 0; j < 4; ++j) xv[(sc + 1) & 1][j] = xlds[((sc + 1) * 4 + j) * kWave + xo];
                }
                if (kXB == 1) {
#pragma unroll
                    for (int j = 0; j < 4; ++j) xv[0][j] = xlds[(sc * 4 + j) * kWave + xo];
                }
                const uint32_t w[4] = {q[p][c][h].x, q[p][c][h].y, q[p][c][h].z, q[p][c][h].w};
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    // codes 0,4 | 16*codes 1,5 | codes 2,6 | 16*codes 3,7, each plus 1024, as fp16
                    const uint32_t w8 = w[j] >> 8;
                    const uint2 a01 = make_uint2((w[j] & 0x000F000Fu) | magic, (w[j] & 0x00F000F0u) | magic);
                    const uint2 a23 = make_uint2((w8 & 0x000F000Fu) | magic, (w8 & 0x00F000F0u) | magic);
                    const uint4 xj = xv[sc & (kXB - 1)][j];
                    d0 = __builtin_amdgcn_mfma_f32_4x4x4f16(__builtin_bit_cast(f16x4_t, a01),
                                                            __builtin_bit_cast(f16x4_t, make_uint2(xj.x, xj.y)), d0, 0, 0, 0);
                    d0 = __builtin_amdgcn_mfma_f32_4x4x4f16(__builtin_bit_cast(f16x4_t, a23),
                                                            __builtin_bit_cast(f16x4_t, make_uint2(xj.z, xj.w)), d0, 0, 0, 0);
                }
            }
            // D[j][j] is register j = lane % 4
            const float e0 = odd ? d0[1] : d0[0], e1 = odd ? d0[3] : d0[2];
            const float dsel = hi ? e1 : e0;
            float cxoff, cxsum, cpost;
            if (kParked) {
                const float4 t = parked[c * kWave + xo];
                cxoff = t.x; cxsum = t.y; cpost = t.z;
            } else {
                cxoff = xoff[c]; cxsum = xsum[c]; cpost = post[c];
            }
            const float s = (float)__builtin_bit_cast(_Float16, sh[p][c]) * cpost;
            const float z = (float)((zw[p][c] >> (4 * (goff[c] & 7))) & 0xFu);
            // sum_k x_k (q_k - z) = (D - xoff) - z * xsum
            acc = fmaf(s, dsel - fmaf(z, cxsum, cxoff), acc);
            asm volatile("" : "+v"(acc), "+v"(xo));
            if (next >= 0) {
                issue(p, c, next);
                __builtin_amdgcn_sched_barrier(0);  // program order = consumption order
            }
        }
        const float v = wave_sum(acc);
        ykeep = (lane == i) ? v : ykeep;
    };

    // main part: every consumed slot is refilled with the row kPR further on (clamped in
    // the last trip); then the last kPR rows are drained without further loads
    int r = 0;
    for (; r + kPR < nrows; r += kPR) {
#pragma unroll
        for (int p = 0; p < kPR; ++p)
            consume(p, r + p, min(rbase + min(r + p + kPR, ilast) * kGemvWaves, it.N - 1));
    }
#pragma unroll
    for (int p = 0; p < kPR; ++p)
        if (r + p < nrows) consume(p, r + p, -1);
    if (lane < nrows) {
        const int row = rbase + lane * kGemvWaves;
        float v = ykeep;
        if (lo) {
            // The adapter's up-projection joins before the single rounding of the output.  All of
            // the row's B is requested at once (up to 8 loads in flight); t was staged in LDS
            // when the kernel started.
            const uint4* brow = reinterpret_cast<const uint4*>(lo->B + (size_t)row * lo->r);
            uint4 bv[8];
#pragma unroll
            for (int c = 0; c < 8; ++c) bv[c] = (c * 8 < lo->r) ? brow[c] : make_uint4(0, 0, 0, 0);
            float dot = 0.f;
#pragma unroll
            for (int c = 0; c < 8; ++c) {
                if (c * 8 < lo->r) {
                    const float4 t0 = lora_t[2 * c], t1 = lora_t[2 * c + 1];
                    const uint32_t w[4] = {bv[c].x, bv[c].y, bv[c].z, bv[c].w};
                    const float tv[8] = {t0.x, t0.y, t0.z, t0.w, t1.x, t1.y, t1.z, t1.w};
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        dot = fmaf(tv[2 * e], __builtin_bit_cast(float, w[e] << 16), dot);
                        dot = fmaf(tv[2 * e + 1], __builtin_bit_cast(float, w[e] & 0xFFFF0000u), dot);
                    }
                }
            }
            v = fmaf(lo->scaling, dot, v);
        }
        if (kChain) {
            // written through to where the other XCDs' agent-scope loads look: the next item's blocks
            // may run anywhere on the chip
            __hip_atomic_store(it.y + row, f32_to_bf16_rne(v), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        } else {
            it.y[row] = f32_to_bf16_rne(v);
        }
    }
}

template <int kUnits, bool kLora>
__device__ __forceinline__ void gemv_body(const GemvArgs& args, const GemvLoraArgs& lora) {
    extern __shared__ uint4 lds[];
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);  // wave-uniform: row
    const int lane = threadIdx.x % kWave;                                  // addresses stay scalar

    // two dependent scalar loads and no division between the start of the block and its first
    // weight load: the block's item from a 4-bit table, then the item's 64-byte record
    int idx = 0;
    if (blockIdx.x < (unsigned)kGemvMaxBlocks) idx = (args.item_of_block[blockIdx.x / 8] >> (4 * (blockIdx.x % 8))) & 15;
    idx = __builtin_amdgcn_readfirstlane(idx);
    const GemvItem it = args.it[idx];
    const GemvLora* lo = kLora ? &lora.l[idx] : nullptr;
    const int K = it.K, N = it.N;
    // 64 k per lane and unit where the layout allows it, else 32
    const bool wide = it.g % (2 * kChunkK) == 0 && K % (2 * kChunkK) == 0;
    const int nu = wide ? (K + 2 * kWaveK - 1) / (2 * kWaveK) : (K + kWaveK - 1) / kWaveK;
    // the adapter's down-projection t (at most 64 floats) sits behind the staged activations; the
    // barrier inside the staging makes it visible
    float4* lora_t = reinterpret_cast<float4*>(lds + nu * kWave * (wide ? 9 : 5));
    if (kLora && (int)threadIdx.x < 64)
        reinterpret_cast<float*>(lora_t)[threadIdx.x] = (int)threadIdx.x < lo->r ? lo->t[threadIdx.x] : 0.f;

    // this block's slab of rows, then this wave's share of the slab
    const int b = (int)blockIdx.x - it.block_begin;
    const int s0 = b * it.rows_base + min(b, it.rows_rem);
    const int s1 = s0 + it.rows_base + (b < it.rows_rem ? 1 : 0);
    // Rows are dealt to the waves of the block in turn, so that at any moment the block's
    // waves read adjacent rows: one contiguous stretch of memory per block.
    const int r0 = s0 + wave;
    const int r1 = max(0, (s1 - s0 - wave + kGemvWaves - 1) / kGemvWaves);  // number of rows

    // about kUnits wave-wide loads (1 KB each) in flight per wave
    if (wide) {
        switch (nu) {
            case 1: stream_rows<1, kUnits / 2, 2, false>(it, lo, lora_t, r0, r1, lane, lds, wave, ChainCtx{}); break;
            case 2: stream_rows<2, kUnits / 4, 2, false>(it, lo, lora_t, r0, r1, lane, lds, wave, ChainCtx{}); break;
            default: stream_rows<3, 1, 2, false>(it, lo, lora_t, r0, r1, lane, lds, wave, ChainCtx{}); break;
        }
        return;
    }
    switch (nu) {
        case 1: stream_rows<1, kUnits, 1, false>(it, lo, lora_t, r0, r1, lane, lds, wave, ChainCtx{}); break;
        case 2: stream_rows<2, kUnits / 2, 1, false>(it, lo, lora_t, r0, r1, lane, lds, wave, ChainCtx{}); break;
        case 3: stream_rows<3, kUnits / 3, 1, false>(it, lo, lora_t, r0, r1, lane, lds, wave, ChainCtx{}); break;
        case 4: stream_rows<4, kUnits / 4, 1, false>(it, lo, lora_t, r0, r1, lane, lds, wave, ChainCtx{}); break;
        case 5: stream_rows<5, 1, 1, false>(it, lo, lora_t, r0, r1, lane, lds, wave, ChainCtx{}); break;
        default: stream_rows<6, 1, 1, false>(it, lo, lora_t, r0, r1, lane, lds, wave, ChainCtx{}); break;
    }
}

template <int kUnits>
__global__ __launch_bounds__(kGemvThreads) void w4a16_gemv_kernel(const GemvArgs args) {
    gemv_body<kUnits, false>(args, GemvLoraArgs{});
}

// The same stream with the adapters' up-projection in the final store.
template <int kUnits>
__global__ __launch_bounds__(kGemvThreads) void w4a16_gemv_lora_kernel(const GemvArgs args, const GemvLoraArgs lora) {
    gemv_body<kUnits, true>(args, lora);
}

// Linears that depend on each other, in ONE launch.  A decoder layer's linears cannot share a
// launch as independent items: each needs what the one before it produced.  Launched one by one
// they each pay a ramp and a tail during which HBM idles.  Here the grid is resident as a whole
// (one or two blocks per CU), every block takes its slab of rows of item 0, then of item 1, and
// so on, and before it reads item i + 1's activations it waits until every block has written
// its rows of item i.  The weights do not depend on the activations, so a wave asks for its
// first rows of item i + 1 before it waits: while the blocks meet, HBM keeps delivering.
//
// Meeting point, in the workspace (cleared by a small kernel in front): one arrival counter per
// item and one flag per block.  A block whose waves' stores of item i have been acknowledged
// adds one to the item's counter; the block that finds it was the last one writes i + 1 into
// every block's flag.  A waiting block looks only at its own flag: 512 blocks spinning on the
// counters themselves delay the very additions they wait for (measured: 26 us per item).
struct ChainArgs {
    GemvItem it[kChainMaxItems];
    uint32_t* ws;
    int count;
};

__global__ __launch_bounds__(256) void w4a16_chain_clear_kernel(uint32_t* ws, int words) {
    for (int i = threadIdx.x; i < words; i += 256) ws[i] = 0u;
}

template <int kUnits>
__global__ __launch_bounds__(kGemvThreads, 4) void w4a16_chain_kernel(const ChainArgs args) {
    extern __shared__ uint4 lds[];
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
    const int lane0 = threadIdx.x % kWave;
    const int P = (int)gridDim.x, b = (int)blockIdx.x;
    ChainCtx cc;
    cc.status = args.ws;
    cc.flag = args.ws + kChainFlagBase + b;
    for (int i = 0; i < args.count; ++i) {
        const GemvItem it = args.it[i];
        cc.need = (uint32_t)i;   // items that must be complete before this one's x is read
        // the lane index is laundered per item: what the compiler derives from it (offsets, masks,
        // picks) would otherwise be hoisted out of this loop for all nine shapes of the stream at
        // once and held in registers across it
        int lane = lane0;
        asm volatile("" : "+v"(lane));
        const int K = it.K;
        const bool wide = it.g % (2 * kChunkK) == 0 && K % (2 * kChunkK) == 0;
        const int nu = wide ? (K + 2 * kWaveK - 1) / (2 * kWaveK) : (K + kWaveK - 1) / kWaveK;
        const int s0 = b * it.rows_base + min(b, it.rows_rem);
        const int s1 = s0 + it.rows_base + (b < it.rows_rem ? 1 : 0);
        const int r0 = s0 + wave;
        const int r1 = max(0, (s1 - s0 - wave + kGemvWaves - 1) / kGemvWaves);
        if (wide) {
            switch (nu) {
                case 1: stream_rows<1, kUnits / 2, 2, true>(it, nullptr, nullptr, r0, r1, lane, lds, wave, cc); break;
                case 2: stream_rows<2, kUnits / 4, 2, true>(it, nullptr, nullptr, r0, r1, lane, lds, wave, cc); break;
                default: stream_rows<3, 1, 2, true>(it, nullptr, nullptr, r0, r1, lane, lds, wave, cc); break;
            }
        } else {
            switch (nu) {
                case 1: stream_rows<1, kUnits, 1, true>(it, nullptr, nullptr, r0, r1, lane, lds, wave, cc); break;
                case 2: stream_rows<2, kUnits / 2, 1, true>(it, nullptr, nullptr, r0, r1, lane, lds, wave, cc); break;
                case 3: stream_rows<3, kUnits / 3, 1, true>(it, nullptr, nullptr, r0, r1, lane, lds, wave, cc); break;
                case 4: stream_rows<4, kUnits / 4, 1, true>(it, nullptr, nullptr, r0, r1, lane, lds, wave, cc); break;
                case 5: stream_rows<5, 1, 1, true>(it, nullptr, nullptr, r0, r1, lane, lds, wave, cc); break;
                default: stream_rows<6, 1, 1, true>(it, nullptr, nullptr, r0, r1, lane, lds, wave, cc); break;
            }
        }
        if (i + 1 < args.count) {
            // This wave's rows of item i went out as agent-scope stores (written through the XCD's L2),
            // so they are visible chip-wide once they are acknowledged: the wave waits for that, the
            // block's waves meet, and one wave reports.  (A release fence at agent scope would
            // do, but it writes back the whole L2 each time: measured 70 us per item.)
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
            __builtin_amdgcn_s_waitcnt(0x0070);   // vmcnt(0) lgkmcnt(0)
            __syncthreads();
            if (wave == 0) {
                uint32_t before = 0;
                if (lane == 0)
                    before = __hip_atomic_fetch_add(args.ws + 16 + i, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                before = __builtin_amdgcn_readfirstlane(before);
                if (before == (uint32_t)(P - 1)) {
                    // the last block to arrive: every block's outputs of item i are visible; tell them all
                    for (int j = lane; j < P; j += kWave)
                        __hip_atomic_store(args.ws + kChainFlagBase + j, (uint32_t)(i + 1), __ATOMIC_RELAXED,
                                           __HIP_MEMORY_SCOPE_AGENT);
                }
            }
        }
    }
}

size_t item_bytes(const qail_wdesc& d) {
    const size_t G = (size_t)d.K / d.group_size;
    return (size_t)d.N * (d.K / 2 + G * 2 + ((G + 7) / 8) * 4);
}

hipError_t launch_chunk(const qail_w4a16_item* items, const GemvLora* loras, int count, hipStream_t st) {
    GemvArgs a;
    memset(a.item_of_block, 0, sizeof(a.item_of_block));
    // Two blocks of eight waves per CU when that leaves every wave three rows or more, else one:
    // the hardware then hands a CU its second helping when the first is done, which evens out the
    // finish (measured against one block of sixteen waves per CU: the layer 3 % faster, the large
    // linears alone 9 %; with fewer rows the extra blocks' fixed cost outweighs it).
    long long rows_total = 0;
    for (int i = 0; i < count; ++i) rows_total += items[i].d.N;
    int grid = device_cu_count();
    if (rows_total >= 2LL * grid * kGemvWaves * 3) grid *= 2;
    if (grid < count) grid = count;
    // blocks per item in proportion to its bytes (largest remainder), at least one each
    double total = 0;
    for (int i = 0; i < count; ++i) total += (double)item_bytes(items[i].d);
    int nb[kGemvMaxItems];
    double frac[kGemvMaxItems];
    int used = 0;
    for (int i = 0; i < count; ++i) {
        const double share = (double)item_bytes(items[i].d) / total * grid;
        nb[i] = (int)share;
        if (nb[i] < 1) nb[i] = 1;
        // a wave keeps its results in one register: at most 64 rows per wave
        const int need = (items[i].d.N + kGemvWaves * kWave - 1) / (kGemvWaves * kWave);
        if (nb[i] < need) nb[i] = need;
        // no more blocks than slabs of one row per wave
        const int cap = (items[i].d.N + kGemvWaves - 1) / kGemvWaves;
        if (nb[i] > cap) nb[i] = cap;
        frac[i] = share - (int)share;
        used += nb[i];
    }
    while (used < grid) {
        int best = -1;
        for (int i = 0; i < count; ++i) {
            const int cap = (items[i].d.N + kGemvWaves - 1) / kGemvWaves;
            if (nb[i] < cap && (best < 0 || frac[i] > frac[best])) best = i;
        }
        if (best < 0) break;
        ++nb[best];
        frac[best] = -1.0;
        ++used;
    }
    if (count > 1 && used > kGemvMaxBlocks) {
        // the block-to-item table is too short: one launch per item (a lone item needs no table)
        for (int i = 0; i < count; ++i) {
            const hipError_t e = launch_chunk(items + i, loras ? loras + i : nullptr, 1, st);
            if (e != hipSuccess) return e;
        }
        return hipSuccess;
    }
    size_t lds = 0;
    int bb = 0;
    for (int i = 0; i < count; ++i) {
        const qail_w4a16_item& s = items[i];
        GemvItem& t = a.it[i];
        t.qw = s.qweight; t.sc = s.scales; t.zr = s.zeros; t.x = s.x; t.y = s.y;
        t.N = s.d.N; t.K = s.d.K; t.g = s.d.group_size;
        t.block_begin = bb;
        t.rows_base = s.d.N / nb[i];
        t.rows_rem = s.d.N % nb[i];
        for (int b = bb; b < bb + nb[i] && b < kGemvMaxBlocks; ++b) a.item_of_block[b / 8] |= (uint32_t)i << (4 * (b % 8));
        bb += nb[i];
        // staged activations and per-unit constants, as laid out by the kernel
        const bool wide = s.d.group_size % (2 * kChunkK) == 0 && s.d.K % (2 * kChunkK) == 0;
        const int nu = wide ? (s.d.K + 2 * kWaveK - 1) / (2 * kWaveK) : (s.d.K + kWaveK - 1) / kWaveK;
        const size_t need_lds = (size_t)nu * kWave * (wide ? 9 : 5) * 16;
        if (need_lds > lds) lds = need_lds;
    }
    for (int i = count; i < kGemvMaxItems; ++i) a.it[i] = a.it[count - 1];
    if (loras) {
        GemvLoraArgs la;
        for (int i = 0; i < kGemvMaxItems; ++i) la.l[i] = loras[i < count ? i : count - 1];
        hipLaunchKernelGGL(w4a16_gemv_lora_kernel<8>, dim3(bb), dim3(kGemvThreads), lds + 256, st, a, la);
    } else {
        hipLaunchKernelGGL(w4a16_gemv_kernel<8>, dim3(bb), dim3(kGemvThreads), lds, st, a);
    }
    return hipGetLastError();
}

}  // namespace

bool gemv_supports(const qail_wdesc& d) {
    // the kernel addresses each tensor through a 32-bit byte offset (codes are the largest)
    return d.K % kChunkK == 0 && d.group_size % kChunkK == 0 && d.K <= kGemvMaxK &&
           (unsigned long long)d.N * d.K / 2 < 0x80000000ull;
}

hipError_t launch_w4a16_gemv(const qail_w4a16_item* items, int count, hipStream_t st) {
    for (int i0 = 0; i0 < count; i0 += kGemvMaxItems) {
        const int c = (count - i0 < kGemvMaxItems) ? count - i0 : kGemvMaxItems;
        const hipError_t e = launch_chunk(items + i0, nullptr, c, st);
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

// Status word, arrival counters of up to 32 items and one flag per block of the largest grid
// (two blocks per CU), in 4-byte words.
static int chain_ws_words() { return kChainFlagBase + 2 * device_cu_count(); }
size_t gemv_chain_workspace(int count) {
    (void)count;
    return ((size_t)chain_ws_words() * sizeof(uint32_t) + 255) / 256 * 256;
}

// Largest grid of the chain kernel that is resident as a whole on the current device with `lds`
// bytes of dynamic LDS per block: two blocks per CU if they fit, else one; 0 if none fits.
static int chain_grid(size_t lds) {
    int per_cu = 0;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, reinterpret_cast<const void*>(&w4a16_chain_kernel<8>),
                                                     kGemvThreads, lds) != hipSuccess)
        return 0;
    if (per_cu > 2) per_cu = 2;
    return per_cu * device_cu_count();
}

bool gemv_chain_supports(const qail_wdesc& d) {
    // every block takes a slab of every item, a wave keeps at most 64 rows' results
    return gemv_supports(d) && (long long)d.N <= 64LL * kGemvWaves * device_cu_count();
}

hipError_t launch_w4a16_chain(const qail_w4a16_item* items, int count, void* ws, hipStream_t st) {
    for (int i0 = 0; i0 < count; i0 += kChainMaxItems) {
        const int c = (count - i0 < kChainMaxItems) ? count - i0 : kChainMaxItems;
        size_t lds = 0;
        for (int i = 0; i < c; ++i) {
            const qail_wdesc& d = items[i0 + i].d;
            const bool wide = d.group_size % (2 * kChunkK) == 0 && d.K % (2 * kChunkK) == 0;
            const int nu = wide ? (d.K + 2 * kWaveK - 1) / (2 * kWaveK) : (d.K + kWaveK - 1) / kWaveK;
            const size_t need_lds = (size_t)nu * kWave * (wide ? 9 : 5) * 16;
            if (need_lds > lds) lds = need_lds;
        }
        int P = chain_grid(lds);
        if (P <= 0) return hipErrorLaunchOutOfResources;
        // two blocks per CU only when that leaves the shortest item a row per wave
        int nmin = items[i0].d.N;
        for (int i = 1; i < c; ++i) nmin = items[i0 + i].d.N < nmin ? items[i0 + i].d.N : nmin;
        if (P > device_cu_count() && nmin < P * kGemvWaves) P = device_cu_count();
        ChainArgs a;
        for (int i = 0; i < c; ++i) {
            const qail_w4a16_item& s = items[i0 + i];
            GemvItem& t = a.it[i];
            t.qw = s.qweight; t.sc = s.scales; t.zr = s.zeros; t.x = s.x; t.y = s.y;
            t.N = s.d.N; t.K = s.d.K; t.g = s.d.group_size;
            t.block_begin = 0;
            t.rows_base = s.d.N / P;
            t.rows_rem = s.d.N % P;
        }
        for (int i = c; i < kChainMaxItems; ++i) a.it[i] = a.it[c - 1];
        a.ws = static_cast<uint32_t*>(ws);
        a.count = c;
        // the status word survives from chunk to chunk; counters and flags are cleared for each launch
        hipLaunchKernelGGL(w4a16_chain_clear_kernel, dim3(1), dim3(256), 0, st, a.ws + (i0 == 0 ? 0 : 1),
                           chain_ws_words() - (i0 == 0 ? 0 : 1));
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
        hipLaunchKernelGGL(w4a16_chain_kernel<8>, dim3(P), dim3(kGemvThreads), lds, st, a);
        e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

// t: fp32 [count][r_max] as written by launch_lora_down for M = 1 (stride t_stride floats).
hipError_t launch_w4a16_gemv_lora(const qail_w4a16_item* items, const qail_lora* loras, const float* t,
                                  int t_stride, int count, hipStream_t st) {
    for (int i0 = 0; i0 < count; i0 += kGemvMaxItems) {
        const int c = (count - i0 < kGemvMaxItems) ? count - i0 : kGemvMaxItems;
        GemvLora gl[kGemvMaxItems];
        for (int i = 0; i < c; ++i) {
            const qail_lora& l = loras[i0 + i];
            gl[i] = GemvLora{l.B, t + (size_t)(i0 + i) * t_stride, l.r, l.scaling};
        }
        const hipError_t e = launch_chunk(items + i0, gl, c, st);
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

}  // namespace qail
