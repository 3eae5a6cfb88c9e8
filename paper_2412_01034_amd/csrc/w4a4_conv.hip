// W4A4 convolution as an implicit GEMM with exact int32 accumulation.
//
//   acc[(b,oh,ow)][n] = sum_{kh,kw,c} a[b][oh*s+kh-p][ow*s+kw-p][c] * w[n][kh][kw][c]
//
// Sec. 2.1 / Sec. 5.1: the driving policy's convolutions are compute-bound, so both
// GEMM operands are 4-bit integers.  CDNA4 has no 4-bit integer matrix
// instruction, so nibbles are widened to int8 in registers and fed to
// v_mfma_i32_32x32x32_i8 (int32 accumulate):
//   * unsigned activation codes:  w & 0x0F0F0F0F  and (w >> 4) & 0x0F0F0F0F
//     give the even and the odd codes of a word as bytes;
//   * signed weight codes are moved to the HIGH nibble of each byte,
//     (w << 4) & 0xF0F0F0F0 and w & 0xF0F0F0F0, which is the int8 value 16*code,
//     so no sign extension is needed; the accumulator is 16x the result and an
//     arithmetic shift by 4 restores it exactly.
// The two operands are permuted along k in the same way (even codes, then odd
// codes of each word), which leaves the sum unchanged.
//
// MFMA operand layout (32x32x32 int8, wave64): lane l supplies row (A) / column
// (B) l%32 and the 16 consecutive k starting at 16*(l/32); register r of its 16
// results is D[8*(r/4) + 4*(l/32) + r%4][l%32].  A = activations (rows m),
// B = weights (columns n).  The 16x16x64 form has the same operand volume per
// multiply-add but a wave issuing nothing else reaches only 0.6 of the matrix
// rate with it (2.7 against 4.5 POP/s over the chip, measured), the 32x32x32 form all of it.
//
// Tiling: a block of 4 waves (2 x 2) owns a BM x BN output tile and walks K in
// steps of 128 codes (16 packed words per row; K is ordered (kh, kw, c), so a step
// is a run of channels of one or two filter taps).  Nibbles stay packed in LDS
// (half the LDS traffic of int8); the load unit writes the tiles of the next two steps
// straight into a ring of three LDS slots, one barrier per step.
// Zero padding costs nothing: code 0 of the unsigned activations is the value 0.
#include "qail_internal.h"
#include <algorithm>
#include <cmath>

namespace qail {

namespace {

constexpr int kStepWords = 16;  // packed words per row per K step (128 codes)

struct ConvGeom {
    int B, H, W, Cin, Cout, KH, KW, stride, pad, OH, OW, M;
    // ceil(2^32 / d) for the four divisors of the tiled kernel's set-up (OH * OW, OW, words per
    // pixel, KW), valid when `fastdiv` is set: the host has checked that the high word of
    // x * magic is x / d for every x the kernel divides.
    uint32_t mg_ohow, mg_ow, mg_cw, mg_kw;
    int fastdiv;
};

// x / d as the high word of x * ceil(2^32 / d): with e = d * magic - 2^32 (0 <= e < d) the product
// is x / d + x e / (d 2^32), and its floor is floor(x / d) as long as x e < 2^32 (then the excess
// stays below 1 / d).  `ok` tells whether that holds for every x up to xmax; d = 1 has no 32-bit
// magic and is marked by 0.
inline uint32_t div_magic(uint32_t d, uint64_t xmax, bool& ok) {
    if (d == 0) ok = false;
    if (d < 2) return 0;
    const uint64_t mg = ((1ull << 32) + d - 1) / d;
    const uint64_t e = mg * d - (1ull << 32);
    if (e * xmax >= (1ull << 32)) ok = false;
    return (uint32_t)mg;
}
__device__ __forceinline__ int div_by(int x, int d, uint32_t magic, int fast) {
    return fast ? (magic ? (int)__umulhi((uint32_t)x, magic) : x) : x / d;
}

typedef __attribute__((ext_vector_type(4))) unsigned u32x4_t;

// Raw buffer descriptor over [p, p + bytes): loads past the end return 0 and stores past the
// end are dropped by the hardware, which turns every image-border, K-tail and tile-edge test
// into the choice of an offset.
__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void* p, uint32_t bytes) {
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(p), 0, bytes, 0x00020000);
}
constexpr uint32_t kOut = 0xFFFFFFF0u;  // an offset no buffer here reaches

// Where the results go.  Plain outputs: acc and / or y = fma(float(acc), scale, bias).
// Fused output (out_u4 != nullptr): the next layer's packed unsigned codes, see fused_code().
struct ConvOut {
    int32_t* acc;
    const float* scale;
    const float* bias;
    float* y;
    uint32_t* out_u4;
    const uint32_t* res_u4;
    const float* res_f32;
    float s_out, res_scale;
    float inv_s_out;  // 1 / s_out, correctly rounded (host division)
    int quick;        // s_out and its reciprocal are normal numbers: the quotient may be tried as a product first
};

// Up to kConvBatch independent convolutions share a launch: item i is the grid's plane z = i
// (its arguments are then at an offset known when the wave starts: no load depends on another);
// the x and y axes are as large as the largest item needs, the blocks outside an item's own tile
// grid leave at once.
constexpr int kConvBatch = 4;
struct ConvItem {
    ConvGeom gm;
    const uint32_t* a;
    const uint32_t* w;
    ConvOut out;
};
struct ConvBatch {
    ConvItem it[kConvBatch];
};

// One output element of the fused epilogue (Sec. 5.1: every activation tensor of the driving
// encoder is 4-bit with one step per tensor, so the consumer's step is known here).  Each
// line is one correctly rounded fp32 operation; contraction to fma is switched off because
// the code is decided by these roundings and must equal the reference bit for bit.
__device__ __forceinline__ float fused_value(int acc, float scale, float bias, float r) {
#pragma clang fp contract(off)
    float t = (float)acc * scale;
    t = t + bias;
    t = t + r;
    return fmaxf(t, 0.f);
}
__device__ __forceinline__ float fused_code(float t, float s_out) {
    return fminf(__builtin_rintf(t / s_out), 15.f);
}
// The same code without the division wherever that is provably the same: u = t * fl(1 / s) is
// within 1.5 * 2^-23 (relative) of fl(t / s), so below 16 the two differ by less than 2^-18 and
// round to the same integer unless u lies within 2^-17 of a half-integer, i.e. |u - rint(u)|
// (an exact difference) exceeds 1/2 - 2^-17; `worst` keeps the largest such distance of a word and
// the caller divides when it is that large.  From 15.6 upwards both round to 16 or more and the
// code is 15 either way.  (The ReLU stays in front of the quotient: behind it, one median-of-three
// would do for both clamps, but negative values would then reach the tie test, and with round
// steps, where ties are exact and common, nearly every wave would divide.)
__device__ __forceinline__ float fused_code_quick(float t, float inv_s, float& worst) {
#pragma clang fp contract(off)
    const float u = t * inv_s;
    const float q = __builtin_rintf(u);
    worst = fmaxf(worst, __builtin_fabsf(u - q));
    return fminf(q, 15.f);
}
// Eight codes (small non-negative integers held as floats) -> one packed word, code e in nibble e.
__device__ __forceinline__ uint32_t pack_codes(const float (&q)[8]) {
    uint32_t word = 0;
#pragma unroll
    for (int e = 0; e < 8; ++e) word |= (uint32_t)q[e] << (4 * e);
    return word;
}

// 8 consecutive channels of one output pixel -> one packed word; sc / bi: their scales and
// biases, r: their shortcut values (0 without a shortcut: t + 0 == t).
__device__ __forceinline__ uint32_t fused_pack(const int (&acc)[8], const float (&sc)[8], const float (&bi)[8],
                                               const float (&r)[8], const ConvOut& o) {
    float t[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) t[e] = fused_value(acc[e], sc[e], bi[e], r[e]);
    float q[8];
    float worst = o.quick ? 0.f : 1.f;
#pragma unroll
    for (int e = 0; e < 8; ++e) q[e] = fused_code_quick(t[e], o.inv_s_out, worst);
    if (__builtin_expect(!(worst <= 0.5f - 0x1p-17f), 0)) {
#pragma unroll
        for (int e = 0; e < 8; ++e) q[e] = fused_code(t[e], o.s_out);
    }
    return pack_codes(q);
}
__device__ __forceinline__ void load8(const float* p, float (&v)[8]) {
    const float4 a = *reinterpret_cast<const float4*>(p), b = *reinterpret_cast<const float4*>(p + 4);
    v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w; v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
}
// Shortcut values of 8 channels from a word of 4-bit codes (each times its step: one rounding).
__device__ __forceinline__ void shortcut_from_codes(uint32_t rw, float res_scale, float (&r)[8]) {
#pragma unroll
    for (int e = 0; e < 8; ++e) {
#pragma clang fp contract(off)
        r[e] = res_scale * (float)((rw >> (4 * e)) & 0xFu);
    }
}
__device__ __forceinline__ uint32_t fused_word(const int (&acc)[8], const ConvOut& o, size_t m, int n0, int cout) {
    float sc[8], bi[8], r[8];
    load8(o.scale + n0, sc);
    load8(o.bias + n0, bi);
    if (o.res_u4) {
        shortcut_from_codes(o.res_u4[m * (size_t)(cout / 8) + n0 / 8], o.res_scale, r);
    } else if (o.res_f32) {
        load8(o.res_f32 + m * (size_t)cout + n0, r);
    } else {
#pragma unroll
        for (int e = 0; e < 8; ++e) r[e] = 0.f;
    }
    return fused_pack(acc, sc, bi, r, o);
}

// Global -> LDS copy by the load unit through a buffer descriptor: lane l's 16 bytes at byte
// offset `off` of the buffer land at LDS address lds + 16 l; a lane whose offset lies outside the
// buffer writes 16 zero bytes (checked on the GPU with a probe), which is exactly what image
// borders, the K tail and tile edges need.  Assembly on purpose: the compiler would make every
// later LDS read wait for all such copies in flight (it cannot tell the ring slots apart).
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
__device__ __forceinline__ u32x4_t make_rsrc_words(const void* p, uint32_t bytes) {
    const uint64_t b = (uint64_t)(uintptr_t)p;
    u32x4_t r = {(uint32_t)b, (uint32_t)(b >> 32) & 0xFFFFu, bytes, 0x00020000u};
    r[0] = __builtin_amdgcn_readfirstlane(r[0]);
    r[1] = __builtin_amdgcn_readfirstlane(r[1]);
    r[2] = __builtin_amdgcn_readfirstlane(r[2]);
    r[3] = __builtin_amdgcn_readfirstlane(r[3]);
    return r;
}
__device__ __forceinline__ void dma16(u32x4_t rsrc, uint32_t off, uint32_t lds) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, 0 offen lds"
                 :: "s"(lds), "v"(off), "s"(rsrc) : "memory", "m0");
}
__host__ __device__ constexpr int waitcnt_vm(int n) { return (n & 15) | ((n >> 4) << 14) | (7 << 4); }  // lgkmcnt 0 too

constexpr int kStages = 3;  // ring of K steps in LDS: step s + 2 is loaded while step s is multiplied
constexpr int kMaxSteps = 128;  // rows of the step table (K steps plus the ring's look-ahead)

// Tiling: a block of 4 waves (2 x 2) owns a BM x BN output tile and walks K in steps of 128
// codes (64 B per row; K is ordered (kh, kw, c) and Cin % 32 == 0, so every 16-byte chunk lies
// inside one filter tap).  Rows are unpadded in LDS; chunk c of row r is kept at position
// c ^ swz(r), swz(r) = ((r / 4) % 4) ^ (r & 2), chosen through the loading lane's address: the
// 16-byte fragment reads of 8 consecutive rows then fall into 8 different 16-byte columns of
// a 128-byte line, and those of 16 consecutive rows into 16 different ones of a 256-byte line.
//
// KS > 1: KS groups of 4 waves share the tile and split K between them (group g takes steps
// g, g + KS, ...), each with its own ring; their int32 partial tiles are added in the epilogue
// (integer sums: exact in any order).  For the deep layers of a small batch, which have few
// tiles and long K, this puts several waves on every SIMD instead of one.
//
// kBits = 8 is the W8A8 variant of the same kernel (Sec. 5.4): bytes are MFMA operands as they
// are, a K step is 64 codes and one MFMA deep, nothing is widened and nothing shifted back.
//
// The tile at rows bm.., columns bn.. of one convolution; the two kernels below call it.
template <int BM, int BN, int KS, int kBits>
__device__ __forceinline__ void w4a4_conv_tile(const ConvGeom& gm, const uint32_t* __restrict__ a,
                                               const uint32_t* __restrict__ w, const ConvOut& out, const int bm,
                                               const int bn) {
    constexpr int kLA = BM / 64;   // wave-wide loads per wave and step for the activation tile
    constexpr int kLB = BN / 64;   // ... for the weight tile
    constexpr int kL = kLA + kLB;
    constexpr int kUM = BM / 64;   // 32 x 32 MFMA tiles per wave along m
    constexpr int kUN = BN / 64;   // ... along n
    constexpr int kAccs = kUM * kUN == 1 ? 2 : 1;  // a lone tile alternates between two accumulators (no dependent pair)
    constexpr int kStageBytes = (BM + BN) * 64;
    constexpr int kSPitch = BN + 4;  // words per row of the int32 staging tile of the epilogue
    constexpr int kPasses = BM * kSPitch * 4 <= kStages * kStageBytes ? 1 : 2;  // epilogue passes over the rows
    constexpr int kPassRows = BM / kPasses;
    constexpr int kGroupBytes = kStages * kStageBytes > kPassRows * kSPitch * 4 ? kStages * kStageBytes
                                                                                 : kPassRows * kSPitch * 4;
    constexpr int kThreads = 256 * KS;
    __shared__ __attribute__((aligned(16))) unsigned char smem_all[KS * kGroupBytes];
    __shared__ uint2 steptab[kMaxSteps * 4];

    const int t = threadIdx.x;
    const int lane = t % kWave;
    const int wave_all = __builtin_amdgcn_readfirstlane(t / kWave);
    const int grp = wave_all / 4, wave = wave_all % 4;   // K group, wave inside the group
    unsigned char* const smem = smem_all + grp * kGroupBytes;
    const int wm = wave / 2, wn = wave % 2;
    const int cw = gm.Cin / (32 / kBits);      // words per pixel
    const int kwords = gm.KH * gm.KW * cw;     // words per filter
    const int gsteps = (kwords + kStepWords - 1) / kStepWords;   // K steps of the whole problem
    const int steps = (gsteps + KS - 1) / KS;                     // ... of one group (the same for all)

    const u32x4_t ra = make_rsrc_words(a, (uint32_t)((size_t)gm.B * gm.H * gm.W * cw * 4));
    const u32x4_t rw = make_rsrc_words(w, (uint32_t)((size_t)gm.Cout * kwords * 4));
    const uint32_t lds0 = __builtin_amdgcn_readfirstlane(
        (uint32_t)(uintptr_t)(const __attribute__((address_space(3))) void*)smem);

    // Loader geometry: load i of this wave fills rows (4 i + wave) * 16 + lane / 4, position
    // lane % 4, with the chunk that belongs there.
    const int lrow = lane >> 2;
    const int chunk = (lane & 3) ^ ((lrow >> 2) & 3) ^ (lrow & 2);  // which 16 bytes of a step this lane fetches
    int abase[kLA];       // byte offset of (b, ih0, iw0, 0); may be negative at the border
    uint32_t amask[kLA];  // bit tap = the tap's pixel is inside the image
#pragma unroll
    for (int i = 0; i < kLA; ++i) {
        const int m = bm + (4 * i + wave) * 16 + lrow;
        abase[i] = 0;
        amask[i] = 0;
        if (m < gm.M) {
            const int b = div_by(m, gm.OH * gm.OW, gm.mg_ohow, gm.fastdiv);
            const int rem = m - b * (gm.OH * gm.OW);
            const int oh = div_by(rem, gm.OW, gm.mg_ow, gm.fastdiv), ow = rem - oh * gm.OW;
            const int ih0 = oh * gm.stride - gm.pad, iw0 = ow * gm.stride - gm.pad;
            abase[i] = ((b * gm.H + ih0) * gm.W + iw0) * cw * 4;
            // taps inside the image: kw in [kw_lo, kw_hi) for every kh in [kh_lo, kh_hi)
            const int kw_lo = max(0, -iw0), kw_hi = min(gm.KW, gm.W - iw0);
            const int kh_lo = max(0, -ih0), kh_hi = min(gm.KH, gm.H - ih0);
            const uint32_t cols = kw_hi > kw_lo ? (0xFFFFFFFFu >> (32 - (kw_hi - kw_lo))) << kw_lo : 0u;
            for (int kh = kh_lo; kh < kh_hi; ++kh) amask[i] |= cols << (kh * gm.KW);
        }
    }
    uint32_t bbase[kLB];
#pragma unroll
    for (int i = 0; i < kLB; ++i) {
        const int n = bn + (4 * i + wave) * 16 + lrow;
        bbase[i] = n < gm.Cout ? (uint32_t)n * kwords * 4 : kOut;
    }

    // Where a K step's chunks come from is the same for every row and every block: a table in
    // LDS, built once, holds for (step, chunk) the byte offset of the chunk from a pixel's
    // (ih0, iw0, 0), its offset inside a filter row, and its tap; steps past the end of K are
    // marked invalid (their loads read nothing and write zeros).
    {
        const int entries = (steps + kStages) * KS * 4;
        for (int e = t; e < entries; e += kThreads) {
            const int kw0 = (e >> 2) * kStepWords + (e & 3) * 4;   // first word of the chunk
            uint2 v = make_uint2(0u, 0xFFFFFFFFu);
            if (kw0 < kwords) {
                const int tap = div_by(kw0, cw, gm.mg_cw, gm.fastdiv), cword = kw0 - tap * cw;
                const int kh = div_by(tap, gm.KW, gm.mg_kw, gm.fastdiv), kwi = tap - kh * gm.KW;
                v.x = (uint32_t)(((kh * gm.W + kwi) * cw + cword) * 4);
                v.y = (uint32_t)(kw0 * 4) | ((uint32_t)tap << 26);
            }
            steptab[e] = v;
        }
    }
    __syncthreads();
    int pstep = 0;
    uint2 pent = steptab[grp * 4 + chunk];  // entry of the next step to plan, read one step ahead
    uint32_t poff[kL];
    auto plan = [&]() {
        const uint2 e = pent;
        ++pstep;
        pent = steptab[(pstep * KS + grp) * 4 + chunk];
        const bool kin = (e.y >> 31) == 0;
        const uint32_t tap = (e.y >> 26) & 31u, kw4 = e.y & 0x03FFFFFFu;
#pragma unroll
        for (int i = 0; i < kLA; ++i) {
            const bool in = kin && ((amask[i] >> tap) & 1u);
            poff[i] = in ? (uint32_t)(abase[i] + (int)e.x) : kOut;
        }
#pragma unroll
        for (int i = 0; i < kLB; ++i) poff[kLA + i] = kin ? bbase[i] + kw4 : kOut;
    };
    auto issue = [&](int i, int slot) {
        if (i < kLA)
            dma16(ra, poff[i], lds0 + slot * kStageBytes + (4 * i + wave) * 1024);
        else
            dma16(rw, poff[i], lds0 + slot * kStageBytes + BM * 64 + (4 * (i - kLA) + wave) * 1024);
    };

    // Fragment reads for the 32 x 32 x 32 MFMA (a wave issuing only 16 x 16 x 64 ones reaches 0.6 of
    // the matrix rate, measured): lane (r32, kh) supplies 16 codes of row r32 to each MFMA, as
    // the half kh of the MFMA's 32.  Which codes those are is free as long as both operands
    // agree, so a lane reads whole 16-byte chunks (an 8-byte read of one half of a chunk by
    // every lane leaves half of the banks idle).  4-bit: chunk 2 sub + kh of the K step, whose
    // first 8 bytes go to the first MFMA of the half-step `sub` and the rest to the second.
    // 8-bit: chunk 2 h + kh for MFMA h of the step.
    const int r32 = lane & 31, kh = lane >> 5;
    const int swz = ((r32 >> 2) & 3) ^ (r32 & 2);
    int foff[2];
#pragma unroll
    for (int u = 0; u < 2; ++u) foff[u] = r32 * 64 + (((2 * u + kh) ^ swz) << 4);

    i32x16_t acc[kUM][kUN][kAccs];
#pragma unroll
    for (int i = 0; i < kUM; ++i)
#pragma unroll
        for (int j = 0; j < kUN; ++j)
#pragma unroll
            for (int c = 0; c < kAccs; ++c)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[i][j][c][r] = 0;

    i32x4_t af[2][kUM][2], bf[2][kUN][2];
    auto widen_a = [](uint32_t x, uint32_t y) {
        return i32x4_t{(int)(x & 0x0F0F0F0Fu), (int)((x >> 4) & 0x0F0F0F0Fu), (int)(y & 0x0F0F0F0Fu),
                       (int)((y >> 4) & 0x0F0F0F0Fu)};
    };
    auto widen_b = [](uint32_t x, uint32_t y) {
        return i32x4_t{(int)((x << 4) & 0xF0F0F0F0u), (int)(x & 0xF0F0F0F0u), (int)((y << 4) & 0xF0F0F0F0u),
                       (int)(y & 0xF0F0F0F0u)};
    };
    auto fetch = [&](int slot, int sub, int reg) {
        const unsigned char* As = smem + slot * kStageBytes + wm * (BM / 2) * 64;
        const unsigned char* Bs = smem + slot * kStageBytes + BM * 64 + wn * (BN / 2) * 64;
        if constexpr (kBits == 4) {
#pragma unroll
            for (int i = 0; i < kUM; ++i) {
                const uint4 p = *reinterpret_cast<const uint4*>(As + foff[sub] + i * 32 * 64);
                af[reg][i][0] = widen_a(p.x, p.y);
                af[reg][i][1] = widen_a(p.z, p.w);
            }
#pragma unroll
            for (int j = 0; j < kUN; ++j) {
                const uint4 p = *reinterpret_cast<const uint4*>(Bs + foff[sub] + j * 32 * 64);
                bf[reg][j][0] = widen_b(p.x, p.y);
                bf[reg][j][1] = widen_b(p.z, p.w);
            }
        } else {
#pragma unroll
            for (int h = 0; h < 2; ++h) {
#pragma unroll
                for (int i = 0; i < kUM; ++i)
                    af[reg][i][h] = *reinterpret_cast<const i32x4_t*>(As + foff[h] + i * 32 * 64);
#pragma unroll
                for (int j = 0; j < kUN; ++j)
                    bf[reg][j][h] = *reinterpret_cast<const i32x4_t*>(Bs + foff[h] + j * 32 * 64);
            }
        }
    };
    auto multiply = [&](int reg) {
#pragma unroll
        for (int h = 0; h < 2; ++h)
#pragma unroll
            for (int i = 0; i < kUM; ++i)
#pragma unroll
                for (int j = 0; j < kUN; ++j)
                    acc[i][j][h % kAccs] = __builtin_amdgcn_mfma_i32_32x32x32_i8(af[reg][i][h], bf[reg][j][h],
                                                                                 acc[i][j][h % kAccs], 0, 0, 0);
        // issue order: the LDS reads and the widening of the next fragments go between the MFMAs
        constexpr int kM = 2 * kUM * kUN, kF = 2 * (kUM + kUN);   // MFMAs, operand fragments
        constexpr int kR = kBits == 4 ? kF / 2 : kF;               // LDS reads (4-bit: one per two fragments)
        constexpr int kRead = (kR + kM - 1) / kM;
#pragma unroll
        for (int u = 0; u < kM; ++u) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            if (u * kRead < kR) __builtin_amdgcn_sched_group_barrier(0x100, kRead, 0);
            if (kBits == 4) __builtin_amdgcn_sched_group_barrier(0x002, (4 * kF + kM - 1) / kM, 0);
        }
    };

    // steps 0 and 1 up front, then step s + 2 during step s
#pragma unroll
    for (int p = 0; p < kStages - 1; ++p) {
        plan();
#pragma unroll
        for (int i = 0; i < kL; ++i) issue(i, p);
    }
    __builtin_amdgcn_s_waitcnt(waitcnt_vm(kL));
    __syncthreads();
    fetch(0, 0, 0);

    if constexpr (kBits == 4) {
        for (int s0 = 0; s0 < steps; s0 += kStages) {
#pragma unroll
            for (int u = 0; u < kStages; ++u) {
                if (s0 + u >= steps) break;
                const int cur = u, nxt = (u + 1) % kStages, fill = (u + 2) % kStages;
                __builtin_amdgcn_sched_barrier(0);
                fetch(cur, 1, 1);
                multiply(0);
                __builtin_amdgcn_sched_barrier(0);
                // slot `fill` held step s - 1, whose last reads were issued before the previous barrier
                plan();
#pragma unroll
                for (int i = 0; i < kL; ++i) issue(i, fill);
                // in flight: step s + 1 (issued one step ago) and step s + 2 (just issued)
                __builtin_amdgcn_s_waitcnt(waitcnt_vm(kL));
                __syncthreads();
                __builtin_amdgcn_sched_barrier(0);
                fetch(nxt, 0, 0);
                multiply(1);
            }
        }
    } else {
        // one MFMA step per K step: the operand registers alternate with the step's parity, so
        // the ring of three is unrolled twice
        for (int s0 = 0; s0 < steps; s0 += 2 * kStages) {
#pragma unroll
            for (int u = 0; u < 2 * kStages; ++u) {
                if (s0 + u >= steps) break;
                const int nxt = (u + 1) % kStages, fill = (u + 2) % kStages, reg = u & 1;
                __builtin_amdgcn_sched_barrier(0);
                plan();
#pragma unroll
                for (int i = 0; i < kL; ++i) issue(i, fill);
                __builtin_amdgcn_s_waitcnt(waitcnt_vm(kL));
                __syncthreads();
                __builtin_amdgcn_sched_barrier(0);
                fetch(nxt, 0, reg ^ 1);
                multiply(reg);
            }
        }
    }
    __builtin_amdgcn_sched_barrier(0);
    __builtin_amdgcn_s_waitcnt(waitcnt_vm(0));  // nothing may still be writing LDS
    __syncthreads();

    // Epilogue: the accumulators (all rows at once if they fit, else half the rows at a time)
    // are staged in LDS (pitch BN + 4 words: conflict-free for the writes below) and leave as
    // whole pieces of rows.
    int32_t* const stage = reinterpret_cast<int32_t*>(smem);
    // A thread writes the same columns in every iteration of the store loops below (the block's
    // thread count is a multiple of the pieces per row), so their scales and biases are fetched
    // once, here, and the shortcut words of a pass before its barrier: a load inside the store
    // loop would wait out its full latency in every iteration, behind the previous store.
    constexpr int kWordsPerRow = BN / 8, kQuadsPerRow = BN / 4;
    static_assert(kThreads % kWordsPerRow == 0 && kThreads % kQuadsPerRow == 0, "columns fixed per thread");
    constexpr int kItF = (kPassRows * kWordsPerRow + kThreads - 1) / kThreads;
    const int n0f = bn + (t % kWordsPerRow) * 8, n0q = bn + (t % kQuadsPerRow) * 4;
    const bool vec = (gm.Cout % 4) == 0;
    float scf[8], bif[8];
    float4 scq = make_float4(0.f, 0.f, 0.f, 0.f), biq = scq;
    if (out.out_u4) {
        if (n0f < gm.Cout) {
            load8(out.scale + n0f, scf);
            load8(out.bias + n0f, bif);
        }
    } else if (out.y && vec && n0q < gm.Cout) {
        scq = *reinterpret_cast<const float4*>(out.scale + n0q);
        biq = *reinterpret_cast<const float4*>(out.bias + n0q);
    }
#pragma unroll
    for (int pass = 0; pass < kPasses; ++pass) {
        if (pass) __syncthreads();  // the previous pass has been read
        uint32_t rwf[kItF];
        if (out.out_u4 && out.res_u4) {
#pragma unroll
            for (int it = 0; it < kItF; ++it) {
                const int idx = t + it * kThreads;
                const int m = bm + pass * kPassRows + idx / kWordsPerRow;
                rwf[it] = (idx < kPassRows * kWordsPerRow && m < gm.M && n0f < gm.Cout)
                              ? out.res_u4[(size_t)m * (gm.Cout / 8) + n0f / 8] : 0u;
            }
        }
        if (kPasses == 1 || wm == pass) {
            const int rbase = kPasses == 1 ? wm * (BM / 2) : 0;
            // 32 x 32 accumulator: register r of lane (c32, hi) is row 8 (r / 4) + 4 hi + r % 4, column c32
#pragma unroll
            for (int i = 0; i < kUM; ++i)
#pragma unroll
                for (int j = 0; j < kUN; ++j)
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const int v = kAccs == 2 ? acc[i][j][0][r] + acc[i][j][kAccs - 1][r] : acc[i][j][0][r];
                        stage[(rbase + i * 32 + 8 * (r / 4) + 4 * kh + (r % 4)) * kSPitch + wn * (BN / 2) + j * 32 + r32] =
                            kBits == 4 ? v >> 4 : v;  // 4-bit: the accumulator is 16 * result
                    }
        }
        __syncthreads();
        if (out.out_u4) {
            // fused output: 8 consecutive channels of a pixel -> one packed word
#pragma unroll
            for (int it = 0; it < kItF; ++it) {
                const int idx = t + it * kThreads;
                if (idx >= kPassRows * kWordsPerRow) break;
                const int row = idx / kWordsPerRow, wd = idx % kWordsPerRow;
                const int m = bm + pass * kPassRows + row, n0 = n0f;
                if (m >= gm.M || n0 >= gm.Cout) continue;
                i32x4_t v0 = {0, 0, 0, 0}, v1 = {0, 0, 0, 0};
#pragma unroll
                for (int g = 0; g < KS; ++g) {
                    const int32_t* sg = reinterpret_cast<const int32_t*>(smem_all + g * kGroupBytes);
                    v0 += *reinterpret_cast<const i32x4_t*>(&sg[row * kSPitch + wd * 8]);
                    v1 += *reinterpret_cast<const i32x4_t*>(&sg[row * kSPitch + wd * 8 + 4]);
                }
                const int av[8] = {v0[0], v0[1], v0[2], v0[3], v1[0], v1[1], v1[2], v1[3]};
                float r[8];
                if (out.res_u4) {
                    shortcut_from_codes(rwf[it], out.res_scale, r);
                } else if (out.res_f32) {
                    load8(out.res_f32 + (size_t)m * gm.Cout + n0, r);
                } else {
#pragma unroll
                    for (int e = 0; e < 8; ++e) r[e] = 0.f;
                }
                out.out_u4[(size_t)m * (gm.Cout / 8) + n0 / 8] = fused_pack(av, scf, bif, r, out);
            }
        } else {
            // plain outputs: 4 consecutive channels per thread, 16-byte stores when Cout allows
            for (int idx = t; idx < kPassRows * kQuadsPerRow; idx += kThreads) {
                const int row = idx / kQuadsPerRow, qd = idx % kQuadsPerRow;
                const int m = bm + pass * kPassRows + row, n0 = bn + qd * 4;
                if (m >= gm.M || n0 >= gm.Cout) continue;
                i32x4_t v = {0, 0, 0, 0};
#pragma unroll
                for (int g = 0; g < KS; ++g)
                    v += *reinterpret_cast<const i32x4_t*>(
                        &reinterpret_cast<const int32_t*>(smem_all + g * kGroupBytes)[row * kSPitch + qd * 4]);
                const size_t o = (size_t)m * gm.Cout + n0;
                if (vec) {
                    if (out.acc) *reinterpret_cast<i32x4_t*>(out.acc + o) = v;
                    if (out.y) {
                        const float4 sc = scq, bi = biq;
                        *reinterpret_cast<float4*>(out.y + o) =
                            make_float4(fmaf((float)v[0], sc.x, bi.x), fmaf((float)v[1], sc.y, bi.y),
                                        fmaf((float)v[2], sc.z, bi.z), fmaf((float)v[3], sc.w, bi.w));
                    }
                } else {
                    for (int e = 0; e < 4 && n0 + e < gm.Cout; ++e) {
                        if (out.acc) out.acc[o + e] = v[e];
                        if (out.y) out.y[o + e] = fmaf((float)v[e], out.scale[n0 + e], out.bias[n0 + e]);
                    }
                }
            }
        }
    }
}

// One convolution per launch: grid (column tiles, row tiles).
template <int BM, int BN, int KS, int kBits>
__global__ __launch_bounds__(256 * KS, (KS > 1 ? 1 : (BM * BN >= 128 * 128 ? 2 : 4))) void w4a4_conv_kernel(
    const ConvGeom gm, const uint32_t* __restrict__ a, const uint32_t* __restrict__ w, const ConvOut out) {
    w4a4_conv_tile<BM, BN, KS, kBits>(gm, a, w, out, blockIdx.y * BM, blockIdx.x * BN);
}

// Several per launch: item i is the grid's plane z = i.
template <int BM, int BN, int KS, int kBits>
__global__ __launch_bounds__(256 * KS, (KS > 1 ? 1 : (BM * BN >= 128 * 128 ? 2 : 4))) void w4a4_conv_batch_kernel(
    const ConvBatch args) {
    const ConvItem& it = args.it[blockIdx.z];
    const ConvGeom gm = it.gm;
    if ((int)blockIdx.x * BN >= gm.Cout || (int)blockIdx.y * BM >= gm.M) return;   // the grid fits the largest item
    w4a4_conv_tile<BM, BN, KS, kBits>(gm, it.a, it.w, it.out, blockIdx.y * BM, blockIdx.x * BN);
}

// Any Cin that fills whole words: one thread per output.  Slow; for shapes whose Cin is not a
// multiple of 32, more than 32 filter taps, or tensors of 4 GB and more.
template <int kBits>
__global__ __launch_bounds__(256) void w4a4_generic_kernel(
    const ConvGeom gm, const uint32_t* __restrict__ a, const uint32_t* __restrict__ w, const ConvOut out) {
    int32_t* const acc_out = out.acc;
    const float* const scale = out.scale;
    const float* const bias = out.bias;
    float* const y_out = out.y;
    const size_t o = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (o >= (size_t)gm.M * gm.Cout) return;
    const int m = (int)(o / gm.Cout), n = (int)(o % gm.Cout);
    const int b = m / (gm.OH * gm.OW);
    const int rem = m - b * (gm.OH * gm.OW);
    const int oh = rem / gm.OW, ow = rem - oh * gm.OW;
    const int cw = gm.Cin / (32 / kBits);
    int acc = 0;
    for (int kh = 0; kh < gm.KH; ++kh)
        for (int kwi = 0; kwi < gm.KW; ++kwi) {
            const int ih = oh * gm.stride + kh - gm.pad, iw = ow * gm.stride + kwi - gm.pad;
            if (ih < 0 || ih >= gm.H || iw < 0 || iw >= gm.W) continue;
            const uint32_t* ap = a + ((size_t)(b * gm.H + ih) * gm.W + iw) * cw;
            const uint32_t* wp = w + ((size_t)(n * gm.KH + kh) * gm.KW + kwi) * cw;
            for (int c = 0; c < cw; ++c) {
                const uint32_t av = ap[c], wv = wp[c];
                if (kBits == 4) {
#pragma unroll
                    for (int j = 0; j < 8; ++j) {
                        const int qa = (av >> (4 * j)) & 0xF;
                        const int qw = (int)(((wv >> (4 * j)) & 0xFu) ^ 8u) - 8;
                        acc += qa * qw;
                    }
                } else {
#pragma unroll
                    for (int j = 0; j < 4; ++j) acc += (int)(int8_t)(av >> (8 * j)) * (int)(int8_t)(wv >> (8 * j));
                }
            }
        }
    if (acc_out) acc_out[o] = acc;
    if (y_out) y_out[o] = fmaf((float)acc, scale[n], bias[n]);
}

// Fused output for the shapes above: one thread per packed output word.
__global__ __launch_bounds__(256) void w4a4_generic_u4_kernel(
    const ConvGeom gm, const uint32_t* __restrict__ a, const uint32_t* __restrict__ w, const ConvOut out) {
    const size_t o = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int wpr = gm.Cout / 8;
    if (o >= (size_t)gm.M * wpr) return;
    const int m = (int)(o / wpr), n0 = (int)(o % wpr) * 8;
    const int b = m / (gm.OH * gm.OW);
    const int rem = m - b * (gm.OH * gm.OW);
    const int oh = rem / gm.OW, ow = rem - oh * gm.OW;
    const int cw = gm.Cin / 8;
    int acc[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    for (int kh = 0; kh < gm.KH; ++kh)
        for (int kwi = 0; kwi < gm.KW; ++kwi) {
            const int ih = oh * gm.stride + kh - gm.pad, iw = ow * gm.stride + kwi - gm.pad;
            if (ih < 0 || ih >= gm.H || iw < 0 || iw >= gm.W) continue;
            const uint32_t* ap = a + ((size_t)(b * gm.H + ih) * gm.W + iw) * cw;
            for (int c = 0; c < cw; ++c) {
                const uint32_t av = ap[c];
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const uint32_t wv = w[((size_t)((n0 + e) * gm.KH + kh) * gm.KW + kwi) * cw + c];
#pragma unroll
                    for (int j = 0; j < 8; ++j)
                        acc[e] += (int)((av >> (4 * j)) & 0xFu) * ((int)(((wv >> (4 * j)) & 0xFu) ^ 8u) - 8);
                }
            }
        }
    out.out_u4[o] = fused_word(acc, out, (size_t)m, n0, gm.Cout);
}

// One convolution made ready for a launch.
struct ConvJob {
    ConvGeom gm;
    const uint32_t* a;
    const uint32_t* w;
    ConvOut out;
    bool tiled;   // the tiled kernel can run it
    int ksteps;   // K steps of the tiled kernel
};

// One launch of the tiled kernel for n jobs (n <= kConvBatch) that share a tile configuration.
template <int kBits, int BM, int BN, int KS = 1>
void launch_tiled(const ConvJob* jobs, int n, hipStream_t st) {
    ConvBatch cb;
    int ny = 0, nx = 0;
    for (int i = 0; i < kConvBatch; ++i) {
        const ConvJob& j = jobs[i < n ? i : 0];
        cb.it[i] = ConvItem{j.gm, j.a, j.w, j.out};
        if (i < n) {
            ny = std::max(ny, (j.gm.M + BM - 1) / BM);
            nx = std::max(nx, (j.gm.Cout + BN - 1) / BN);
        }
    }
    if (kBits == 4 && n > 1)
        hipLaunchKernelGGL((w4a4_conv_batch_kernel<BM, BN, KS, 4>), dim3(nx, ny, n), dim3(256 * KS), 0, st, cb);
    else
        hipLaunchKernelGGL((w4a4_conv_kernel<BM, BN, KS, kBits>), dim3(nx, ny, 1), dim3(256 * KS), 0, st, jobs[0].gm,
                           jobs[0].a, jobs[0].w, jobs[0].out);
}

template <int kBits>
ConvJob make_job(const qail_conv_desc& d, const uint32_t* a, const uint32_t* w, const ConvOut& out) {
    constexpr int kPerWord = 32 / kBits;
    ConvJob job;
    ConvGeom& gm = job.gm;
    gm.B = d.B; gm.H = d.H; gm.W = d.W; gm.Cin = d.Cin; gm.Cout = d.Cout;
    gm.KH = d.KH; gm.KW = d.KW; gm.stride = d.stride; gm.pad = d.pad;
    gm.OH = (d.H + 2 * d.pad - d.KH) / d.stride + 1;
    gm.OW = (d.W + 2 * d.pad - d.KW) / d.stride + 1;
    gm.M = d.B * gm.OH * gm.OW;
    {
        // the tiled kernel divides m < M by OH OW, the remainder by OW, a word index below the
        // filter's words by the words per pixel and a tap below KH KW by KW
        const uint32_t cw = (uint32_t)(gm.Cin / kPerWord);
        bool ok = gm.M > 0;
        gm.mg_ohow = div_magic((uint32_t)(gm.OH * gm.OW), (uint64_t)gm.M, ok);
        gm.mg_ow = div_magic((uint32_t)gm.OW, (uint64_t)gm.OH * gm.OW, ok);
        gm.mg_cw = div_magic(cw, (uint64_t)gm.KH * gm.KW * cw, ok);
        gm.mg_kw = div_magic((uint32_t)gm.KW, (uint64_t)gm.KH * gm.KW, ok);
        gm.fastdiv = ok ? 1 : 0;
    }
    const size_t cwb = (size_t)gm.Cin / kPerWord * 4;  // bytes per pixel
    const bool fits32 = (size_t)gm.B * gm.H * gm.W * cwb < 0xFFFFFFF0ull &&
                        (size_t)gm.Cout * gm.KH * gm.KW * cwb < 0xFFFFFFF0ull &&
                        (size_t)gm.M * gm.Cout * 4 < 0xFFFFFFF0ull;
    job.ksteps = (gm.KH * gm.KW * (gm.Cin / kPerWord) + kStepWords - 1) / kStepWords;
    // a 16-byte chunk (32 or 16 codes) must lie inside one filter tap
    job.tiled = d.Cin % (4 * kPerWord) == 0 && d.KH * d.KW <= 32 && fits32 && job.ksteps + 4 * (kStages + 1) <= kMaxSteps;
    job.a = a;
    job.w = w;
    job.out = out;
    return job;
}

// Launches n jobs the tiled kernel can run (n <= kConvBatch) as one grid.  The tile is chosen for
// the job with the longest K (the one that decides how long the launch takes); whether K is split
// between groups of waves depends on how many blocks all jobs together put on a CU.
template <int kBits>
void launch_tiled_jobs(const ConvJob* jobs, int n, hipStream_t st) {
    int lead = 0;
    for (int i = 1; i < n; ++i)
        if ((long long)jobs[i].ksteps * jobs[i].gm.M > (long long)jobs[lead].ksteps * jobs[lead].gm.M) lead = i;
    const ConvGeom& gm = jobs[lead].gm;
    const int ksteps = jobs[lead].ksteps;
    // the largest tile that still gives every CU about two blocks
    const long long want = 2LL * device_cu_count();
    auto blocks = [&](int bm, int bn) {
        return (long long)((gm.M + bm - 1) / bm) * ((gm.Cout + bn - 1) / bn);
    };
    long long all64 = 0;
    for (int i = 0; i < n; ++i)
        all64 += (long long)((jobs[i].gm.M + 63) / 64) * ((jobs[i].gm.Cout + 63) / 64);
    const bool wide = gm.Cout > 64;
    // (the 128 x 128 tile already from one and a half blocks per CU: at batch 256 it takes the
    // 512 -> 512 layers from 45.7 to 37.6 us against the 128 x 64 tile)
    if (wide && 4 * blocks(128, 128) >= 3 * want) launch_tiled<kBits, 128, 128>(jobs, n, st);
    else if (blocks(128, 64) >= want) launch_tiled<kBits, 128, 64>(jobs, n, st);
    else if (wide && blocks(64, 128) >= want / 2) launch_tiled<kBits, 64, 128>(jobs, n, st);
    else if (all64 <= device_cu_count() && ksteps >= 16) launch_tiled<kBits, 64, 64, 4>(jobs, n, st);
    else if (all64 <= 2 * device_cu_count() && ksteps >= 8) launch_tiled<kBits, 64, 64, 2>(jobs, n, st);
    else launch_tiled<kBits, 64, 64>(jobs, n, st);
}

template <int kBits>
hipError_t launch_job(const ConvJob& job, hipStream_t st) {
    if (job.tiled) {
        launch_tiled_jobs<kBits>(&job, 1, st);
    } else if (job.out.out_u4) {
        const size_t words = (size_t)job.gm.M * (job.gm.Cout / 8);
        hipLaunchKernelGGL(w4a4_generic_u4_kernel, dim3((unsigned)((words + 255) / 256)), dim3(256), 0, st, job.gm,
                           job.a, job.w, job.out);
    } else {
        const size_t outs = (size_t)job.gm.M * job.gm.Cout;
        hipLaunchKernelGGL(w4a4_generic_kernel<kBits>, dim3((unsigned)((outs + 255) / 256)), dim3(256), 0, st, job.gm,
                           job.a, job.w, job.out);
    }
    return hipGetLastError();
}

template <int kBits>
hipError_t launch_conv(const qail_conv_desc& d, const uint32_t* a, const uint32_t* w, const ConvOut& out,
                       hipStream_t st) {
    return launch_job<kBits>(make_job<kBits>(d, a, w, out), st);
}

ConvOut fused_out(const float* scale, const float* bias, float s_out, const uint32_t* res_u4, float res_scale,
                  const float* res_f32, uint32_t* out_u4) {
    const float inv = 1.0f / s_out;
    const int quick = std::isnormal(s_out) && std::isnormal(inv) && s_out > 0.f;
    return ConvOut{nullptr, scale, bias, nullptr, out_u4, res_u4, res_f32, s_out, res_scale, inv, quick};
}
}  // namespace

// Independent W4A4 convolutions (plain or fused output each) in few launches: consecutive ones the
// tiled kernel can run share a launch, kConvBatch at a time, as long as their tile grids are of
// similar size (every plane of the launch's grid is as large as the largest); the others go one by one.
hipError_t launch_w4a4_conv_batch(const qail_conv_item* items, int count, hipStream_t st) {
    ConvJob tiled[kConvBatch];
    int n = 0;
    long long lo = 0, hi = 0;   // smallest and largest tile grid (in 64 x 64 tiles) of the pending launch
    auto flush = [&]() -> hipError_t {
        if (n > 0) launch_tiled_jobs<4>(tiled, n, st);
        n = 0;
        return hipGetLastError();
    };
    for (int i = 0; i < count; ++i) {
        const qail_conv_item& it = items[i];
        const ConvOut out = it.out_u4 ? fused_out(it.scale, it.bias, it.s_out, it.res_u4, it.res_scale, it.res_f32, it.out_u4)
                                      : ConvOut{it.acc_out, it.scale, it.bias, it.y_out, nullptr, nullptr, nullptr, 1.f, 0.f, 1.f, 0};
        const ConvJob job = make_job<4>(it.d, it.a_u4, it.w_s4, out);
        if (!job.tiled) {
            const hipError_t e = launch_job<4>(job, st);
            if (e != hipSuccess) return e;
            continue;
        }
        const long long t = (long long)((job.gm.M + 63) / 64) * ((job.gm.Cout + 63) / 64);
        if (n == kConvBatch || (n > 0 && (2 * std::min(lo, t) < std::max(hi, t)))) {
            const hipError_t e = flush();
            if (e != hipSuccess) return e;
        }
        lo = n ? std::min(lo, t) : t;
        hi = n ? std::max(hi, t) : t;
        tiled[n++] = job;
    }
    return flush();
}

hipError_t launch_w4a4_conv(const qail_conv_desc& d, const uint32_t* a, const uint32_t* w, int32_t* acc,
                            const float* scale, const float* bias, float* y, hipStream_t st) {
    const ConvOut out{acc, scale, bias, y, nullptr, nullptr, nullptr, 1.f, 0.f, 1.f, 0};
    return launch_conv<4>(d, a, w, out, st);
}

hipError_t launch_w8a8_conv(const qail_conv_desc& d, const uint32_t* a, const uint32_t* w, int32_t* acc,
                            const float* scale, const float* bias, float* y, hipStream_t st) {
    const ConvOut out{acc, scale, bias, y, nullptr, nullptr, nullptr, 1.f, 0.f, 1.f, 0};
    return launch_conv<8>(d, a, w, out, st);
}

hipError_t launch_w4a4_conv_u4(const qail_conv_desc& d, const uint32_t* a, const uint32_t* w, const float* scale,
                               const float* bias, float s_out, const uint32_t* res_u4, float res_scale,
                               const float* res_f32, uint32_t* out_u4, hipStream_t st) {
    return launch_conv<4>(d, a, w, fused_out(scale, bias, s_out, res_u4, res_scale, res_f32, out_u4), st);
}

}  // namespace qail
