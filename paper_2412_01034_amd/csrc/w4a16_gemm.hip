// W4A16 linear for M > 16 on the fp16 matrix cores:
//   y[m][n] = sum_k x[m][k] * (q[n][k] - z[n][k/g]) * s[n][k/g].
//
// Appendix "Analysis": prefill is the compute-heavy stage of the backbone, so this is
// the one W4A16 kernel bound by the matrix pipe rather than by HBM.  The design goal is
// to keep vector-ALU and LDS work per MFMA low:
//
//   * The weights never pass through LDS.  A wave owns 64 columns n; lane (c, kb) loads
//     the 8 packed words (64 consecutive k) of row n = c of a 128-k step straight from
//     global memory and expands one word into the 8 fp16 values one
//     v_mfma_f32_32x32x16_f16 needs from it as B operand:  0x6400 | q is the fp16 number
//     1024 + q and 0x6400 | (q << 4) is 1024 + 16 q, so a v_and_or_b32 yields two codes,
//     one packed add (or fma with 1/16) removes the offset together with the zero-point
//     exactly, and one packed multiply applies the scale: 13 vector operations per word,
//     used by BM / 32 MFMAs.
//   * Only the activations are staged in LDS, once per block, and every wave reads the
//     whole tile: one 16-byte LDS read per two MFMAs.
//   * fp16 holds every bf16 significand but not its range, so a small kernel first
//     rewrites x per row as fp16 scaled by a power of two (largest magnitude in
//     [2^14, 2^15)), with the k order inside each group of 8 that the expansion above
//     produces (0,4,1,5,2,6,3,7).  Group scales are divided by the power of two of the
//     row's largest scale, which keeps (q - z) * s below 32 in fp16; both powers of two
//     are multiplied back in fp32 at the end.  A weight is therefore rounded once to 11
//     significant bits (the bf16 alternative keeps 8).
//
// kBits = 8 is the 8-bit weight-only variant (Sec. 5.4 deploys the backbone with 8-bit weights
// too): signed bytes, one fp16 scale per group, no zero-point.  A byte q becomes fp16 without a
// conversion: (q ^ 0x80) is q + 128 as an unsigned byte u, and 0x6400 | u is the fp16 number
// 1024 + u, so one XOR per word, one byte permute per pair of codes, a packed add of -1152 (exact)
// and a packed multiply by the scale give (q * s): 14 vector operations per 8 codes.  The codes
// come out in their natural order, so x is stored in natural order for this variant.  A lane's
// 64 k of a step are four 16-byte pieces instead of two; with that the ring only fits LDS with
// 128-column tiles.
//
// MFMA operand layout (32x32x16, wave64): lane l supplies row (A) / column (B) l%32 and
// the 8 consecutive k starting at 8*(l/32); it receives D[8*(r/4) + 4*(l/32) + r%4][l%32]
// for r = 0..15.  A = activations (rows m), B = weights (columns n).
#include <algorithm>

#include <atomic>

#include "qail_internal.h"

namespace qail {

namespace {

typedef _Float16 f16x2_t __attribute__((ext_vector_type(2)));
typedef _Float16 f16x8_t __attribute__((ext_vector_type(8)));
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));

constexpr int kBK = 128;                // k per step
constexpr int kMaxGemmBlocks = 512;     // upper bound of the grid (the workspace has two slots per block)
constexpr int kRowPad = 128;            // workspace rows are padded to this

__host__ __device__ inline int round_up(int v, int m) { return (v + m - 1) / m * m; }

constexpr int kGemmBatch = 8;           // linears that can share one launch

// ---------------------------------------------------------------------------------------
// Preparation, for up to kGemmBatch linears at once (blockIdx.y): blocks [0, Mpad) rewrite one
// row of x each, the rest find the power of two of each weight row's largest scale.
struct PrepItem {
    const uint16_t* x;
    const uint16_t* sc;
    uint16_t* xh;
    float* rscale;
    float* wmul;
    int N, K, Kpad, G;
};
struct PrepBatch {
    PrepItem it[kGemmBatch];
    int M, Mpad;
    int natural;   // 8-bit codes expand in their natural order, 4-bit ones as 0,4,1,5,2,6,3,7
};

__global__ __launch_bounds__(256) void gemm_prep_kernel(const PrepBatch args) {
    __shared__ uint32_t red[4];
    const int t = threadIdx.x;
    const PrepItem pi = args.it[blockIdx.y];
    const uint16_t* __restrict__ x = pi.x;
    const uint16_t* __restrict__ sc = pi.sc;
    uint16_t* __restrict__ xh = pi.xh;
    float* __restrict__ rscale = pi.rscale;
    float* __restrict__ wmul = pi.wmul;
    const int M = args.M, Mpad = args.Mpad, N = pi.N, K = pi.K, Kpad = pi.Kpad, G = pi.G;
    if ((int)blockIdx.x >= Mpad + (N + 31) / 32) return;   // the grid is as wide as the largest linear needs
    if ((int)blockIdx.x < Mpad) {
        const int m = blockIdx.x;
        uint4* dst = reinterpret_cast<uint4*>(xh + (size_t)m * Kpad);
        if (m >= M) {
            for (int i = t; i < Kpad / 8; i += 256) dst[i] = make_uint4(0, 0, 0, 0);
            if (t == 0) rscale[m] = 0.f;
            return;
        }
        const uint4* src = reinterpret_cast<const uint4*>(x + (size_t)m * K);
        // the row is read once: a thread keeps its pieces (up to kKeep of them: rows up to 2048 kKeep long) in
        // registers between the search for the largest magnitude and the rewrite; longer rows are read again
        constexpr int kKeep = 6;
        uint4 keep[kKeep];
        uint32_t mx = 0;  // largest magnitude bit pattern (order-preserving for bf16 magnitudes)
#pragma unroll
        for (int r = 0; r < kKeep; ++r) {
            const int i = t + 256 * r;
            keep[r] = i < K / 8 ? src[i] : make_uint4(0, 0, 0, 0);
        }
#pragma unroll
        for (int r = 0; r < kKeep; ++r) {
            const uint32_t w[4] = {keep[r].x, keep[r].y, keep[r].z, keep[r].w};
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                mx = max(mx, w[j] & 0x7FFFu);
                mx = max(mx, (w[j] >> 16) & 0x7FFFu);
            }
        }
        for (int i = t + 256 * kKeep; i < K / 8; i += 256) {
            const uint4 v = src[i];
            const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                mx = max(mx, w[j] & 0x7FFFu);
                mx = max(mx, (w[j] >> 16) & 0x7FFFu);
            }
        }
#pragma unroll
        for (int o = 32; o >= 1; o >>= 1) mx = max(mx, (uint32_t)__shfl_xor((int)mx, o));
        if (t % kWave == 0) red[t / kWave] = mx;
        __syncthreads();
        mx = max(max(red[0], red[1]), max(red[2], red[3]));
        // x * 2^p has its largest magnitude in [2^14, 2^15); p is kept in the normal fp32 range
        const int e = (int)(mx >> 7);  // biased exponent of the largest magnitude
        int p = mx == 0 ? 0 : 141 - e;
        p = p > 126 ? 126 : (p < -126 ? -126 : p);
        const float up = __builtin_bit_cast(float, (uint32_t)(127 + p) << 23);
        if (t == 0) rscale[m] = __builtin_bit_cast(float, (uint32_t)(127 - p) << 23);
        auto rewrite = [&](const uint4 v) {
            const uint16_t b[8] = {(uint16_t)v.x, (uint16_t)(v.x >> 16), (uint16_t)v.y, (uint16_t)(v.y >> 16),
                                   (uint16_t)v.z, (uint16_t)(v.z >> 16), (uint16_t)v.w, (uint16_t)(v.w >> 16)};
            uint32_t h[8];
#pragma unroll
            for (int j = 0; j < 8; ++j)
                h[j] = __builtin_bit_cast(uint16_t, (_Float16)(bf16_bits_to_f32(b[j]) * up));
            // stored order inside the 8: 0,4,1,5,2,6,3,7 (4-bit codes) or as they are (8-bit codes)
            return args.natural
                       ? make_uint4(h[0] | (h[1] << 16), h[2] | (h[3] << 16), h[4] | (h[5] << 16), h[6] | (h[7] << 16))
                       : make_uint4(h[0] | (h[4] << 16), h[1] | (h[5] << 16), h[2] | (h[6] << 16), h[3] | (h[7] << 16));
        };
#pragma unroll
        for (int r = 0; r < kKeep; ++r) {
            const int i = t + 256 * r;
            // (a kept piece past the end of the row is zero, and so is its rewrite: the padding up to Kpad)
            if (i < Kpad / 8) dst[i] = rewrite(keep[r]);
        }
        for (int i = t + 256 * kKeep; i < Kpad / 8; i += 256)
            dst[i] = i < K / 8 ? rewrite(src[i]) : make_uint4(0, 0, 0, 0);
        return;
    }
    // 8 lanes per weight row, 32 rows per block
    const int n = ((int)blockIdx.x - Mpad) * 32 + t / 8;
    const int part = t % 8;
    uint32_t mx = 0;
    if (n < N)
        for (int gi = part; gi < G; gi += 8) mx = max(mx, (uint32_t)sc[(size_t)n * G + gi]);
#pragma unroll
    for (int o = 4; o >= 1; o >>= 1) mx = max(mx, (uint32_t)__shfl_xor((int)mx, o));
    if (n < N && part == 0) {
        // scales are positive fp16, at least 2^-14 (a stored subnormal is treated as 2^-14)
        int e = (int)(mx >> 10) & 31;
        e = e < 1 ? 1 : e;
        wmul[n] = __builtin_bit_cast(float, (uint32_t)(127 + e - 15) << 23);
    }
}

// ---------------------------------------------------------------------------------------
// 8 codes of a word -> 8 fp16 (q - z) * s in the order 0,4,1,5,2,6,3,7.
//   nz  = -(1024 + z) in both halves, nz6 = -(64 + z), s2 = scale in both halves.
__device__ __forceinline__ f16x8_t expand_word(uint32_t w, uint32_t magic, f16x2_t nz, f16x2_t nz6, f16x2_t s2) {
    const f16x2_t sixteenth = {(_Float16)0.0625f, (_Float16)0.0625f};
    const uint32_t w8 = w >> 8;
    const f16x2_t p0 = __builtin_bit_cast(f16x2_t, (w & 0x000F000Fu) | magic);
    const f16x2_t p1 = __builtin_bit_cast(f16x2_t, (w & 0x00F000F0u) | magic);
    const f16x2_t p2 = __builtin_bit_cast(f16x2_t, (w8 & 0x000F000Fu) | magic);
    const f16x2_t p3 = __builtin_bit_cast(f16x2_t, (w8 & 0x00F000F0u) | magic);
    const f16x2_t h0 = (p0 + nz) * s2;
    const f16x2_t h1 = (p1 * sixteenth + nz6) * s2;
    const f16x2_t h2 = (p2 + nz) * s2;
    const f16x2_t h3 = (p3 * sixteenth + nz6) * s2;
    return f16x8_t{h0[0], h0[1], h1[0], h1[1], h2[0], h2[1], h3[0], h3[1]};
}

// 8 signed bytes (two words) -> 8 fp16 q * s in their natural order.
//   flip = 0x80808080, sixfour = 0x64646464 (in vector registers), off = -1152 in both halves.
__device__ __forceinline__ f16x8_t expand_bytes(uint32_t w0, uint32_t w1, uint32_t flip, uint32_t sixfour, f16x2_t off,
                                                f16x2_t s2) {
    const uint32_t u0 = w0 ^ flip, u1 = w1 ^ flip;
    // v_perm_b32: bytes 0-3 of the selector pick from {second operand (bytes 0-3), first operand (bytes 4-7)}
    const f16x2_t p0 = __builtin_bit_cast(f16x2_t, __builtin_amdgcn_perm(sixfour, u0, 0x04010400u));
    const f16x2_t p1 = __builtin_bit_cast(f16x2_t, __builtin_amdgcn_perm(sixfour, u0, 0x04030402u));
    const f16x2_t p2 = __builtin_bit_cast(f16x2_t, __builtin_amdgcn_perm(sixfour, u1, 0x04010400u));
    const f16x2_t p3 = __builtin_bit_cast(f16x2_t, __builtin_amdgcn_perm(sixfour, u1, 0x04030402u));
    const f16x2_t h0 = (p0 + off) * s2, h1 = (p1 + off) * s2, h2 = (p2 + off) * s2, h3 = (p3 + off) * s2;
    return f16x8_t{h0[0], h0[1], h1[0], h1[1], h2[0], h2[1], h3[0], h3[1]};
}

// Global -> LDS copies by the load unit: lane l's 16 (or 4) bytes at base + off land at LDS
// address lds + 16 l (4 l).  Written as assembly on purpose: the compiler would otherwise
// make every later LDS read wait for all such copies in flight (it cannot see that the ring
// slots are distinct), which would drain the prefetch ring at every step.  The waits are
// explicit s_waitcnt vmcnt(n) at the points where a slot is handed over.
__device__ __forceinline__ uint32_t lds_addr(const void* p) {
    return (uint32_t)(uintptr_t)(const __attribute__((address_space(3))) void*)p;
}
__device__ __forceinline__ void dma16(const void* base, uint32_t off, uint32_t lds) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                 :: "s"(lds), "v"(off), "s"(base) : "memory", "m0");
}
__device__ __forceinline__ void dma4(const void* base, uint32_t off, uint32_t lds) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dword %1, %2"
                 :: "s"(lds), "v"(off), "s"(base) : "memory", "m0");
}

struct GemmArgs {
    const uint32_t* qw;
    const uint16_t* sc;
    const uint32_t* zr;
    const uint16_t* xh;     // [Mpad][Kpad] fp16, scaled and permuted
    const float* rscale;    // [Mpad]
    const float* wmul;      // [N]
    uint16_t* y;
    int M, N, K, Kpad, g;
    // work decomposition: tiles are numbered with m running fastest.  The first `whole` tiles
    // are dealt whole, tile i to block i % P; the K steps of the others are dealt as units (one
    // K step of one tile): block b of P owns the units [b * units / P, (b + 1) * units / P)
    int Tm, tiles, steps, whole;
    float* partial;  // [2 P][tile] fp32: sums of tiles whose K range is shared between blocks
    int block_begin, P;  // the linear is worked on by blocks [block_begin, block_begin + P) of the grid
};

// Up to kGemmBatch linears share a launch: each gets a share of the grid and is dealt to its
// blocks exactly as if it had a launch of P blocks to itself.
struct GemmBatch {
    GemmArgs it[kGemmBatch];
    int count;
};

// First unit of block b when `units` units are dealt to P blocks, and the block that owns unit u.
__host__ __device__ inline long long first_unit(long long b, long long units, int P) { return b * units / P; }
__host__ __device__ inline int owner_of(long long u, long long units, int P) { return (int)(((u + 1) * P - 1) / units); }

// Block tile (32 * MB) x (128 * WN): 4 waves side by side along n, each (32 * MB) x (32 * WN).
//
// The x tile of a step (32 * MB rows x 128 k, 256 B per row) is written into LDS by the
// load unit itself (global_load_lds_dwordx4: lane l's 16 bytes land at base + 16 l, so a
// wave fills four rows per instruction) and costs no registers.  Rows are not padded;
// instead the 16-byte chunk s of row r is kept at position s ^ (r % 16), which the
// loading lane arranges by choosing its global address, and which makes the 16 lanes of a
// fragment read (16 consecutive rows, same s) hit 16 different positions: conflict-free.
//
// Latency.  A step is only about a microsecond of matrix work, less than a trip to L2 or
// HBM under load, so the loads of step s + 2 are issued during step s: a ring of three x
// tiles (and three sets of packed weights) in LDS.  Every load is unconditional (steps past the end of K
// reload the last tile, which nothing reads), so the number of loads in flight at each
// wait is a compile-time constant and the wait is an exact vmcnt, not a drain.
//
// The K loop is one continuous pipeline of sub-steps (16 k of every lane pair = one MFMA per
// 32 x 32 output block): the LDS reads and the expansion for sub-step u + 1 are issued
// among the MFMAs of sub-step u.  The tile of step s + 1 must be complete one sub-step
// before step s ends, so the wait + barrier sits between sub-steps 6 and 7.
//
// The grid has at most one block per CU.  Tiles are dealt whole to the blocks as long as they
// fill complete rounds; what is left (fewer tiles than blocks) can be dealt in K steps instead:
// every block gets the same number of (tile, K step) units, a contiguous run of them, so no CU
// idles through a last, mostly empty round.  A block therefore works on a sequence of
// segments (a tile and a range of its K steps).  A segment that covers a tile's whole K is
// finished on the spot; otherwise its fp32 sums go to a slot of the workspace (two slots per
// block: one for its first shared segment, one for any later one) and a second kernel adds the
// slots of each such tile in K order, which keeps the result independent of timing.
constexpr int kStages = 3;

// s_waitcnt immediate: vmcnt(n), lgkmcnt(0), expcnt untouched.
__host__ __device__ constexpr int waitcnt_vm(int n) { return (n & 15) | ((n >> 4) << 14) | (7 << 4); }

//
// LW > 0: LW more waves per block that only load.  The first LW - LW / 2 of them share the x tile loads
// of a step, the other LW / 2 the weight loads (for all four column groups, with the addresses the
// owning lanes would use); each waits for the step that is due and meets the four MFMA waves at the
// step's barrier.  The MFMA waves then issue no memory instruction in the K loop: with one wave per
// SIMD every load instruction otherwise sits in the same instruction stream as the MFMAs it delays.
// A second wave on a SIMD halves the registers a wave may have (256), which the 128 x 256 tile just
// fits.  Measured on a decoder layer's four linears with nibble weights: three loading waves (two for
// x, one for the weights) are 4-9 % faster than none at every M from 33 to 2048; two are as good on
// 96-row tiles and much slower on 128-row ones (32 x loads per step from one wave), four are slower
// than three (a loading wave on every SIMD).
template <int MB, int WN, int kBits, int LW>
__global__ __launch_bounds__(256 + 64 * LW) void w4a16_gemm_f16_kernel(const GemmBatch args) {
    static_assert(LW == 0 || LW == 2 || LW == 3 || LW == 4, "no loader waves, or LW - LW / 2 for x and LW / 2 for the weights");
    constexpr int kThreads = 256 + 64 * LW;
    constexpr int kBM = 32 * MB;
    constexpr int kBN = 128 * WN;
    constexpr int kALoads = kBM / 16;             // wave-wide 1 KB loads per wave per step
    constexpr int kCodeLoads = kBits == 4 ? 2 : 4;               // 16-byte pieces of a lane's 64 codes of a step
    constexpr int kBParts = kCodeLoads + (kBits == 4 ? 2 : 1);   // ... plus the scale word and (4-bit) the zero word
    constexpr int kStepLoads = kALoads + kBParts * WN;           // all loads a lane issues per step
    constexpr int kBufBytes = kBM * 256;          // one x tile
    constexpr int kCPitch = kBN * 2 + 16;         // bytes per row of the output staging tile
    extern __shared__ __attribute__((aligned(16))) unsigned char As[];  // [kStages][kBM][256 B]

    const int t = threadIdx.x;
    const int lane = t % kWave;
    const int wave = __builtin_amdgcn_readfirstlane(t / kWave);
    const int c = lane & 31, kb = lane >> 5;
    const bool loader = LW > 0 && wave >= 4;   // wave-uniform
    int item = 0;
#pragma unroll
    for (int i = 1; i < kGemmBatch; ++i)
        if (i < args.count && (int)blockIdx.x >= args.it[i].block_begin) item = i;
    const GemmArgs ga = args.it[item];
    const int bid = (int)blockIdx.x - ga.block_begin, P = ga.P;   // this block among the linear's own
    const int G = ga.K / ga.g, zwords = (G + 7) / 8, kw = ga.K / (32 / kBits);

    uint32_t magic = kBits == 4 ? 0x64006400u : 0x64646464u;
    asm volatile("" : "+v"(magic));  // in a VGPR: v_and_or_b32 takes one scalar operand only
    uint32_t flip = 0x80808080u;
    asm volatile("" : "+v"(flip));

    const long long units = (long long)(ga.tiles - ga.whole) * ga.steps;
    const int unit0 = (int)first_unit(bid, units, P);
    const int unit1 = (int)first_unit(bid + 1, units, P);
    // Whole tiles are numbered with m running fastest, so consecutive tiles share their weight columns.
    // Where the x of all row tiles fits an L2 beside the weights passing through (2.5 MB), the blocks of
    // an XCD take consecutive tiles: workgroup b of the launch runs on XCD b mod 8, so this block's rank
    // among its linear's blocks is counted XCD by XCD.  A weight tile is then fetched by one or two L2s
    // instead of one per row tile.  Measured on a decoder layer's four linears as one launch: 2 % faster
    // with three row tiles (M = 272, 288), 3-5 % slower with two (M = 160 .. 256), which stay as they
    // were.  (Taller linears: see the dealing of eight row tiles below.)
    int vbid = bid;
    const bool x_fits_l2 = ga.Tm >= 3 && (long long)ga.Tm * kBM * ga.Kpad * 2 <= 2560 * 1024;
    // Taller linears with an even number of row tiles, where the x of two row tiles fits: the same
    // ranks, and the whole tiles are walked pair of row tiles by pair of row tiles (inside a pair column
    // by column), so that an XCD's consecutive tiles are two row tiles of a few columns.
    // Only where a round of the linear's blocks stays inside a pair (a share of a launch: all XCDs then
    // share the pair's x at the same time and each has weight columns of its own; a linear on the whole
    // grid has several pairs at once and is 7-15 % slower this way, see the dealing of eight row tiles).
    const int whole_cols = ga.whole / ga.Tm;
    // Measured on a decoder layer's four linears as one launch: 0.4 / 1.1 / 1.4 % faster with 4 / 8 / 16 row
    // tiles, 1.1 % slower with 6, which keeps the launch order.
    const bool pair_order = !x_fits_l2 && ga.Tm >= 4 && (ga.Tm & 3) == 0 && 2ll * kBM * ga.Kpad * 2 <= 2560 * 1024 &&
                            P <= 2 * whole_cols;
    if (x_fits_l2 || pair_order) {
        const int q = ga.block_begin & 7, mine = (q + bid) & 7;
        int before = 0;
        for (int x = 0; x < 8; ++x) {
            const int first = (x - q) & 7;   // the first of the linear's blocks on XCD x
            const int count = first < P ? (P - first + 7) >> 3 : 0;
            if (x < mine) before += count;
        }
        vbid = before + ((bid - ((mine - q) & 7)) >> 3);
    }
    int wtile = vbid, unit = unit0;
    for (;;) {
    // ---- one segment: K steps [ka, ka + steps) of one tile
    int tile, ka, steps;
    bool first_shared = false;
    if (wtile < ga.whole) {
        tile = wtile;
        ka = 0;
        steps = ga.steps;
        wtile += P;
    } else if (unit < unit1) {
        const int tt = unit / ga.steps;
        tile = ga.whole + tt;
        ka = unit - tt * ga.steps;
        steps = min(ga.steps - ka, unit1 - unit);
        first_shared = unit == unit0;
        unit += steps;
    } else {
        break;
    }
    const bool whole = steps == ga.steps;
    float* const pslot = ga.partial + (size_t)(2 * bid + (first_shared ? 0 : 1)) * (kBM * kBN);
    int tm = tile % ga.Tm, tn = tile / ga.Tm;
    if (pair_order && tile < ga.whole) {
        // (a last, partial column among the whole tiles keeps its order)
        if (tile < whole_cols * ga.Tm) {
            const int pair = tile / (2 * whole_cols), rem = tile - pair * 2 * whole_cols;
            tm = 2 * pair + (rem & 1);
            tn = rem >> 1;
        }
    } else if (ga.Tm == 8 && !x_fits_l2 && (P & 15) == 0 && (ga.block_begin & 7) == 0 && tile < ga.whole) {
        // Whole tiles of a linear that is eight row tiles high and has the grid to itself: in launch order
        // the eight row tiles that share a weight tile would sit on eight XCDs and every L2 would fetch
        // every weight column.  A round's P tiles (P / 8 columns) are dealt instead so that an XCD works on
        // two row tiles (their x fits its L2) and on every other column: a weight tile is then fetched by
        // four L2s, not eight.
        const int round = tile / P, idx = tile - round * P;
        const int xcd = idx & 7, j = idx >> 3;
        tm = 2 * (xcd & 3) + (j & 1);
        tn = round * (P >> 3) + 2 * (j >> 1) + (xcd >> 2);
    }
    const int bm = tm * kBM, bn = tn * kBN;

    // Byte offsets of this lane's weight rows (WN 32-column blocks).  All tensors here are
    // below 4 GB (checked by the host), so addresses are a uniform base plus a 32-bit offset.
    uint32_t qoff[WN], soff[WN], zoff[WN];
    float winv[WN];
    const int cwave = LW > 0 ? (wave & 3) : wave;   // (a loader's own values of these are not used)
#pragma unroll
    for (int j = 0; j < WN; ++j) {
        const int n = min(bn + (cwave * WN + j) * 32 + c, ga.N - 1);
        qoff[j] = (uint32_t)n * (uint32_t)kw * 4u;
        soff[j] = (uint32_t)n * (uint32_t)G * 2u;
        zoff[j] = (uint32_t)n * (uint32_t)zwords * 4u;
        winv[j] = __builtin_bit_cast(float, 0x7F000000u - __builtin_bit_cast(uint32_t, ga.wmul[n]));
    }
    const char* qbase = reinterpret_cast<const char*>(ga.qw);
    const char* sbase = reinterpret_cast<const char*>(ga.sc);
    const char* zbase = reinterpret_cast<const char*>(ga.zr);
    const char* xbase = reinterpret_cast<const char*>(ga.xh);

    // x tile loader: load i of this thread fills LDS slot (row 16 i + t / 16, position t % 16)
    // with chunk (t % 16) ^ (row % 16) of that row.
    uint32_t xoff0;
    {
        const int row0 = t >> 4, pos = t & 15;
        xoff0 = ((uint32_t)(bm + row0) * (uint32_t)ga.Kpad + (uint32_t)((pos ^ (row0 & 15)) * 8)) * 2u;
    }
    const uint32_t xstride = 16u * (uint32_t)ga.Kpad * 2u;  // 16 rows further per load
    const uint32_t as_lds = __builtin_amdgcn_readfirstlane(lds_addr(As));
    // One step's loads are issued a few at a time between the sub-steps of an earlier step
    // (all at once they would queue up behind each other in the load unit while the matrix
    // pipe idles).  plan() fixes the offsets of a step, issue(i, slot) sends its i-th load.
    uint32_t pk0b = 0;                    // x: byte offset of the step inside a row
    uint32_t pq[WN], ps[WN], pz[WN];      // weights: byte offsets of codes, scale word, zero word
    // fragment read offsets of this lane for the 8 sub-steps (row c of a 32-row block)
    // (sub-step jj < 8 only touches the low three bits of the chunk index, so it folds in by an XOR)
    const int aoff0 = c * 256 + (((8 * kb) ^ (c & 15)) << 4);

    // Weight loader: the lane's 64 k of a step (two 16-byte pieces per column block) plus the
    // 4-byte words holding its group's scale and zero-point, again through the load unit into
    // LDS: each lane only ever reads back its own slots, so LDS is a per-lane FIFO here and
    // no registers (and no compiler-inserted load waits) are tied up while the loads fly.
    // The group of a lane's 64 k is tracked without divisions (the group size is a multiple
    // of 64, so they never straddle two groups).
    unsigned char* const Bs = As + kStages * kBufBytes;  // [kStages][4 waves][WN][2560 B]
    constexpr int kBLane = kCodeLoads * 1024 + 512;       // codes, then 256 (scale) + 256 (zero)
    constexpr int kBStage = 4 * WN * kBLane;
    int lk = ka * kBK + 64 * kb, lgrp = lk / ga.g, lkin = lk - lgrp * ga.g;  // position of the next planned step
    int pstep = ka;
    auto plan = [&]() {
        pk0b = (uint32_t)(min(pstep, ga.steps - 1) * kBK) * 2u;  // past the end of K: the last tile again, unused
        ++pstep;
        const bool v = lk < ga.K;
        const uint32_t kc = v ? (uint32_t)lk : 0u;  // past the end: any valid address, the scale becomes 0
        const uint32_t grp = v ? (uint32_t)lgrp : 0u;
#pragma unroll
        for (int j = 0; j < WN; ++j) {
            pq[j] = qoff[j] + kc * kBits / 8;
            ps[j] = (soff[j] + grp * 2u) & ~3u;
            pz[j] = zoff[j] + (grp / 8u) * 4u;
        }
        lk += kBK;
        lkin += kBK;
#pragma unroll
        for (int r = 0; r < 2; ++r) {  // the step is at most two groups long
            const int over = lkin >= ga.g;
            lkin -= over * ga.g;
            lgrp += over;
        }
    };
    auto issue = [&](int i, int slot) {
        if (i < kALoads) {
            dma16(xbase, xoff0 + i * xstride + pk0b, as_lds + slot * kBufBytes + (i * 256 + cwave * 64) * 16);
        } else {
            const int j = (i - kALoads) / kBParts, part = (i - kALoads) % kBParts;
            const uint32_t dst = as_lds + kStages * kBufBytes + slot * kBStage + (cwave * WN + j) * kBLane;
            if (part < kCodeLoads) dma16(qbase, pq[j] + 16 * part, dst + 1024 * part);
            if (part == kCodeLoads) dma4(sbase, ps[j], dst + kCodeLoads * 1024);
            if (part == kCodeLoads + 1) dma4(zbase, pz[j], dst + kCodeLoads * 1024 + 256);
        }
    };

    // operands of the step being multiplied; ck / cgrp follow the consumed steps like lk / lgrp.
    // A step's codes, scale word and zero word are read back from the per-lane FIFO (take_read) and
    // turned into the expansion's constants (take_convert) in two parts, so that the reads can be in
    // flight, and the conversions issue, under the MFMAs of the previous step's last sub-step.
    uint32_t wq[WN][4 * kCodeLoads];
    uint32_t tsw[WN], tzw[WN];
    f16x2_t nz[WN], nz6[WN], s2[WN];
    int ck = ka * kBK + 64 * kb, cgrp = ck / ga.g, ckin = ck - cgrp * ga.g;
    auto take_read = [&](int stage) {
#pragma unroll
        for (int j = 0; j < WN; ++j) {
            const unsigned char* src = Bs + stage * kBStage + (cwave * WN + j) * kBLane;
#pragma unroll
            for (int pc = 0; pc < kCodeLoads; ++pc) {
                const u32x4_t v = *reinterpret_cast<const u32x4_t*>(src + pc * 1024 + lane * 16);
                wq[j][4 * pc] = v.x; wq[j][4 * pc + 1] = v.y; wq[j][4 * pc + 2] = v.z; wq[j][4 * pc + 3] = v.w;
            }
            tsw[j] = *reinterpret_cast<const uint32_t*>(src + kCodeLoads * 1024 + lane * 4);
            tzw[j] = kBits == 4 ? *reinterpret_cast<const uint32_t*>(src + kCodeLoads * 1024 + 256 + lane * 4) : 0u;
        }
    };
    auto take_convert = [&]() {
        const bool v = ck < ga.K;
        const uint32_t grp = v ? (uint32_t)cgrp : 0u;
        // past the end of K the scale becomes 0 by a factor, in a register: as a conditional value the
        // compiler turns it into a masked section, which nothing can be scheduled across
        float live = v ? 1.f : 0.f;
        asm volatile("" : "+v"(live));
#pragma unroll
        for (int j = 0; j < WN; ++j) {
            // the scale's 2 bytes inside the aligned word that was fetched
            const uint32_t sbits = (tsw[j] >> (8u * ((soff[j] + grp * 2u) & 2u))) & 0xFFFFu;
            const float sf = (float)__builtin_bit_cast(_Float16, (uint16_t)sbits);
            const float z = kBits == 4 ? (float)((tzw[j] >> (4u * (grp & 7u))) & 0xFu) : 128.f;   // bytes: the flip's 128
            const _Float16 srel = (_Float16)(sf * (winv[j] * live));
            const _Float16 a = (_Float16)(-1024.f - z), b = (_Float16)(-64.f - z);
            nz[j] = f16x2_t{a, a};
            nz6[j] = f16x2_t{b, b};
            s2[j] = f16x2_t{srel, srel};
        }
        ck += kBK;
        ckin += kBK;
#pragma unroll
        for (int r = 0; r < 2; ++r) {
            const int over = ckin >= ga.g;
            ckin -= over * ga.g;
            cgrp += over;
        }
    };

    f32x16_t acc[MB][WN];
#pragma unroll
    for (int i = 0; i < MB; ++i)
#pragma unroll
        for (int j = 0; j < WN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    f16x8_t af[2][MB], bf[2][WN];
    auto fetch = [&](int stage, int jj, int slot) {
#pragma unroll
        for (int i = 0; i < MB; ++i)
            af[slot][i] = *reinterpret_cast<const f16x8_t*>(As + stage * kBufBytes + i * (32 * 256) + (aoff0 ^ (jj << 4)));
#pragma unroll
        for (int j = 0; j < WN; ++j) {
            if constexpr (kBits == 4)
                bf[slot][j] = expand_word(wq[j][jj], magic, nz[j], nz6[j], s2[j]);
            else
                bf[slot][j] = expand_bytes(wq[j][2 * jj], wq[j][2 * jj + 1], flip, magic, nz[j], s2[j]);
        }
    };
    auto multiply = [&](int slot) {
#pragma unroll
        for (int i = 0; i < MB; ++i)
#pragma unroll
            for (int j = 0; j < WN; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(af[slot][i], bf[slot][j], acc[i][j], 0, 0, 0);
        // issue order: each MFMA is followed by one LDS read and a share of the vector
        // operations that prepare the next sub-step
#pragma unroll
        for (int u = 0; u < MB * WN; ++u) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);  // MFMA
            __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);  // LDS read
            __builtin_amdgcn_sched_group_barrier(0x002, ((kBits == 4 ? 13 : 14) * WN + MB * WN - 1) / (MB * WN), 0);  // VALU
        }
    };

    if (loader) {
        // ---- the loading waves: one barrier after the first step has landed, then one per step, as
        // the MFMA waves have them.  The first LW / 2 of them share the x tile: load q fills rows
        // 4 q + lane / 16 (chunk lane % 16 of the row at its swizzled position) and wave i takes the
        // loads q = i mod LW / 2.  The others share the 4 WN column blocks the same way: codes, scale
        // words and zero words, each lane with the offsets of the lane that will read them.
        constexpr int kXW = LW > 0 ? (LW + 1) / 2 : 1;   // waves sharing the x tile (LW = 0: this branch is never taken)
        constexpr int kWW = LW > 1 ? LW / 2 : 1;         // waves sharing the weights
        constexpr int kXLoads = kBM / 4 / kXW;           // per x wave and step
        constexpr int kWBlocks = 4 * WN / kWW;           // column blocks per weight wave
        constexpr int kWLoads = kWBlocks * kBParts;      // per weight wave and step
        static_assert(kBM / 4 % kXW == 0 && 4 % kXW == 0 && 4 * WN % kWW == 0, "loads divide evenly");
        static_assert(2 * kXLoads <= 64 && 2 * kWLoads <= 64, "two steps in flight fit the load counter (a 64th load only waits for the oldest)");
        const bool xwave = wave < 4 + kXW;
        const int share = xwave ? wave - 4 : wave - 4 - kXW;   // which of the waves of its kind
        const int lr = lane >> 4, lp = lane & 15;
        const uint32_t pitchb = (uint32_t)ga.Kpad * 2u;
        const uint32_t xrow0 = (uint32_t)(bm + 4 * share + lr) * pitchb;
        uint32_t xsw[4 / kXW];                           // swizzled chunk of load qq (period 4 rows x 4 loads)
#pragma unroll
        for (int qm = 0; qm < 4 / kXW; ++qm) xsw[qm] = (uint32_t)((lp ^ ((4 * (kXW * qm + share) + lr) & 15)) * 16);
        uint32_t qo[kWBlocks], so[kWBlocks], zo[kWBlocks];
#pragma unroll
        for (int mm = 0; mm < kWBlocks; ++mm) {
            const int n = min(bn + (kWW * mm + share) * 32 + c, ga.N - 1);
            qo[mm] = (uint32_t)n * (uint32_t)kw * 4u;
            so[mm] = (uint32_t)n * (uint32_t)G * 2u;
            zo[mm] = (uint32_t)n * (uint32_t)zwords * 4u;
        }
        int lk = ka * kBK + 64 * kb, lgrp = lk / ga.g, lkin = lk - lgrp * ga.g;
        int pstep = ka;
        auto load_step = [&](int slot) {
            const uint32_t slot_x = as_lds + (uint32_t)slot * kBufBytes + (uint32_t)share * 1024u;
            const uint32_t slot_w = as_lds + kStages * kBufBytes + (uint32_t)slot * kBStage + (uint32_t)share * kBLane;
            if (xwave) {
                const uint32_t k0b = (uint32_t)(min(pstep, ga.steps - 1) * kBK) * 2u;
#pragma unroll
                for (int qq = 0; qq < kXLoads; ++qq)
                    dma16(xbase, xrow0 + (uint32_t)(qq * kXW) * 4u * pitchb + xsw[qq % (4 / kXW)] + k0b,
                          slot_x + qq * kXW * 1024);
            } else {
                const bool v = lk < ga.K;
                const uint32_t kc = v ? (uint32_t)lk : 0u;
                const uint32_t grp = v ? (uint32_t)lgrp : 0u;
#pragma unroll
                for (int mm = 0; mm < kWBlocks; ++mm) {
                    const uint32_t dst = slot_w + mm * kWW * kBLane;
#pragma unroll
                    for (int part = 0; part < kCodeLoads; ++part)
                        dma16(qbase, qo[mm] + kc * kBits / 8 + 16 * part, dst + 1024 * part);
                    dma4(sbase, (so[mm] + grp * 2u) & ~3u, dst + kCodeLoads * 1024);
                    if (kBits == 4) dma4(zbase, zo[mm] + (grp / 8u) * 4u, dst + kCodeLoads * 1024 + 256);
                }
            }
            ++pstep;
            lk += kBK;
            lkin += kBK;
#pragma unroll
            for (int r = 0; r < 2; ++r) {
                const int over = lkin >= ga.g;
                lkin -= over * ga.g;
                lgrp += over;
            }
        };
        load_step(0);
        load_step(1);
        // in flight: steps 0 and 1; step 0 has to be complete
        if (xwave) __builtin_amdgcn_s_waitcnt(waitcnt_vm(kXLoads));
        else __builtin_amdgcn_s_waitcnt(waitcnt_vm(kWLoads));
        __syncthreads();
        int fill = 2;
        for (int s = 0; s < steps; ++s) {
            // slot `fill` held step s - 1 and is free since the previous barrier
            load_step(fill);
            fill = fill == 2 ? 0 : fill + 1;
            if (xwave) __builtin_amdgcn_s_waitcnt(waitcnt_vm(kXLoads));
            else __builtin_amdgcn_s_waitcnt(waitcnt_vm(kWLoads));
            __syncthreads();
        }
    } else {
    // steps 0 and 1 are loaded up front; from then on step s + 2 is loaded during step s
    if constexpr (LW == 0) {
#pragma unroll
        for (int p = 0; p < kStages - 1; ++p) {
            plan();
#pragma unroll
            for (int i = 0; i < kStepLoads; ++i) issue(i, p);
            __builtin_amdgcn_sched_barrier(0);
        }
        __builtin_amdgcn_s_waitcnt(waitcnt_vm(kStepLoads));
    }
    __syncthreads();
    take_read(0);
    take_convert();
    fetch(0, 0, 0);

    for (int s0 = 0; s0 < steps; s0 += kStages) {
#pragma unroll
        for (int u = 0; u < kStages; ++u) {
            if (s0 + u >= steps) break;
            const int cur = u, nxt = (u + 1) % kStages, fill = (u + 2) % kStages;
            // slot `fill` held step s - 1 and is free since the previous barrier
            if constexpr (LW == 0) plan();
#pragma unroll
            for (int jj = 0; jj < 7; ++jj) {
                __builtin_amdgcn_sched_barrier(0);
                fetch(cur, jj + 1, (jj + 1) & 1);
                multiply(jj & 1);
                __builtin_amdgcn_sched_barrier(0);
                if constexpr (LW == 0) {
#pragma unroll
                    for (int i = 0; i < kStepLoads; ++i)
                        if (i * 7 / kStepLoads == jj) issue(i, fill);
                }
            }
            __builtin_amdgcn_sched_barrier(0);
            // In flight: step s+1 (issued during step s-1) and step s+2 (just issued).  Step
            // s+1 has to be complete; the wait also covers this wave's LDS reads (lgkmcnt 0),
            // so after the barrier slot `cur` is dead for everyone once sub-step 7 is done
            // (its operands are already in registers).
            __builtin_amdgcn_s_waitcnt(waitcnt_vm(LW == 0 ? kStepLoads : 0));
            __syncthreads();
            __builtin_amdgcn_sched_barrier(0);
            // Sub-step 7 of this step (operands already in registers) with the next step's set-up under
            // it: all LDS reads first (FIFO and A fragments), a few MFMAs while they are in flight, then
            // the conversions and the first expansion shared out among the remaining MFMAs.
            take_read(nxt);
            take_convert();
            fetch(nxt, 0, 0);
#pragma unroll
            for (int i = 0; i < MB; ++i)
#pragma unroll
                for (int j = 0; j < WN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(af[1][i], bf[1][j], acc[i][j], 0, 0, 0);
            constexpr int kLead = MB * WN < 4 ? 1 : 3;                     // MFMAs issued before any conversion
            constexpr int kSetupValu = (kBits == 4 ? 13 + 16 : 14 + 12) * WN + 8;
            __builtin_amdgcn_sched_group_barrier(0x100, WN * (kCodeLoads + 2) + MB, 0);
            __builtin_amdgcn_sched_group_barrier(0x008, kLead, 0);
            if constexpr (MB * WN > kLead) {
#pragma unroll
                for (int u = 0; u < MB * WN - kLead; ++u) {
                    __builtin_amdgcn_sched_group_barrier(0x002, (kSetupValu + MB * WN - kLead - 1) / (MB * WN - kLead), 0);
                    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                }
            }
        }
    }
    }  // MFMA waves
    __builtin_amdgcn_sched_barrier(0);
    __builtin_amdgcn_s_waitcnt(waitcnt_vm(0));  // nothing may still be writing LDS
    __syncthreads();

    if (!whole) {
        // part of a tile's K: the raw sums go to this block's slot, tile-shaped [kBM][kBN],
        // through LDS so that they leave as 16-byte pieces of full lines
        constexpr int kPPitch = kBN + 4;  // floats per staged row
        static_assert(kBM * kPPitch * 4 <= kStages * (kBufBytes + 4 * WN * kBLane), "the fp32 tile fits in the ring");
        float* const stage = reinterpret_cast<float*>(As) + (4 * kb) * kPPitch + cwave * WN * 32 + c;
        if (!loader) {
#pragma unroll
            for (int j = 0; j < WN; ++j)
#pragma unroll
                for (int i = 0; i < MB; ++i)
#pragma unroll
                    for (int r = 0; r < 16; ++r)
                        stage[(i * 32 + 8 * (r / 4) + (r % 4)) * kPPitch + j * 32] = acc[i][j][r];
        }
        __syncthreads();
        for (int idx = t; idx < kBM * (kBN / 4); idx += kThreads) {
            const int row = idx / (kBN / 4), c4 = idx % (kBN / 4);
            *reinterpret_cast<f32x4_t*>(pslot + row * kBN + c4 * 4) =
                *reinterpret_cast<const f32x4_t*>(reinterpret_cast<const float*>(As) + row * kPPitch + c4 * 4);
        }
        // the next segment counts its loads in flight exactly and reuses LDS
        __builtin_amdgcn_s_waitcnt(waitcnt_vm(0));
        __syncthreads();
        continue;
    }
    // y = acc * 2^-p(m) * 2^E(n), rounded once to bf16, staged in LDS so that rows leave as
    // 16-byte pieces of full lines.
    if (!loader) {
    float wm[WN];
#pragma unroll
    for (int j = 0; j < WN; ++j) wm[j] = ga.wmul[min(bn + (cwave * WN + j) * 32 + c, ga.N - 1)];
    // the row factors of the lane's 16 MB rows, four neighbouring rows per load, all requested before
    // the first is used (fetched where they are used, each load waited for the one before it: 4 MB
    // round trips per tile)
    f32x4_t rsv[MB][4];
#pragma unroll
    for (int i = 0; i < MB; ++i)
#pragma unroll
        for (int qd = 0; qd < 4; ++qd)
            rsv[i][qd] = *reinterpret_cast<const f32x4_t*>(ga.rscale + bm + i * 32 + 8 * qd + 4 * kb);
#pragma unroll
    for (int i = 0; i < MB; ++i)
#pragma unroll
        for (int r = 0; r < 16; r += 2) {
            // registers r and r + 1 are two neighbouring rows of the lane's column
            const int row = i * 32 + 8 * (r / 4) + 4 * kb + (r % 4);
            const float rs0 = rsv[i][r / 4][r % 4], rs1 = rsv[i][r / 4][r % 4 + 1];
#pragma unroll
            for (int j = 0; j < WN; ++j) {
                const int col = (cwave * WN + j) * 32 + c;
                const uint32_t h = f32x2_to_bf16x2_rne(acc[i][j][r] * rs0 * wm[j], acc[i][j][r + 1] * rs1 * wm[j]);
                *reinterpret_cast<uint16_t*>(As + row * kCPitch + col * 2) = (uint16_t)h;
                *reinterpret_cast<uint16_t*>(As + (row + 1) * kCPitch + col * 2) = (uint16_t)(h >> 16);
            }
        }
    }
    __syncthreads();
    constexpr int kChunks = kBN / 8;  // 16-byte pieces per row
    const bool vec_ok = (ga.N % 8) == 0;
    for (int idx = t; idx < kBM * kChunks; idx += kThreads) {
        const int row = idx / kChunks, ch = idx % kChunks;
        const int m = bm + row, n = bn + ch * 8;
        if (m >= ga.M || n >= ga.N) continue;
        const u32x4_t v = *reinterpret_cast<const u32x4_t*>(As + row * kCPitch + ch * 16);
        uint16_t* dst = ga.y + (size_t)m * ga.N + n;
        if (vec_ok && n + 8 <= ga.N) {
            *reinterpret_cast<u32x4_t*>(dst) = v;
        } else {
            const uint32_t w[4] = {v.x, v.y, v.z, v.w};
            for (int e = 0; e < 8 && n + e < ga.N; ++e) dst[e] = (uint16_t)(w[e / 2] >> (16 * (e & 1)));
        }
    }
    __builtin_amdgcn_s_waitcnt(waitcnt_vm(0));
    __syncthreads();  // the staging tile is about to be overwritten by the next segment's loads
    }  // segments
}

// Adds up the slots of every tile whose K range was shared between blocks (in K order) and
// finishes it like the main kernel does: y = sum * 2^-p(m) * 2^E(n), rounded once to bf16.
// Grid: (tiles dealt in K steps, pieces of 256 4-float groups per tile, linears); a thread owns one group.
template <int MB, int WN>
__global__ __launch_bounds__(256) void w4a16_gemm_fixup_kernel(const GemmBatch args) {
    constexpr int kBM = 32 * MB, kBN = 128 * WN;
    static_assert((kBM * kBN / 4) % 256 == 0, "tiles split into whole pieces");
    const int t = threadIdx.x, lane = t % kWave, wave = t / kWave;
    const GemmArgs ga = args.it[blockIdx.z];
    const int P = ga.P;
    if ((int)blockIdx.x >= ga.tiles - ga.whole) return;   // the grid is as wide as the largest tail
    const int tile = ga.whole + blockIdx.x;
    const long long units = (long long)(ga.tiles - ga.whole) * ga.steps;
    const long long u_first = (long long)blockIdx.x * ga.steps, u_last = u_first + ga.steps - 1;
    const int b_lo = owner_of(u_first, units, P), b_hi = owner_of(u_last, units, P);
    if (b_lo == b_hi) return;  // one block had the whole tile and has finished it

    // The slots to add, in K order, worked out once per block (the divisions are slow) and
    // packed, so that the loads below can be issued several at a time.
    __shared__ int slots[kMaxGemmBlocks];
    __shared__ int wave_count[4];
    int count = 0;
    for (int b0 = b_lo; b0 <= b_hi; b0 += 256) {
        const int b = b0 + t;
        int sl = -1;  // with fewer units than blocks some blocks own none
        if (b <= b_hi) {
            const long long fu = first_unit(b, units, P);
            // a block's first shared segment is in its slot 0, a later one in slot 1
            if (fu != first_unit(b + 1, units, P)) sl = 2 * b + ((int)blockIdx.x == (int)(fu / ga.steps) ? 0 : 1);
        }
        const unsigned long long have = __ballot(sl >= 0);
        if (lane == 0) wave_count[wave] = __popcll(have);
        __syncthreads();
        int at = count + __popcll(have & ((1ull << lane) - 1ull));
        for (int w = 0; w < wave; ++w) at += wave_count[w];
        if (sl >= 0) slots[at] = sl;
        count += wave_count[0] + wave_count[1] + wave_count[2] + wave_count[3];
        __syncthreads();
    }

    const int idx = blockIdx.y * 256 + t;
    const int row = idx / (kBN / 4), c4 = idx % (kBN / 4);
    const int m = (tile % ga.Tm) * kBM + row, n = (tile / ga.Tm) * kBN + c4 * 4;
    if (m >= ga.M || n >= ga.N) return;
    const float* src = ga.partial + row * kBN + c4 * 4;
    f32x4_t sum = {0.f, 0.f, 0.f, 0.f};
    int i = 0;
    for (; i + 4 <= count; i += 4) {
        f32x4_t v[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) v[e] = *reinterpret_cast<const f32x4_t*>(src + (size_t)slots[i + e] * (kBM * kBN));
#pragma unroll
        for (int e = 0; e < 4; ++e) sum += v[e];
    }
    for (; i < count; ++i) sum += *reinterpret_cast<const f32x4_t*>(src + (size_t)slots[i] * (kBM * kBN));
    const float rs = ga.rscale[m];
    uint16_t* dst = ga.y + (size_t)m * ga.N + n;
    uint16_t h[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) h[e] = f32_to_bf16_rne(sum[e] * rs * ga.wmul[min(n + e, ga.N - 1)]);
    if ((ga.N % 4) == 0) {
        *reinterpret_cast<uint2*>(dst) = make_uint2(h[0] | ((uint32_t)h[1] << 16), h[2] | ((uint32_t)h[3] << 16));
    } else {
        for (int e = 0; e < 4 && n + e < ga.N; ++e) dst[e] = h[e];
    }
}

int gemm_max_blocks() { return device_cu_count() < kMaxGemmBlocks ? device_cu_count() : kMaxGemmBlocks; }

// Fills in the work decomposition of one linear on `cus` blocks; returns the blocks it uses.
template <int MB, int WN>
int plan_tiles(GemmArgs& ga, bool split_tail, int cus) {
    constexpr int kBM = 32 * MB, kBN = 128 * WN;
    ga.Tm = (ga.M + kBM - 1) / kBM;
    ga.tiles = ga.Tm * ((ga.N + kBN - 1) / kBN);
    ga.steps = ga.Kpad / kBK;
    ga.whole = split_tail ? ga.tiles / cus * cus : ga.tiles;
    const int tail = ga.tiles - ga.whole;
    const long long units = (long long)tail * ga.steps;
    int P = ga.whole >= cus ? cus : ga.whole;
    if (tail > 0 && P < cus) P = units < cus ? (int)units : cus;  // here whole == 0
    ga.P = P;
    return P;
}

// One launch for `n` linears that use the same tile, each on its own blocks (ga[i].block_begin, P set).
// Loading waves per block (see the kernel), by code width.
constexpr int kLoaderWaves4 = 3, kLoaderWaves8 = 0;
template <int MB, int WN, int kBits, int LW = (kBits == 4 ? kLoaderWaves4 : kLoaderWaves8)>
hipError_t launch_tile(const GemmArgs* gas, int n, hipStream_t st) {
    constexpr int kBM = 32 * MB, kBN = 128 * WN;
    const size_t lds = (size_t)kStages * (kBM * 256 + 4 * WN * ((kBits == 4 ? 2 : 4) * 1024 + 512));
    // more than 64 KB of LDS needs an opt-in; the call is idempotent, so two host threads that
    // both find the flag clear may both make it
    static std::atomic<bool> attr_set{false};
    if (!attr_set.load(std::memory_order_acquire)) {
        const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&w4a16_gemm_f16_kernel<MB, WN, kBits, LW>),
                                                 hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
        attr_set.store(true, std::memory_order_release);
    }
    GemmBatch gb;
    int grid = 0, max_tail = 0;
    for (int i = 0; i < kGemmBatch; ++i) {
        gb.it[i] = gas[i < n ? i : n - 1];
        if (i < n) {
            grid += gas[i].P;
            // the second kernel is only needed when some block boundary falls inside a tile
            const int tail = gas[i].tiles - gas[i].whole;
            const long long units = (long long)tail * gas[i].steps;
            bool shared = false;
            for (int b = 1; b < gas[i].P && tail > 0 && !shared; ++b) shared = first_unit(b, units, gas[i].P) % gas[i].steps != 0;
            if (shared && tail > max_tail) max_tail = tail;
        }
    }
    gb.count = n;
    hipLaunchKernelGGL((w4a16_gemm_f16_kernel<MB, WN, kBits, LW>), dim3(grid), dim3(256 + 64 * LW), lds, st, gb);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    if (max_tail > 0) {
        hipLaunchKernelGGL((w4a16_gemm_fixup_kernel<MB, WN>), dim3(max_tail, kBM * kBN / 4 / 256, n), dim3(256), 0, st, gb);
        e = hipGetLastError();
    }
    return e;
}

// Tile width and the treatment of the last, incomplete round of tiles, for a linear that has
// `cus` blocks to itself.
template <int MB>
void choose_tile(const GemmArgs& ga, int cus, bool alone, bool narrow_only, int* wn_out, bool* split_out) {
    if (narrow_only) {
        // 8-bit codes: the ring fits LDS only with 128-column tiles.  A round or more of them: the
        // incomplete last round in K steps when it is short; less than a round: everything in K steps.
        const int t1 = ((ga.M + 32 * MB - 1) / (32 * MB)) * ((ga.N + 127) / 128);
        *wn_out = 1;
        *split_out = t1 < cus ? true : (t1 % cus) * 5 <= cus * 2;
        return;
    }
    // Measured on the four linears of a 7B decoder layer at M = 288 and 1024 (256 CUs), one launch each:
    //   * a round or more of wide tiles: wide tiles, and the incomplete last round is dealt in
    //     K steps only when it is short (a fuller one is cheaper left as it is: blocks that
    //     share tiles pay for slots and a second kernel, and a chip that is not full clocks higher);
    //   * between half a round and a round of wide tiles: wide tiles, whole;
    //   * less: narrow tiles (twice as many), dealt in K steps when K is long or the tiles are few.
    // A linear that shares the launch with others has only its share of the blocks, which it must
    // keep busy to the end because the others cannot use them: less than a round of wide tiles is
    // dealt in K steps, and as narrow tiles when M is a single tile high (measured 3-6 % faster than
    // wide ones at M = 17 .. 128, 2-9 % slower at M = 200 and 288).
    const int t2 = ((ga.M + 32 * MB - 1) / (32 * MB)) * ((ga.N + 255) / 256);
    int wn = 2;
    bool split = false;
    if (ga.N <= 128) {
        wn = 1;
        split = ga.Kpad / kBK >= 64;
    } else if (t2 >= cus) {
        split = (t2 % cus) * 5 <= cus * 2;
    } else if (!alone) {
        wn = ga.M <= 32 * MB ? 1 : 2;
        split = true;
    } else if (t2 * 2 <= cus) {
        wn = 1;
        // in K steps when K is long, or when whole narrow tiles would leave half of the CUs idle
        // (measured on single linears at M = 48 .. 288: the out projection 27 -> 19 us at M = 64,
        // 37 -> 25 us at M = 128; with more tiles than that the shared tiles cost more than they give)
        split = ga.Kpad / kBK >= 64 || (t2 * 4 <= cus && ga.Kpad / kBK >= 16);
    }
    *wn_out = wn;
    *split_out = split;
}

// tile height: the multiple of 32 rows (at most 128) that pads M least
int tile_rows(int M) {
    if (M <= 96) return round_up(M, 32);
    return round_up(M, 96) < round_up(M, 128) ? 96 : 128;
}

}  // namespace

bool gemm_f16_supports(const qail_wdesc& d, int M) {
    if (d.K % 64 != 0 || d.group_size % 64 != 0) return false;
    // A scale is fetched as the aligned 4-byte word that holds it; with an odd number of scales
    // the word of the last one would reach two bytes past the caller's buffer.
    if (((unsigned long long)d.N * (unsigned long long)(d.K / d.group_size)) % 2 != 0) return false;
    // 32-bit byte offsets inside the kernel
    const unsigned long long lim = 0xFFFFFFFFull;
    const unsigned long long Mpad = (unsigned long long)round_up(M, kRowPad), Kpad = (unsigned long long)round_up(d.K, kBK);
    const unsigned long long code_bytes = (unsigned long long)d.N * d.K / (d.scheme == QAIL_W8_SYM_GROUP ? 1 : 2);
    return code_bytes <= lim && Mpad * Kpad * 2 <= lim && (unsigned long long)M * d.N * 2 <= lim;
}

// Workspace of one linear without the slots: x as fp16, the row scales, the weight rows' powers of two.
static size_t gemm_head_bytes(const qail_wdesc& d, int M) {
    const size_t Mpad = (size_t)round_up(M, kRowPad), Kpad = (size_t)round_up(d.K, kBK);
    const size_t b = Mpad * Kpad * 2 + Mpad * 4 + (size_t)round_up(d.N, 64) * 4;
    return (b + 255) / 256 * 256;
}

// Two tile-shaped fp32 slots per block of the grid for tiles whose K range is shared between blocks.
static size_t gemm_slot_bytes(int M, bool wide) {   // wide: 256-column tiles (4-bit codes with N > 128)
    return 2 * (size_t)gemm_max_blocks() * (size_t)tile_rows(M) * (wide ? 256 : 128) * 4;
}

size_t gemm_f16_workspace(const qail_wdesc& d, int M) {
    return gemm_head_bytes(d, M) + gemm_slot_bytes(M, d.N > 128 && d.scheme != QAIL_W8_SYM_GROUP);
}

size_t gemm_f16_batch_workspace(const qail_w4a16_item* items, int count, int M) {
    // linears that share a launch (kGemmBatch at a time) need their heads side by side; the
    // slots are shared out with the blocks
    size_t need = 0;
    for (int i0 = 0; i0 < count; i0 += kGemmBatch) {
        size_t b = 0;
        bool wide = false;
        for (int i = i0; i < count && i < i0 + kGemmBatch; ++i) {
            b += gemm_head_bytes(items[i].d, M);
            wide = wide || (items[i].d.N > 128 && items[i].d.scheme != QAIL_W8_SYM_GROUP);
        }
        b += gemm_slot_bytes(M, wide);
        if (b > need) need = b;
    }
    return need;
}

template <int MB>
static hipError_t launch_chunk(const qail_w4a16_item* items, int n, int M, void* ws, hipStream_t st) {
    const bool bytes = items[0].d.scheme == QAIL_W8_SYM_GROUP;   // all items of a call have the same code width
    const int Mpad = round_up(M, kRowPad);
    const int cus = gemm_max_blocks();
    GemmArgs ga[kGemmBatch];
    PrepBatch pb;
    pb.M = M;
    pb.Mpad = Mpad;
    pb.natural = bytes ? 1 : 0;
    char* at = static_cast<char*>(ws);
    int prep_blocks = 0;
    for (int i = 0; i < n; ++i) {
        const qail_wdesc& d = items[i].d;
        const int Kpad = round_up(d.K, kBK), G = d.K / d.group_size;
        uint16_t* xh = reinterpret_cast<uint16_t*>(at);
        float* rscale = reinterpret_cast<float*>(xh + (size_t)Mpad * Kpad);
        float* wmul = rscale + Mpad;
        at += gemm_head_bytes(d, M);
        pb.it[i] = PrepItem{items[i].x, items[i].scales, xh, rscale, wmul, d.N, d.K, Kpad, G};
        ga[i] = GemmArgs{items[i].qweight, items[i].scales, items[i].zeros, xh, rscale, wmul, items[i].y,
                         M, d.N, d.K, Kpad, d.group_size, 0, 0, 0, 0, nullptr, 0, 0};
        prep_blocks = std::max(prep_blocks, Mpad + (d.N + 31) / 32);
    }
    for (int i = n; i < kGemmBatch; ++i) pb.it[i] = pb.it[n - 1];
    float* slots = reinterpret_cast<float*>(at);
    hipLaunchKernelGGL(gemm_prep_kernel, dim3(prep_blocks, n), dim3(256), 0, st, pb);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;

    // every linear gets blocks in proportion to its weights (at least one), then its own tiling
    int share[kGemmBatch], wn[kGemmBatch];
    bool split[kGemmBatch];
    auto deal = [&](const int* idx, int m, int avail) {
        double sum = 0;
        for (int j = 0; j < m; ++j) sum += (double)items[idx[j]].d.N * items[idx[j]].d.K;
        int used = 0;
        for (int j = 0; j < m; ++j) {
            const int i = idx[j];
            share[i] = std::max(1, (int)((double)items[i].d.N * items[i].d.K / sum * avail));
            used += share[i];
        }
        for (int j = 0; used < avail; j = (j + 1) % m, ++used) ++share[idx[j]];
        while (used > avail) {   // the floors of one block each were too many: take from the largest
            int big = idx[0];
            for (int j = 1; j < m; ++j)
                if (share[idx[j]] > share[big]) big = idx[j];
            --share[big];
            --used;
        }
    };
    int all[kGemmBatch];
    for (int i = 0; i < n; ++i) all[i] = i;
    deal(all, n, std::max(cus, n));
    for (int i = 0; i < n; ++i) choose_tile<MB>(ga[i], share[i], n == 1, bytes, &wn[i], &split[i]);
    // linears with the same tile width go out together, each group on the whole chip
    for (int w = 2; w >= 1; --w) {
        int idx[kGemmBatch], m = 0;
        for (int i = 0; i < n; ++i)
            if (wn[i] == w) idx[m++] = i;
        if (m == 0) continue;
        if (m < n) {
            deal(idx, m, std::max(cus, m));
            for (int j = 0; j < m; ++j) {
                int w2;
                choose_tile<MB>(ga[idx[j]], share[idx[j]], n == 1, bytes, &w2, &split[idx[j]]);
            }
        }
        GemmArgs grp[kGemmBatch];
        int begin = 0;
        for (int j = 0; j < m; ++j) {
            GemmArgs& g = ga[idx[j]];
            const int P = w == 2 ? plan_tiles<MB, 2>(g, split[idx[j]], share[idx[j]]) : plan_tiles<MB, 1>(g, split[idx[j]], share[idx[j]]);
            g.block_begin = begin;
            g.partial = slots + (size_t)2 * begin * (32 * MB) * (128 * w);
            begin += P;
            grp[j] = g;
        }
        e = bytes ? launch_tile<MB, 1, 8>(grp, m, st)
                  : (w == 2 ? launch_tile<MB, 2, 4>(grp, m, st) : launch_tile<MB, 1, 4>(grp, m, st));
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

hipError_t launch_w4a16_gemm_f16_batch(const qail_w4a16_item* items, int count, int M, void* ws, hipStream_t st) {
    for (int i0 = 0; i0 < count; i0 += kGemmBatch) {
        const int n = std::min(kGemmBatch, count - i0);
        hipError_t e;
        switch (tile_rows(M)) {
            case 32: e = launch_chunk<1>(items + i0, n, M, ws, st); break;
            case 64: e = launch_chunk<2>(items + i0, n, M, ws, st); break;
            case 96: e = launch_chunk<3>(items + i0, n, M, ws, st); break;
            default: e = launch_chunk<4>(items + i0, n, M, ws, st); break;
        }
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

hipError_t launch_w4a16_gemm_f16(const qail_w4a16_item& it, int M, void* ws, hipStream_t st) {
    return launch_w4a16_gemm_f16_batch(&it, 1, M, ws, st);
}

}  // namespace qail
