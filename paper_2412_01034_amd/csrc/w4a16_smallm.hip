// W4A16 linear for a small batch, 2 <= M <= 16: y[m][n] = sum_k x[m][k] (q[n][k] - z[n][k/g]) s[n][k/g].
//
// Appendix "Analysis": decode is bound by streaming the packed weights; with a few
// sequences decoded together the weights are still read once, so the kernel keeps the
// structure of the M = 1 stream and lets the matrix cores serve all M rows of x at once.
//
//   * A tile is 16 weight rows.  For v_mfma_f32_16x16x32_bf16 lane l = 16*kb + i supplies, as
//     B operand, 8 consecutive k of column (weight row) i starting at 8*kb: exactly one packed
//     word.  A lane loads 16 bytes = 4 words = 32 k of its row, so one wave-wide load covers
//     16 rows x 128 k (64 contiguous bytes per row) and feeds 4 MFMAs; 128 k lies inside one
//     quantisation group (group_size is a multiple of 128), so the group's scale and
//     zero-point are applied to the 16 x 16 result of those 4 MFMAs:
//         sum_k x (q - z) s = s * ( sum_k x (q + 128)  -  (128 + z) * sum_k x )
//     with (q + 128) as bf16 = 0x4300 | q (one AND-OR per nibble pair) and sum_k x per
//     (row of x, 128-k step) computed once per block.
//   * The activations of the block's linear are staged once in LDS as ready-made A operands
//     (all of K when M * K * 2 bytes fit in 128 KB, else pass by pass), so a wave can walk any
//     stretch of K of a tile without holding x in registers and the stream has no barrier.
//   * Two kernels.  Group size 128 with an even number of groups per row (every shape of the
//     7B model): smallm_stream_kernel, whose description stands in front of it.  Other group
//     sizes: w4a16_smallm_general_kernel, in which a block owns at most 16 tiles, its 16 waves
//     are dealt to (tile, K part) pairs and every step fetches its own scale and zero-point.
//     Both keep a ring of loads in flight with exact load waits (unconditional loads, program
//     order = consumption order, nothing stored while loads fly); K parts' 16 x 16 partial
//     results meet once, after the stream, in LDS and are added in a fixed order.
//   * As for M = 1, one launch serves a list of linears, blocks divided by bytes.
#include <string.h>

#include <algorithm>
#include <atomic>

#include "qail_internal.h"

namespace qail {

namespace {

constexpr int kSmMaxItems = 16;
constexpr int kSmWaves = 16;
constexpr int kSmThreads = kSmWaves * kWave;
constexpr int kStepK = 128;               // k per wave-wide load
constexpr int kRing = 8;                  // wave-wide loads in flight per wave
constexpr int kXBytes = 32 * 16 * 17 * 16; // LDS for the staged activations: M = 16 at K = 4096 in one pass
constexpr int kTilesPerBlock = 16;

// 64 bytes, so that a block fetches everything it needs to know with one scalar load.
struct SmItem {
    const uint32_t* qw;
    const uint16_t* sc;
    const uint32_t* zr;
    const uint16_t* x;
    uint16_t* y;
    int N, K, g;
    int block_begin;  // first block of the grid that works on this item
    int tiles_base;   // block b of the item owns tiles_base tiles, one more if b < tiles_rem,
    int tiles_rem;    // in the order of the blocks
};

constexpr int kSmMaxBlocks = 4096;  // blocks of a launch that serves more than one item

// What the kernel with one group per step needs to know about an item's division of labour and
// would otherwise divide for: worked out on the host (a CU has one scalar unit for its 16 waves,
// and a dozen integer divisions per wave held the first load back by microseconds).
struct SmPlan {
    uint16_t rows, pass_steps, npass, last_steps;   // rows per LDS block; steps of a pass / of the last pass
    uint32_t inv_steps[2];   // ceil(2^32 / steps) of a full pass [0] and of the last pass [1]: p / steps = mulhi(p, inv) for p < 2^16
    uint16_t r64[2];         // 64 % steps
    uint8_t q64[2];          // 64 / steps
    uint8_t ks[2];           // K parts per tile in a block of tiles_base [0] / tiles_base + 1 [1] tiles
    uint8_t gshift[2];       // K parts are whole chunks of 8 >> gshift steps of the ring (8, 4 or 2)
    uint32_t inv_ks[2];      // ceil(2^16 / ks): v / ks = (v * inv) >> 16 for v <= 4096
};

struct SmArgs {
    SmItem it[kSmMaxItems];
    uint32_t item_of_block[kSmMaxBlocks / 8];  // 4 bits per block; blocks past the table work on item 0
    int M;
    SmPlan plan[kSmMaxItems];   // read by the kernel with one group per step only
};

// LDS: [kXBytes] activations (after the stream: [16 waves][256] fp32 partials), [max steps per pass][16]
// fp32 step sums.
constexpr int kMaxPassSteps = kXBytes / (16 * 3 * 16) + 6;  // M >= 2 (3 rows per block): steps per pass, rounded up
constexpr size_t kSmLdsBytes = (size_t)kXBytes + (size_t)kMaxPassSteps * 16 * 4;
static_assert(kSmWaves * 2 * 256 * 4 <= kXBytes, "the partial tiles (two row blocks) reuse the activations' space");

// Rows per LDS block and 128-k steps per pass over K for a batch of M rows and S steps in all.
// Rows beyond M read a row of zeros appended to every block (M = 16 needs none).  A block holds
// an odd number of 16-byte rows, so that the 16 pieces of one row of x in one step, which 16
// neighbouring threads write into the step's 16 blocks, fall into 16 different groups of LDS
// banks -- unless that costs a pass more over K.  A pass is at most 512 (row, step) pairs, so
// that its x travels through 8 registers per thread.
__host__ __device__ inline void sm_plan(int M, int S, int* rows, int* pass_steps) {
    const int rmin = M % 16 == 0 ? M : M + 1;
    const int cap = 512 / M;
    // a pass that is not the whole of K is a multiple of eight steps, so that every pass starts at one
    auto whole = [&](int steps) { return steps >= S ? S : (steps >= 8 ? steps & ~7 : steps); };
    const int smin = whole(min(kXBytes / (256 * rmin), cap)), sodd = whole(min(kXBytes / (256 * (rmin | 1)), cap));
    const bool odd = (S + sodd - 1) / sodd <= (S + smin - 1) / smin;
    *rows = odd ? (rmin | 1) : rmin;
    *pass_steps = odd ? sodd : smin;
}

__global__ __launch_bounds__(kSmThreads) void w4a16_smallm_general_kernel(const SmArgs args) {
    extern __shared__ __attribute__((aligned(16))) unsigned char sm_lds[];
    unsigned char* xl = sm_lds;
    float* xs_tab = reinterpret_cast<float*>(sm_lds + kXBytes);
    float* partial = reinterpret_cast<float*>(sm_lds);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
    const int lane = threadIdx.x % kWave;
    const int li = lane & 15, kb = lane >> 4;
    const int M = args.M;

    // two dependent scalar loads and no division between the start of the block and its first
    // weight load: the block's item from a 4-bit table, then the item's 64-byte record
    int idx = 0;
    if (blockIdx.x < (unsigned)kSmMaxBlocks) idx = (args.item_of_block[blockIdx.x / 8] >> (4 * (blockIdx.x % 8))) & 15;
    idx = __builtin_amdgcn_readfirstlane(idx);
    const SmItem it = args.it[idx];
    const int K = it.K, N = it.N, g = it.g;
    const int G = K / g, zwords = (G + 7) / 8, kw = K / 8;
    const int b = (int)blockIdx.x - it.block_begin;
    const int tile0 = b * it.tiles_base + min(b, it.tiles_rem);
    const int nt = it.tiles_base + (b < it.tiles_rem ? 1 : 0);   // at most kTilesPerBlock (the launcher sees to it)
    if (nt <= 0) return;            // block-uniform

    // (tile, K part) of this wave: as many K parts as keep the 16 waves busy
    const int ksplit = kSmWaves / nt;
    const int slot = wave / ksplit, kpart = wave % ksplit;
    const bool active = slot < nt;
    const int S = K / kStepK;
    const int my0 = (int)(((long long)S * kpart) / ksplit), my1 = (int)(((long long)S * (kpart + 1)) / ksplit);
    const int row = min((tile0 + min(slot, nt - 1)) * 16 + li, N - 1);

    // LDS layout of x: block (step, j, kb) holds, for each row m, the 16 bytes that lane (m, kb)
    // feeds to MFMA j of that step: x[m][128 step + 32 kb + 8 j + (0..7)] in the pair order
    // x0,x4 | x1,x5 | x2,x6 | x3,x7 that the nibble expansion produces.
    int Mp, pass_steps;
    sm_plan(M, S, &Mp, &pass_steps);
    const int step_bytes = 16 * Mp * 16;                       // 16 (j, kb) blocks per step
    const int npass = (S + pass_steps - 1) / pass_steps;
    const int xrow = min(li, M) * 16;                          // this lane's row inside a block (li <= 15)

    uint32_t magic = 0x43004300u;    // bf16 pair (128, 128); in a vector register so that the
    asm volatile("" : "+v"(magic));  // AND-OR needs only one scalar operand

    f32x4_t acc = {0.f, 0.f, 0.f, 0.f};

    // register ring of wave-wide weight loads
    uint4 q[kRing];
    _Float16 sh[kRing];  // kept in its loaded type: a widening at the load would wait there
    uint32_t zw[kRing];
    // addresses as a uniform base plus a 32-bit byte offset (the launcher checks that the tensors
    // are below 4 GB); the group of a step is a shift when a group is a power-of-two number of steps
    const char* qbase = reinterpret_cast<const char*>(it.qw);
    const char* sbase = reinterpret_cast<const char*>(it.sc);
    const char* zbase = reinterpret_cast<const char*>(it.zr);
    const uint32_t qoff = (uint32_t)row * (uint32_t)kw * 4u + 16u * kb;
    const uint32_t soff = (uint32_t)row * (uint32_t)G * 2u;
    const uint32_t zoff = (uint32_t)row * (uint32_t)zwords * 4u;
    const int spg = g / kStepK;                                   // steps per group
    const int gshift = __builtin_ctz(spg);                         // spg is a power of two (host check)
    auto group_of = [&](int step) { return step >> gshift; };
    auto issue = [&](int p, int step) {
        const uint32_t grp = (uint32_t)group_of(step);
        q[p] = *reinterpret_cast<const uint4*>(qbase + (qoff + (uint32_t)step * (kStepK / 2)));
        sh[p] = *reinterpret_cast<const _Float16*>(sbase + (soff + grp * 2u));
        zw[p] = *reinterpret_cast<const uint32_t*>(zbase + (zoff + (grp >> 3) * 4u));
    };
    auto prologue = [&](int k0, int k1) {
#pragma unroll
        for (int p = 0; p < kRing; ++p) {
            issue(p, min(k0 + p, k1 - 1));  // slots past the end re-read the last step and are not consumed
            __builtin_amdgcn_sched_barrier(0);  // program order = consumption order
        }
    };
    // Staging: 16 neighbouring threads take the 16 pieces (16 bytes each) of one (step, row) pair,
    // pair p = step * M + row; p / M for p < 4096 is a multiplication.
    const uint32_t inv_m = (65536u + (uint32_t)M - 1u) / (uint32_t)M;
    const int tg = threadIdx.x >> 4, t16 = threadIdx.x & 15;
    const int blk_off = ((t16 & 3) * 4 + (t16 >> 2)) * (Mp * 16);   // block (j, kb) of piece 4 kb + j
    uint4 xr[8];
    const char* xbase = reinterpret_cast<const char*>(it.x);   // M * K < 2^31 elements: 32-bit offsets

    for (int pass = 0; pass < npass; ++pass) {
        const int p0 = pass * pass_steps, p1 = min(S, p0 + pass_steps);
        const int pairs = (p1 - p0) * M;
        if (pass) __syncthreads();  // the previous pass's activations are no longer read
        // ---- the pass's x is requested first, then the first weights of the pass: loads return
        // in order, x is needed first, and the staging then hides the weights' latency
        int tg1 = tg;                    // worked out per pass rather than kept in registers
        asm volatile("" : "+v"(tg1));
        // (every load is issued, a pair past the last one re-reads the last: behind a condition each
        // load waits for the one before it)
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int pi = min(tg1 + 64 * u, pairs - 1);
            const int sx = (int)(((uint32_t)pi * inv_m) >> 16), m = pi - sx * M;
            xr[u] = *reinterpret_cast<const uint4*>(xbase + ((uint32_t)(m * K + (p0 + sx) * kStepK + t16 * 8) * 2u));
        }
        __builtin_amdgcn_sched_barrier(0);
        const int k0 = max(my0, p0), k1 = min(my1, p1);
        const int n = active ? max(0, k1 - k0) : 0;
        if (n > 0) prologue(k0, k1);
        // ---- stage x[:, 128 p0 .. 128 p1), its sums over each step, and the zero rows
        int tg2 = tg;                    // the pairs are worked out again rather than kept in
        asm volatile("" : "+v"(tg2));    // registers across the loads
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int pi = tg2 + 64 * u;
            if (pi < pairs) {
                const int sx = (int)(((uint32_t)pi * inv_m) >> 16), m = pi - sx * M;
                const uint4 v = xr[u];
                uint4 o;
                o.x = (v.x & 0xFFFFu) | (v.z << 16);      // x0,x4
                o.y = (v.x >> 16) | (v.z & 0xFFFF0000u);  // x1,x5
                o.z = (v.y & 0xFFFFu) | (v.w << 16);      // x2,x6
                o.w = (v.y >> 16) | (v.w & 0xFFFF0000u);  // x3,x7
                *reinterpret_cast<uint4*>(xl + sx * step_bytes + blk_off + m * 16) = o;
                // the step's sum of this row: 8 values here, then the 16 pieces in a fixed tree
                const uint32_t w4[4] = {v.x, v.y, v.z, v.w};
                float t = 0.f;
#pragma unroll
                for (int q4 = 0; q4 < 4; ++q4)
                    t += __builtin_bit_cast(float, w4[q4] << 16) + __builtin_bit_cast(float, w4[q4] & 0xFFFF0000u);
                t += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, t), 0x128, 0xF, 0xF, true));  // row_ror:8
                t += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, t), 0x124, 0xF, 0xF, true));  // row_ror:4
                t += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, t), 0x122, 0xF, 0xF, true));  // row_ror:2
                t += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, t), 0x121, 0xF, 0xF, true));  // row_ror:1
                if (t16 == 0) xs_tab[sx * 16 + m] = t;
            }
        }
        if (Mp != M)
            for (int e = threadIdx.x; e < (p1 - p0) * 16; e += kSmThreads)
                *reinterpret_cast<uint4*>(xl + (e >> 4) * step_bytes + (e & 15) * (Mp * 16) + M * 16) = make_uint4(0, 0, 0, 0);
        __syncthreads();

        // ---- this wave's steps inside the pass
        if (n > 0) {
            auto consume = [&](int p, int step) {
                const unsigned char* xb = xl + (step - p0) * step_bytes + kb * (Mp * 16) + xrow;
                const uint32_t w[4] = {q[p].x, q[p].y, q[p].z, q[p].w};
                f32x4_t d = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const uint4 a = *reinterpret_cast<const uint4*>(xb + j * 4 * (Mp * 16));
                    const uint4 bq = make_uint4((w[j] & 0x000F000Fu) | magic, ((w[j] >> 4) & 0x000F000Fu) | magic,
                                                ((w[j] >> 8) & 0x000F000Fu) | magic, ((w[j] >> 12) & 0x000F000Fu) | magic);
                    d = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, a),
                                                                __builtin_bit_cast(bf16x8_t, bq), d, 0, 0, 0);
                }
                const int grp = group_of(step);
                const float s = (float)sh[p];
                const float zc = (float)(128u + ((zw[p] >> (4 * (grp & 7))) & 0xFu));
                const float4 xs = *reinterpret_cast<const float4*>(xs_tab + (step - p0) * 16 + 4 * kb);
                acc[0] = fmaf(s, fmaf(-zc, xs.x, d[0]), acc[0]);
                acc[1] = fmaf(s, fmaf(-zc, xs.y, d[1]), acc[1]);
                acc[2] = fmaf(s, fmaf(-zc, xs.z, d[2]), acc[2]);
                acc[3] = fmaf(s, fmaf(-zc, xs.w, d[3]), acc[3]);
            };
            const int last = k1 - 1;
            int t = 0;
            // Refills go out four at a time: the four loads of a row then cover 256 contiguous
            // bytes and reach DRAM together, instead of 64 isolated bytes from each of 16 rows.
            for (; t + kRing < n; t += kRing) {
#pragma unroll
                for (int h = 0; h < kRing; h += 4) {
#pragma unroll
                    for (int p = h; p < h + 4; ++p) consume(p, k0 + t + p);
#pragma unroll
                    for (int p = h; p < h + 4; ++p) {
                        issue(p, min(k0 + t + p + kRing, last));
                        __builtin_amdgcn_sched_barrier(0);
                    }
                }
            }
#pragma unroll
            for (int p = 0; p < kRing; ++p)
                if (t + p < n) consume(p, k0 + t + p);
        }
    }

    // ---- the K parts of a tile meet in LDS; y[m][tile*16 + n] = sum over parts, parts in order
    __syncthreads();  // x is no longer read
    float* dst = partial + wave * 256 + lane;
#pragma unroll
    for (int r = 0; r < 4; ++r) dst[r * kWave] = acc[r];
    __syncthreads();
    for (int e = threadIdx.x; e < nt * 256; e += kSmThreads) {
        const int tl = e >> 8, rem = e & 255;
        const int m = rem >> 4, nn = rem & 15;   // consecutive threads -> consecutive n
        // register r of lane l holds row m = 4 (l / 16) + r, column n = l % 16
        const int o = (m & 3) * kWave + (m >> 2) * 16 + nn;
        float sum = 0.f;
        for (int kp = 0; kp < ksplit; ++kp) sum += partial[(tl * ksplit + kp) * 256 + o];
        const int rown = (tile0 + tl) * 16 + nn;
        if (m < M && rown < N) it.y[(size_t)m * N + rown] = f32_to_bf16_rne(sum);
    }
}


// ---- The kernel for group_size 128 (a step is a group) and an even number of groups per row.
//
// A block owns up to 32 consecutive tiles.  With more than 16 a wave owns one or two whole tiles
// and walks all of K for them; with fewer, the block's 16 waves are dealt to (tile, K part) pairs,
// K parts being whole turns of the ring (eight steps), and the parts' 16 x 16 results meet once,
// after the stream, in LDS (added in the order of the parts: deterministic).  After the staging
// of a pass's x there is no barrier: a wave's stream is one ring of loads over its (tile, step)
// pairs.  The scales and zero-points
// of eight steps are one 16-byte piece and one word of the lane's row and are fetched once per
// turn of the ring, with the first load of the turn: fetched per step, as two more load
// instructions that each touch 16 lines, they cost more than the codes themselves (a bare model
// of this loop runs at 3.7 TB/s with them and at 5.0 TB/s without).  A tile's steps are padded to
// a multiple of eight per pass, so slot p of the ring always holds a step whose group is p of
// the turn's eight; padded steps re-read the last step and are not consumed.
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4_t;
constexpr int kTilesPerWave = 2;

// kB8: the weights are signed bytes (symmetric, no zero-points) instead of unsigned nibbles.  A
// wave-wide load is then 16 rows x 64 k, two steps make a group, and a byte b = q + 128 (one XOR per
// word) is taken as two nibbles, q = 16 hi + lo - 128: the word goes through the same nibble
// expansion, its low nibbles into one MFMA chain and its high nibbles into another against the
// same x, and sum_k x q = 16 d_hi + d_lo - (16 * 128 + 128 + 128) sum_k x.  x stays bf16: nothing
// is rounded before the fp32 accumulation.
// kRB: blocks of 16 rows of x (M <= 16 kRB).  With two, every expanded operand feeds two MFMAs (rows
// 0-15 and 16-31 of x) and a wave owns one tile (the launcher gives a block at most 16).
template <bool kB8, int kRB>
__global__ __launch_bounds__(kSmThreads) void smallm_stream_kernel(const SmArgs args) {
    constexpr int kWS = kB8 ? 2 : 1;   // wave-wide loads ("steps" of the ring) per 128 k of x
    constexpr int kTPW = kRB == 1 ? kTilesPerWave : 1;   // tiles a wave can own
    extern __shared__ __attribute__((aligned(16))) unsigned char sm_lds[];
    unsigned char* xl = sm_lds;
    float* xs_tab = reinterpret_cast<float*>(sm_lds + kXBytes);   // [steps of a pass][row blocks][16] sums of x
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
    const int lane = threadIdx.x % kWave;
    const int li = lane & 15, kb = lane >> 4;
    const int M = args.M;

    int idx = 0;
    if (blockIdx.x < (unsigned)kSmMaxBlocks) idx = (args.item_of_block[blockIdx.x / 8] >> (4 * (blockIdx.x % 8))) & 15;
    idx = __builtin_amdgcn_readfirstlane(idx);
    const SmItem it = args.it[idx];
    const SmPlan pl = args.plan[idx];
    const int K = it.K, N = it.N;
    const int G = K / kStepK, zwords = (G + 7) / 8, S = G;
    const int rowbytes = kB8 ? K : K / 2;
    // the block's tiles, then this wave's: whole tiles (one or two) when the block has more than
    // 16, else one (tile, K part) pair with as many K parts as the waves and the turns of K allow
    const int b = (int)blockIdx.x - it.block_begin;
    const int tile0 = b * it.tiles_base + min(b, it.tiles_rem);
    const int nt = it.tiles_base + (b < it.tiles_rem ? 1 : 0);   // at most 32 (the launcher sees to it)
    const int Mp = pl.rows, pass_steps = pl.pass_steps, npass = pl.npass;
    // K parts per tile (block-uniform): every pass over K is divided among them in whole turns, so
    // that all waves of the block work in every pass
    const int ks = b < it.tiles_rem ? pl.ks[1] : pl.ks[0];
    const int inv_ks = (int)(b < it.tiles_rem ? pl.inv_ks[1] : pl.inv_ks[0]);
    const int gsh = b < it.tiles_rem ? pl.gshift[1] : pl.gshift[0], gran = 8 >> gsh;
    int t0, ntw, kpart = 0;
    if (nt > kSmWaves) {
        t0 = tile0 + (nt * wave) / kSmWaves;
        ntw = tile0 + (nt * (wave + 1)) / kSmWaves - t0;           // 1 or 2
    } else {
        const int slot = (wave * inv_ks) >> 16;
        kpart = wave - slot * ks;
        t0 = tile0 + min(slot, max(nt - 1, 0));
        ntw = slot < nt ? 1 : 0;
    }

    const int step_bytes = 16 * Mp * 16;                       // 16 (j, kb) blocks per step
    int xrow[kRB];                                             // this lane's rows inside a block (past M: the row of zeros)
#pragma unroll
    for (int rb = 0; rb < kRB; ++rb) xrow[rb] = min(16 * rb + li, M) * 16;

    uint32_t magic = 0x43004300u;    // bf16 pair (128, 128); in a vector register so that the
    asm volatile("" : "+v"(magic));  // AND-OR needs only one scalar operand
    uint4 ones = make_uint4(0x3F803F80u, 0x3F803F80u, 0x3F803F80u, 0x3F803F80u);   // eight bf16 ones,
    asm volatile("" : "+v"(ones.x), "+v"(ones.y), "+v"(ones.z), "+v"(ones.w));         // kept in vector registers

    const __amdgpu_buffer_rsrc_t rq = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint32_t*>(it.qw), 0, N * rowbytes, 0x00020000);
    const __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t*>(it.sc), 0, N * G * 2, 0x00020000);
    const __amdgpu_buffer_rsrc_t rz = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint32_t*>(it.zr), 0, kB8 ? 0 : N * zwords * 4, 0x00020000);
    // per tile of the wave: lane offsets of its row in the three tensors (rows past N: the last row)
    uint32_t qlane[kTilesPerWave], slane[kTilesPerWave], zlane[kTilesPerWave];
#pragma unroll
    for (int tw = 0; tw < kTilesPerWave; ++tw) {
        const int row = min((t0 + min(tw, max(ntw - 1, 0))) * 16 + li, N - 1);
        qlane[tw] = (uint32_t)row * (uint32_t)rowbytes + 16u * kb;
        slane[tw] = (uint32_t)row * (uint32_t)(G * 2);
        zlane[tw] = (uint32_t)row * (uint32_t)(zwords * 4);
    }

    f32x4_t acc[kTPW][kRB];
#pragma unroll
    for (int tw = 0; tw < kTPW; ++tw)
#pragma unroll
        for (int rb = 0; rb < kRB; ++rb) acc[tw][rb] = f32x4_t{0.f, 0.f, 0.f, 0.f};
    // acc[tile of the wave][row block] += s * r
    auto add_scaled = [&](int ctw, int rb, float s, const f32x4_t& r) {
        if (kTPW == 1 || ctw == 0) {   // wave-uniform
#pragma unroll
            for (int i = 0; i < 4; ++i) acc[0][rb][i] = fmaf(s, r[i], acc[0][rb][i]);
        } else {
#pragma unroll
            for (int i = 0; i < 4; ++i) acc[kTPW - 1][rb][i] = fmaf(s, r[i], acc[kTPW - 1][rb][i]);
        }
    };

    u32x4_t q[kRing];
    u32x4_t msc = {0u, 0u, 0u, 0u}, nsc = msc;   // scales of the eight steps of the turn being consumed / being fetched
    uint32_t mzw = 0, nzw = 0;                   // ... their zero-points

    // Staging: 16 neighbouring threads take the 16 pieces (16 bytes each) of one (row, step) pair,
    // pair p = row * (steps of the pass) + step: neighbouring groups of threads fetch neighbouring
    // 256-byte stretches of one row of x.  (With the rows of one step side by side, every block of
    // the grid asks for addresses 2 K bytes apart at the same moment, which one L2 channel serves:
    // the fetch of x then took 5 us.)  p / steps as a multiplication, exact for p < 2^16.
    const int tg = threadIdx.x >> 4, t16 = threadIdx.x & 15;
    // piece t16 of a (row, 128 k) pair is k = 8 t16 .. 8 t16 + 7: for nibbles block (j, kb) of piece 4 kb + j,
    // for bytes block (half, j, kb) of piece 8 half + 2 kb + j (a lane's 16 bytes are 16 k: two MFMAs' worth)
    const int blk_off = (kB8 ? (t16 >> 3) * 8 + (t16 & 1) * 4 + ((t16 & 7) >> 1) : (t16 & 3) * 4 + (t16 >> 2)) * (Mp * 16);
    uint4 xr[8];
    const char* xbase = reinterpret_cast<const char*>(it.x);   // M * K < 2^31 elements: 32-bit offsets

    for (int pass = 0; pass < npass; ++pass) {
        const int p0 = pass * pass_steps, p1 = min(S, p0 + pass_steps);   // p0 is a multiple of eight
        const int pw0 = p0 * kWS, pw1 = p1 * kWS;                          // the pass in steps of the ring
        // the pass in chunks of `gran` steps (a turn of the ring, or, where a block has too few tiles to keep its
        // waves busy with whole turns, half or a quarter of one: then a K part is a single chunk, so that its
        // steps never straddle a word of zero-points or the 16 bytes of scales fetched for them)
        const int pchunks = (pw1 - pw0 + gran - 1) >> (3 - gsh);
        const int k0 = pw0 + gran * ((pchunks * kpart * inv_ks) >> 16);   // this wave's steps in the pass; k0 is a multiple of gran
        const int k1 = min(pw1, pw0 + gran * ((pchunks * (kpart + 1) * inv_ks) >> 16));
        const int z8 = 4 * (k0 & 7);                                       // where the chunk's zero-points start in their word
        const int psteps = max(0, k1 - k0), upt = (psteps + 7) & ~7;      // steps and ring slots per tile in this pass
        const int units = ntw * upt;                                       // a multiple of eight
        // Pair p = row * ps + step of the pass; a thread's pairs are tg + 64 u.  Row and step of the
        // first come from one multiplication by a reciprocal the host worked out, those of the next
        // by adding 64 / ps and 64 % ps with a carry: no division and no 32-bit multiplication here.
        const int last = pass == npass - 1 ? 1 : 0;
        const int ps = p1 - p0;
        const int q64 = pl.q64[last], r64 = pl.r64[last];
        const int m0 = (int)__umulhi((uint32_t)tg, pl.inv_steps[last]);
        const int sx0 = tg - __mul24(m0, ps);
        if (pass) __syncthreads();  // the previous pass's activations are no longer read
        // ---- the pass's x is requested first, then the first weights of the pass: loads return
        // in order, x is needed first, and the staging then hides the weights' latency
        // (every load is issued, a pair past the last one re-reads the last: behind a condition each
        // load waited for the one before it, and the fetch of x took eight round trips instead of one)
        {
            int m = m0, sx = sx0;
            asm volatile("" : "+v"(m), "+v"(sx));   // worked out again for the staging rather than kept
            const uint32_t xlast = (uint32_t)((M - 1) * K + (p1 - 1) * kStepK + t16 * 8) * 2u;
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const uint32_t off = m < M ? (uint32_t)(__mul24(m, K) + (p0 + sx) * kStepK + t16 * 8) * 2u : xlast;
                xr[u] = *reinterpret_cast<const uint4*>(xbase + off);
                m += q64;
                sx += r64;
                if (sx >= ps) sx -= ps, ++m;
            }
        }
        __builtin_amdgcn_sched_barrier(0);
        // With 96 KB of x and more per pass, every wave's x is asked for before any wave's weights
        // (block-uniform): the CU serves its loads in the order of issue, and the last wave's x,
        // queued behind the other waves' weights, held the block's first step back (measured:
        // 0.5-0.9 us of the layer at M = 12 and 16, nothing or a loss below).
        if (ps * M >= 384) __builtin_amdgcn_s_barrier();
        __builtin_amdgcn_sched_barrier(0);

        // The ring walks (tile of the wave, step of the pass); both counters are wave-uniform and
        // advance by one per load / per consumed slot.  Past the last pair the last one is repeated.
        int itw = 0, is = 0;   // tile and step (relative to p0, may run into the padding) of the next load
        // a wave without steps in this pass asks for offsets past the end of every tensor (they fit 2 GB):
        // the range check answers those with zeros and fetches nothing
        uint32_t ql[kTilesPerWave], sl[kTilesPerWave], zl[kTilesPerWave];
#pragma unroll
        for (int tw = 0; tw < kTilesPerWave; ++tw) {
            ql[tw] = units > 0 ? qlane[tw] : 0x80000000u;
            sl[tw] = units > 0 ? slane[tw] : 0x80000000u;
            zl[tw] = units > 0 ? zlane[tw] : 0x80000000u;
        }
        auto issue = [&](int p) {
            const int tw = min(itw, max(ntw - 1, 0));
            const uint32_t step = (uint32_t)max(k0 + min(is, psteps - 1), 0);
            // (a padded slot and a slot past the end of the wave's stream ask past the end of the tensor: no fetch)
            const bool real = itw < ntw && is < psteps;
            q[p] = __builtin_amdgcn_raw_buffer_load_b128(rq, real ? (tw ? ql[1] : ql[0]) : 0x80000000u, step * (kStepK / 2), 0);
            if (p == 0) {   // is is a multiple of eight here; the eight groups from p0 + is on
                // (the whole offset in the lane part, which is the part the hardware checks against the tensor's
                // size: the last turn of the last row may reach past the end of the scales, and then reads zeros)
                if constexpr (kB8) {   // four groups a turn
                    typedef __attribute__((ext_vector_type(2))) uint32_t u32x2_t;
                    const u32x2_t t = __builtin_amdgcn_raw_buffer_load_b64(rs, (tw ? sl[1] : sl[0]) + (uint32_t)(k0 + is), 0, 0);
                    nsc[0] = t[0];
                    nsc[1] = t[1];
                } else {
                    nsc = __builtin_amdgcn_raw_buffer_load_b128(rs, (tw ? sl[1] : sl[0]) + (uint32_t)(k0 + is) * 2u, 0, 0);
                    nzw = __builtin_amdgcn_raw_buffer_load_b32(rz, tw ? zl[1] : zl[0], (uint32_t)((k0 + is) >> 3) * 4u, 0);
                }
            }
            __builtin_amdgcn_sched_barrier(0);  // program order = consumption order
            if (itw < ntw) {
                ++is;
                if (is == upt) is = 0, ++itw;
            }
        };
        // (issued by every wave, whether it has steps in this pass or not: behind a condition the
        // compiler can no longer count the loads in flight and drains the ring before every use)
#pragma unroll
        for (int p = 0; p < kRing; ++p) issue(p);
        // ---- stage x[:, 128 p0 .. 128 p1) and the zero rows (the sums of x over a step that the
        // offset form needs come from the matrix cores, see below: summed here they tripled the
        // vector work of the staging, which nothing hides)
        int m = m0, sx = sx0;
        asm volatile("" : "+v"(m), "+v"(sx));
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            if (m < M) {
                const uint4 v = xr[u];
                uint4 o;
                if constexpr (kB8) {   // the order in which the expansion lays out the bytes of two words
                    o.x = (v.x & 0xFFFFu) | (v.y << 16);      // x0,x2
                    o.y = (v.x >> 16) | (v.y & 0xFFFF0000u);  // x1,x3
                    o.z = (v.z & 0xFFFFu) | (v.w << 16);      // x4,x6
                    o.w = (v.z >> 16) | (v.w & 0xFFFF0000u);  // x5,x7
                } else {               // ... the nibbles of one word
                    o.x = (v.x & 0xFFFFu) | (v.z << 16);      // x0,x4
                    o.y = (v.x >> 16) | (v.z & 0xFFFF0000u);  // x1,x5
                    o.z = (v.y & 0xFFFFu) | (v.w << 16);      // x2,x6
                    o.w = (v.y >> 16) | (v.w & 0xFFFF0000u);  // x3,x7
                }
                *reinterpret_cast<uint4*>(xl + __mul24(sx, step_bytes) + blk_off + m * 16) = o;
            }
            m += q64;
            sx += r64;
            if (sx >= ps) sx -= ps, ++m;
        }
        if (Mp != M)
            for (int e = threadIdx.x; e < (p1 - p0) * 16; e += kSmThreads)
                *reinterpret_cast<uint4*>(xl + (e >> 4) * step_bytes + (e & 15) * (Mp * 16) + M * 16) = make_uint4(0, 0, 0, 0);
        __syncthreads();
        // ---- sum_k x over every 128 k of the pass, per row: the offset form needs it with every step, every
        // wave would otherwise compute it again (a second MFMA chain against ones cost 3 us of the layer at
        // M = 16).  The waves share the steps out; with ones as B every lane's register i is the sum of row
        // 4 kb + i, so the four lanes with li = 0 hold a step's 16 sums.
        for (int sx = wave; sx < ps; sx += kSmWaves) {
#pragma unroll
            for (int rb = 0; rb < kRB; ++rb) {
                f32x4_t t = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int j = 0; j < 4; ++j) {   // the step's 16 blocks are 4 j + kb in either layout
                    const uint4 a = *reinterpret_cast<const uint4*>(xl + sx * step_bytes + (4 * j + kb) * (Mp * 16) + xrow[rb]);
                    t = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, a),
                                                                __builtin_bit_cast(bf16x8_t, ones), t, 0, 0, 0);
                }
                if (li == 0) *reinterpret_cast<f32x4_t*>(xs_tab + ((sx * kRB + rb) * 16 + 4 * kb)) = t;
            }
        }
        __syncthreads();

        // ---- this wave's (tile, step) pairs of the pass
        if (units > 0) {
            int ctw = 0, cs = 0;   // tile and step of the slot being consumed
            // bytes: slots p and p + 1 are the two halves of one group (p even; a wave's steps in a pass are an
            // even number, so both are padding or neither is)
            auto consume_bytes = [&](int p) {
                if (cs < psteps) {   // wave-uniform
                    const unsigned char* xb = xl + ((k0 - pw0 + cs) >> 1) * step_bytes + kb * (Mp * 16);
                    f32x4_t dl[kRB], dh[kRB], xs[kRB];
#pragma unroll
                    for (int rb = 0; rb < kRB; ++rb) {
                        dl[rb] = dh[rb] = f32x4_t{0.f, 0.f, 0.f, 0.f};
                        xs[rb] = *reinterpret_cast<const f32x4_t*>(xs_tab + ((((k0 - pw0 + cs) >> 1) * kRB + rb) * 16 + 4 * kb));
                    }
#pragma unroll
                    for (int hf = 0; hf < 2; ++hf) {
                        const u32x4_t wq = q[p + hf] ^ 0x80808080u;   // b = q + 128
#pragma unroll
                        for (int j = 0; j < 2; ++j) {
                            const uint32_t w0 = wq[2 * j], w1 = wq[2 * j + 1];
                            const uint4 lo = make_uint4((w0 & 0x000F000Fu) | magic, ((w0 >> 8) & 0x000F000Fu) | magic,
                                                        (w1 & 0x000F000Fu) | magic, ((w1 >> 8) & 0x000F000Fu) | magic);
                            const uint4 hi = make_uint4(((w0 >> 4) & 0x000F000Fu) | magic, ((w0 >> 12) & 0x000F000Fu) | magic,
                                                        ((w1 >> 4) & 0x000F000Fu) | magic, ((w1 >> 12) & 0x000F000Fu) | magic);
#pragma unroll
                            for (int rb = 0; rb < kRB; ++rb) {
                                const uint4 a = *reinterpret_cast<const uint4*>(xb + (hf * 8 + j * 4) * (Mp * 16) + xrow[rb]);
                                dl[rb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, a),
                                                                                 __builtin_bit_cast(bf16x8_t, lo), dl[rb], 0, 0, 0);
                                dh[rb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, a),
                                                                                 __builtin_bit_cast(bf16x8_t, hi), dh[rb], 0, 0, 0);
                            }
                        }
                    }
                    const int g4 = p >> 1;   // the group among the turn's four
                    const uint16_t sbits = (uint16_t)(msc[g4 >> 1] >> (16 * (g4 & 1)));
                    const float s = (float)__builtin_bit_cast(_Float16, sbits);
                    // sum_k x q = 16 dh + dl - (16 * 128 + 128 + 128) sum_k x
#pragma unroll
                    for (int rb = 0; rb < kRB; ++rb) {
                        f32x4_t r;
#pragma unroll
                        for (int i = 0; i < 4; ++i) r[i] = fmaf(-2304.f, xs[rb][i], fmaf(16.f, dh[rb][i], dl[rb][i]));
                        add_scaled(ctw, rb, s, r);
                    }
                }
                cs += 2;
                if (cs == upt) cs = 0, ++ctw;
            };
            auto consume_nibbles = [&](int p) {
                if (cs < psteps) {   // wave-uniform: not a padded slot
                    const unsigned char* xb = xl + (k0 - p0 + cs) * step_bytes + kb * (Mp * 16);
                    const u32x4_t wq = q[p];
                    // d = sum_k x (q + 128); xs = sum_k x of the rows of d's registers, from the pass's table
                    f32x4_t d[kRB], xs[kRB];
#pragma unroll
                    for (int rb = 0; rb < kRB; ++rb) {
                        d[rb] = f32x4_t{0.f, 0.f, 0.f, 0.f};
                        xs[rb] = *reinterpret_cast<const f32x4_t*>(xs_tab + (((k0 - p0 + cs) * kRB + rb) * 16 + 4 * kb));
                    }
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        const uint4 bq = make_uint4((wq[j] & 0x000F000Fu) | magic, ((wq[j] >> 4) & 0x000F000Fu) | magic,
                                                    ((wq[j] >> 8) & 0x000F000Fu) | magic, ((wq[j] >> 12) & 0x000F000Fu) | magic);
#pragma unroll
                        for (int rb = 0; rb < kRB; ++rb) {
                            const uint4 a = *reinterpret_cast<const uint4*>(xb + j * 4 * (Mp * 16) + xrow[rb]);
                            d[rb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, a),
                                                                            __builtin_bit_cast(bf16x8_t, bq), d[rb], 0, 0, 0);
                        }
                    }
                    // slot p holds the step whose group is p of the turn's eight
                    const uint16_t sbits = (uint16_t)(msc[p >> 1] >> (16 * (p & 1)));
                    const float s = (float)__builtin_bit_cast(_Float16, sbits);
                    const float zc = (float)(128u + ((mzw >> (4 * p + z8)) & 0xFu));
#pragma unroll
                    for (int rb = 0; rb < kRB; ++rb) {
                        f32x4_t r;
#pragma unroll
                        for (int i = 0; i < 4; ++i) r[i] = fmaf(-zc, xs[rb][i], d[rb][i]);
                        add_scaled(ctw, rb, s, r);
                    }
                }
                ++cs;
                if (cs == upt) cs = 0, ++ctw;
            };
            auto consume = [&](int p) {   // slot p; the bytes' two-slot groups are consumed at their second slot
                if constexpr (kB8) {
                    if (p & 1) consume_bytes(p - 1);
                } else {
                    consume_nibbles(p);
                }
            };
            msc = nsc;   // the first turn's scales and zero-points
            mzw = nzw;
            // Refills go out four at a time: the four loads of a row then cover 256 contiguous
            // bytes and reach DRAM together, instead of 64 isolated bytes from each of 16 rows.
            for (int u = 0; u + kRing < units; u += kRing) {
#pragma unroll
                for (int h = 0; h < kRing; h += 4) {
#pragma unroll
                    for (int p = h; p < h + 4; ++p) consume(p);
#pragma unroll
                    for (int p = h; p < h + 4; ++p) issue(p);
                }
                msc = nsc;
                mzw = nzw;
            }
#pragma unroll
            for (int p = 0; p < kRing; ++p) consume(p);   // the last turn (units is a multiple of eight)
        }
    }

    // ---- y[m][tile * 16 + n]: register i of lane l holds row m = 4 (l / 16) + i, column n = l % 16
    if (ks > 1) {   // block-uniform: the K parts of a tile meet in LDS, parts in order
        float* partial = reinterpret_cast<float*>(sm_lds);
        __syncthreads();  // x is no longer read
#pragma unroll
        for (int rb = 0; rb < kRB; ++rb)
#pragma unroll
            for (int i = 0; i < 4; ++i) partial[(wave * kRB + rb) * 256 + i * kWave + lane] = acc[0][rb][i];
        __syncthreads();
        for (int e = threadIdx.x; e < nt * kRB * 256; e += kSmThreads) {
            const int tl = e / (kRB * 256), rb = (e >> 8) % kRB, rem = e & 255;
            const int mm = rem >> 4, nn = rem & 15;   // consecutive threads -> consecutive n
            const int o = (mm & 3) * kWave + (mm >> 2) * 16 + nn;
            float sum = 0.f;
            for (int kp = 0; kp < ks; ++kp) sum += partial[((tl * ks + kp) * kRB + rb) * 256 + o];
            const int rown = (tile0 + tl) * 16 + nn, m = 16 * rb + mm;
            if (m < M && rown < N) it.y[(size_t)m * N + rown] = f32_to_bf16_rne(sum);
        }
        return;
    }
#pragma unroll
    for (int tw = 0; tw < kTPW; ++tw) {
        const int n = (t0 + tw) * 16 + li;
        if (tw < ntw && n < N) {
#pragma unroll
            for (int rb = 0; rb < kRB; ++rb)
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const int m = 16 * rb + 4 * kb + i;
                    if (m < M) it.y[(size_t)m * N + n] = f32_to_bf16_rne(acc[tw][rb][i]);
                }
        }
    }
}

size_t sm_item_bytes(const qail_wdesc& d) {
    const size_t G = (size_t)d.K / d.group_size;
    return (size_t)d.N * (d.K / 2 + G * 2 + ((G + 7) / 8) * 4);
}

// Shapes of the kernel with one group per step: group_size 128 and an even number of groups per row
// (the eight scales of a turn are fetched as words), tensors below 2 GB (32-bit offsets).
bool sm_one_group_per_step(const qail_wdesc& d) {
    return d.group_size == kStepK && (d.K / kStepK) % 2 == 0 && (unsigned long long)d.N * d.K / 2 <= 0x7FFFFFFFull;
}

// Every item of the list is of that shape: whole tiles per wave, blocks divided by bytes.
// b8: the items' weights are signed bytes (zeros unused) instead of nibbles.
hipError_t sm_launch_tiles_per_wave(const qail_w4a16_item* items, int count, int M, hipStream_t st, bool b8) {
    // more than 64 KB of LDS needs an opt-in; the call is idempotent, so two host threads that
    // both find the flag clear may both make it
    const bool two = M > 16;   // two blocks of 16 rows of x
    const void* const kernels[4] = {reinterpret_cast<const void*>(&smallm_stream_kernel<false, 1>),
                                    reinterpret_cast<const void*>(&smallm_stream_kernel<true, 1>),
                                    reinterpret_cast<const void*>(&smallm_stream_kernel<false, 2>),
                                    reinterpret_cast<const void*>(&smallm_stream_kernel<true, 2>)};
    const int which = (two ? 2 : 0) + (b8 ? 1 : 0);
    static std::atomic<bool> attr_done[4];
    if (!attr_done[which].load(std::memory_order_acquire)) {
        const hipError_t e = hipFuncSetAttribute(kernels[which], hipFuncAttributeMaxDynamicSharedMemorySize, (int)kSmLdsBytes);
        if (e != hipSuccess) return e;
        attr_done[which].store(true, std::memory_order_release);
    }
    SmArgs a;
    int grid = device_cu_count();
    if (grid < count) grid = count;
    // A block's cost: its share of the item's bytes, plus x, which every block fetches once, plus, per
    // further pass over K, the bytes it could have streamed while the pass's activations are fetched
    // and staged (a figure measured on this GPU).  A block owns at most 32 tiles, and at most 16 (one
    // per wave, the step count of the longest wave halved) where the grid has the blocks for that.
    constexpr double kPassCost = 100.0 * 1024;
    int nb[kSmMaxItems], lo[kSmMaxItems], hi[kSmMaxItems];
    double bytes[kSmMaxItems], fixed[kSmMaxItems];
    double t_lo = 0, t_hi = 0;
    int one_tile_per_wave = 0;
    for (int i = 0; i < count; ++i) one_tile_per_wave += ((items[i].d.N + 15) / 16 + kSmWaves - 1) / kSmWaves;
    // (with two row blocks a wave owns one tile: more blocks than CUs then, if it takes that)
    const int most_tiles = (two || one_tile_per_wave <= grid) ? kSmWaves : kSmWaves * kTilesPerWave;
    for (int i = 0; i < count; ++i) {
        const int ntiles = (items[i].d.N + 15) / 16;
        lo[i] = (ntiles + most_tiles - 1) / most_tiles;
        hi[i] = ntiles;
        int rows, ps;
        const int S = items[i].d.K / kStepK;
        sm_plan(M, S, &rows, &ps);
        bytes[i] = (double)sm_item_bytes(items[i].d) * (b8 ? 2 : 1);   // (twice the codes; no zero-points, which are a percent)
        fixed[i] = 2.0 * M * items[i].d.K + kPassCost * ((S + ps - 1) / ps - 1);
        if (fixed[i] + bytes[i] > t_hi) t_hi = fixed[i] + bytes[i];
    }
    auto blocks_for = [&](double T, int* out) {
        int used = 0;
        for (int i = 0; i < count; ++i) {
            int n = hi[i];
            if (T > fixed[i]) {
                const double need = bytes[i] / (T - fixed[i]);
                n = need >= (double)hi[i] ? hi[i] : (int)need + 1;
            }
            if (n < lo[i]) n = lo[i];
            if (n > hi[i]) n = hi[i];
            out[i] = n;
            used += n;
        }
        return used;
    };
    for (int iter = 0; iter < 40; ++iter) {
        const double T = 0.5 * (t_lo + t_hi);
        if (blocks_for(T, nb) <= grid) t_hi = T;
        else t_lo = T;
    }
    int used = blocks_for(t_hi, nb);
    while (used < grid) {   // left-over blocks go where a block's cost is highest
        int best = -1;
        double best_cost = 0;
        for (int i = 0; i < count; ++i) {
            const double c = fixed[i] + bytes[i] / nb[i];
            if (nb[i] < hi[i] && (best < 0 || c > best_cost)) best = i, best_cost = c;
        }
        if (best < 0) break;
        ++nb[best];
        ++used;
    }
    if (count > 1 && used > kSmMaxBlocks) {
        // the block-to-item table is too short: one launch per item (a lone item needs no table)
        for (int i = 0; i < count; ++i) {
            const hipError_t e = sm_launch_tiles_per_wave(items + i, 1, M, st, b8);
            if (e != hipSuccess) return e;
        }
        return hipSuccess;
    }
    memset(a.item_of_block, 0, sizeof(a.item_of_block));
    int bb = 0;
    for (int i = 0; i < count; ++i) {
        const qail_w4a16_item& s = items[i];
        SmItem& t = a.it[i];
        t.qw = s.qweight; t.sc = s.scales; t.zr = s.zeros; t.x = s.x; t.y = s.y;
        t.N = s.d.N; t.K = s.d.K; t.g = s.d.group_size;
        t.block_begin = bb;
        const int ntiles = (s.d.N + 15) / 16;
        t.tiles_base = ntiles / nb[i];
        t.tiles_rem = ntiles % nb[i];
        for (int b = bb; b < bb + nb[i] && b < kSmMaxBlocks; ++b) a.item_of_block[b / 8] |= (uint32_t)i << (4 * (b % 8));
        bb += nb[i];
        // the divisions the kernel would otherwise do
        SmPlan& pl = a.plan[i];
        int rows, ps;
        const int S = s.d.K / kStepK;
        sm_plan(M, S, &rows, &ps);
        if (ps > S) ps = S;
        const int npass = (S + ps - 1) / ps, last = S - (npass - 1) * ps;
        if (ps < 2 || last < 2) return hipErrorInvalidValue;   // cannot happen: S is even, a pass is S or a multiple of eight
        pl.rows = (uint16_t)rows; pl.pass_steps = (uint16_t)ps; pl.npass = (uint16_t)npass; pl.last_steps = (uint16_t)last;
        const int steps[2] = {ps, last};
        for (int v = 0; v < 2; ++v) {
            pl.inv_steps[v] = (uint32_t)((((uint64_t)1 << 32) + steps[v] - 1) / steps[v]);
            pl.q64[v] = (uint8_t)(64 / steps[v]);
            pl.r64[v] = (uint16_t)(64 % steps[v]);
            const int nt = t.tiles_base + v;
            // K parts of a tile: as many as the waves allow, in whole turns of the ring; where a full pass has
            // fewer turns than that, in single chunks of 2 or 4 steps if the pass then has no more chunks than
            // the waves allow (the finest such division)
            const int psw = ps * (b8 ? 2 : 1), want = nt > kSmWaves ? 1 : kSmWaves / std::max(nt, 1);
            int ks = std::max(1, std::min(want, (psw + 7) / 8)), gshift = 0;
            if (ks < want)
                for (int g = b8 ? 1 : 2; g >= 1; --g)   // (a chunk's scales start at a whole word: two groups, i.e. 4 steps of bytes)
                    if (((psw + (8 >> g) - 1) >> (3 - g)) <= want) { gshift = g; ks = (psw + (8 >> g) - 1) >> (3 - g); break; }
            pl.ks[v] = (uint8_t)ks;
            pl.gshift[v] = (uint8_t)gshift;
            pl.inv_ks[v] = (uint32_t)((65536 + ks - 1) / ks);
        }
    }
    for (int i = count; i < kSmMaxItems; ++i) a.it[i] = a.it[count - 1], a.plan[i] = a.plan[count - 1];
    a.M = M;
    switch (which) {
        case 0: hipLaunchKernelGGL((smallm_stream_kernel<false, 1>), dim3(bb), dim3(kSmThreads), kSmLdsBytes, st, a); break;
        case 1: hipLaunchKernelGGL((smallm_stream_kernel<true, 1>), dim3(bb), dim3(kSmThreads), kSmLdsBytes, st, a); break;
        case 2: hipLaunchKernelGGL((smallm_stream_kernel<false, 2>), dim3(bb), dim3(kSmThreads), kSmLdsBytes, st, a); break;
        default: hipLaunchKernelGGL((smallm_stream_kernel<true, 2>), dim3(bb), dim3(kSmThreads), kSmLdsBytes, st, a); break;
    }
    return hipGetLastError();
}

hipError_t sm_launch_chunk(const qail_w4a16_item* items, int count, int M, hipStream_t st) {
    bool one_group = true;
    for (int i = 0; i < count; ++i) one_group = one_group && sm_one_group_per_step(items[i].d);
    if (one_group) return sm_launch_tiles_per_wave(items, count, M, st, false);
    // more than 64 KB of LDS needs an opt-in; the call is idempotent, so two host threads that
    // both find the flag clear may both make it
    static std::atomic<bool> attr_done{false};
    if (!attr_done.load(std::memory_order_acquire)) {
        const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&w4a16_smallm_general_kernel),
                                                 hipFuncAttributeMaxDynamicSharedMemorySize, (int)kSmLdsBytes);
        if (e != hipSuccess) return e;
        attr_done.store(true, std::memory_order_release);
    }
    SmArgs a;
    int grid = device_cu_count();
    if (grid < count) grid = count;
    // Blocks per item: a block's time is taken as its bytes plus, per pass over K, the bytes it could
    // have streamed while a pass's activations are fetched and staged (a figure measured on this GPU);
    // the smallest common bound T on that cost that the grid can meet decides the division.
    constexpr double kPassCost = 100.0 * 1024;
    int nb[kSmMaxItems], lo[kSmMaxItems], hi[kSmMaxItems];
    double bytes[kSmMaxItems], fixed[kSmMaxItems];
    double t_lo = 0, t_hi = 0;
    for (int i = 0; i < count; ++i) {
        const int ntiles = (items[i].d.N + 15) / 16;
        lo[i] = (ntiles + kTilesPerBlock - 1) / kTilesPerBlock;  // a block owns at most 16 tiles
        hi[i] = ntiles;
        int rows, ps;
        const int S = items[i].d.K / kStepK;
        sm_plan(M, S, &rows, &ps);
        bytes[i] = (double)sm_item_bytes(items[i].d);
        fixed[i] = kPassCost * ((S + ps - 1) / ps);
        if (fixed[i] + bytes[i] > t_hi) t_hi = fixed[i] + bytes[i];
    }
    auto blocks_for = [&](double T, int* out) {
        int used = 0;
        for (int i = 0; i < count; ++i) {
            int n = hi[i];
            if (T > fixed[i]) {
                const double need = bytes[i] / (T - fixed[i]);
                n = need >= (double)hi[i] ? hi[i] : (int)need + 1;
            }
            if (n < lo[i]) n = lo[i];
            if (n > hi[i]) n = hi[i];
            out[i] = n;
            used += n;
        }
        return used;
    };
    for (int iter = 0; iter < 40; ++iter) {
        const double T = 0.5 * (t_lo + t_hi);
        if (blocks_for(T, nb) <= grid) t_hi = T;
        else t_lo = T;
    }
    int used = blocks_for(t_hi, nb);
    while (used < grid) {   // left-over blocks go where a block's cost is highest
        int best = -1;
        double best_cost = 0;
        for (int i = 0; i < count; ++i) {
            const double c = fixed[i] + bytes[i] / nb[i];
            if (nb[i] < hi[i] && (best < 0 || c > best_cost)) best = i, best_cost = c;
        }
        if (best < 0) break;
        ++nb[best];
        ++used;
    }
    if (count > 1 && used > kSmMaxBlocks) {
        // the block-to-item table is too short: one launch per item (a lone item needs no table)
        for (int i = 0; i < count; ++i) {
            const hipError_t e = sm_launch_chunk(items + i, 1, M, st);
            if (e != hipSuccess) return e;
        }
        return hipSuccess;
    }
    memset(a.item_of_block, 0, sizeof(a.item_of_block));
    int bb = 0;
    for (int i = 0; i < count; ++i) {
        const qail_w4a16_item& s = items[i];
        SmItem& t = a.it[i];
        const int ntiles = (s.d.N + 15) / 16;
        t.qw = s.qweight; t.sc = s.scales; t.zr = s.zeros; t.x = s.x; t.y = s.y;
        t.N = s.d.N; t.K = s.d.K; t.g = s.d.group_size;
        t.block_begin = bb;
        t.tiles_base = ntiles / nb[i];
        t.tiles_rem = ntiles % nb[i];
        for (int b = bb; b < bb + nb[i] && b < kSmMaxBlocks; ++b) a.item_of_block[b / 8] |= (uint32_t)i << (4 * (b % 8));
        bb += nb[i];
    }
    for (int i = count; i < kSmMaxItems; ++i) a.it[i] = a.it[count - 1];
    a.M = M;
    hipLaunchKernelGGL(w4a16_smallm_general_kernel, dim3(bb), dim3(kSmThreads), kSmLdsBytes, st, a);
    return hipGetLastError();
}

}  // namespace

bool smallm_supports(const qail_wdesc& d, int M) {
    const int spg = d.group_size / kStepK;
    if (M > 16) return M <= 32 && d.K % kStepK == 0 && sm_one_group_per_step(d);   // two row blocks: that kernel only
    return M >= 2 && d.K % kStepK == 0 && d.group_size % kStepK == 0 && (spg & (spg - 1)) == 0 &&
           (unsigned long long)d.N * d.K / 2 <= 0xFFFFFFFFull;   // 32-bit byte offsets in the kernel
}

// 8-bit weights (signed bytes, one fp16 scale per group, no zero-points) on the kernel with one group
// per 128 k: group size 128, an even number of groups per row, N * K below 2 GB.
bool smallm_w8_supports(const qail_wdesc& d, int M) {
    return M >= 2 && M <= 32 && d.group_size == kStepK && d.K % kStepK == 0 && (d.K / kStepK) % 2 == 0 &&
           (unsigned long long)d.N * d.K <= 0x7FFFFFFFull;
}

// items: the 8-bit linears in the W4A16 item record (zeros unused)
hipError_t launch_w8a16_smallm(const qail_w4a16_item* items, int count, int M, hipStream_t st) {
    for (int i0 = 0; i0 < count; i0 += kSmMaxItems) {
        const int c = (count - i0 < kSmMaxItems) ? count - i0 : kSmMaxItems;
        const hipError_t e = sm_launch_tiles_per_wave(items + i0, c, M, st, true);
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
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
