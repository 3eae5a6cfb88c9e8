// Weight-only 8-bit linear for M = 1 (Sec. 5.4: the backbone is also deployed with 8-bit weights):
//   y[n] = sum_k x[k] * q[n,k] * s[n,k/g],   q signed bytes.
//
// Bandwidth-bound like the 4-bit decode kernel (w4a16_gemv.hip), at twice the bytes, and built
// the same way: a lane fetches 16 bytes (16 codes) of a row per load, a wave 1 KB of one row; x
// is staged once per block in LDS as fp16 with a power of two per 16-k stretch; the products run
// on v_mfma_f32_4x4x4_16b_f16, whose D[j][j] (register j of lane 4b + j) is the lane's private
// 4-element dot product; every wave keeps a ring of loads in flight with exact waits; results
// stay in registers until the wave has finished its rows.
//
// Bytes become fp16 without conversion instructions: with u = q + 128 (q ^ 0x80 as a byte),
// 0x6400 | u is the fp16 number 1024 + u, and 0x6400 | (q ^ 0x80) = 0x6480 ^ q.  One v_perm_b32
// spreads two bytes of a word over the low bytes of two halfwords, one XOR with 0x64806480
// finishes both.  Then
//
//   sum_k x_k q_k  =  sum_k x_k (1024 + u_k)  -  1152 sum_k x_k ,
//
// with the second term per stretch computed once per block at staging.
#include <algorithm>

#include "qail_internal.h"

namespace qail {

namespace {

constexpr int kW8Waves = 8;    // two blocks share a CU
constexpr int kW8Threads = kW8Waves * kWave;
constexpr int kW8Ring = 8;            // wave-wide loads (1 KB each) in flight per wave
constexpr int kW8ChunkK = 1024;       // k of a row per wave-wide load (16 per lane)
constexpr int kW8MaxChunks = 12;      // K <= 12288
constexpr int kW8XRuns = (kW8MaxChunks * (kW8ChunkK / 8) + kW8Threads - 1) / kW8Threads;  // 8-k runs of x per thread

typedef __attribute__((ext_vector_type(4))) uint32_t u32x4_t;
typedef __attribute__((ext_vector_type(4))) _Float16 f16x4_t;

struct W8Args {
    const uint32_t* qw;
    const uint16_t* sc;
    const uint16_t* x;
    uint16_t* y;
    int N, K, g;
    int rows_base, rows_rem;  // block b owns rows_base rows, one more if b < rows_rem, in the order of the blocks
    int block_begin;          // first block of the grid that works on this linear
};

// Up to kW8Batch linears share a launch, each on its own run of blocks.
constexpr int kW8Batch = 8;
struct W8Batch {
    W8Args it[kW8Batch];
    int count;
};

template <int kCtrl>
__device__ __forceinline__ float dpp8_f(float v) {
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), kCtrl, 0xF, 0xF, true));
}

// Sum over the 64 lanes; the result is wave-uniform.
__device__ __forceinline__ float wave_sum8(float v) {
    v += dpp8_f<0xB1>(v);   // quad_perm [1,0,3,2]
    v += dpp8_f<0x4E>(v);   // quad_perm [2,3,0,1]
    v += dpp8_f<0x141>(v);  // row_half_mirror
    v += dpp8_f<0x140>(v);  // row_mirror: every lane of a 16-lane row holds the row sum
    const int vi = __builtin_bit_cast(int, v);
    return __builtin_bit_cast(float, __builtin_amdgcn_readlane(vi, 0)) +
           __builtin_bit_cast(float, __builtin_amdgcn_readlane(vi, 16)) +
           (__builtin_bit_cast(float, __builtin_amdgcn_readlane(vi, 32)) +
            __builtin_bit_cast(float, __builtin_amdgcn_readlane(vi, 48)));
}

// LDS map of a block, nc = ceil(K / 1024) chunks per row:
//   uint4  [nc*2*64]   staged activations: word e (8 k) of lane L in chunk c at (c*2 + e)*64 + L
//   float2 [nc*64]     constants of lane L's stretch of chunk c at c*64 + L, with P = 2^e:
//                      (P * 1152 * sum of the staged values, P)
// Lane L owns, in chunk c, the 16 k starting at 1024 c + 16 L; they are staged as fp16 times 2^-e
// (largest magnitude of the stretch in [2^14, 2^15)).  Everything past K is zero.
__global__ __launch_bounds__(kW8Threads) void w8a16_stream_kernel(const W8Batch args) {
    extern __shared__ uint4 w8_lds[];
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
    const int lane = threadIdx.x % kWave;
    int item = 0;
#pragma unroll
    for (int i = 1; i < kW8Batch; ++i)
        if (i < args.count && (int)blockIdx.x >= args.it[i].block_begin) item = i;
    const W8Args a = args.it[item];
    const int K = a.K, N = a.N, g = a.g;
    const int G = K / g;
    const int nc = (K + kW8ChunkK - 1) / kW8ChunkK;
    uint4* const xl = w8_lds;
    float2* const consts = reinterpret_cast<float2*>(w8_lds + nc * 2 * kWave);

    // x first: it is needed first and loads return in order.  Run r = 8 consecutive k; two
    // neighbouring threads hold the two runs of one stretch.
    // (Through a buffer descriptor of K elements: runs past K read zeros without a fetch, so every
    // load is issued and no condition stands before it.)
    const int row_runs = K / 8;
    const __amdgpu_buffer_rsrc_t rx = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t*>(a.x), 0, K * 2, 0x00020000);
    uint4 xr[kW8XRuns];
#pragma unroll
    for (int u = 0; u < kW8XRuns; ++u) {
        const u32x4_t v = __builtin_amdgcn_raw_buffer_load_b128(rx, (threadIdx.x + u * kW8Threads) * 16, 0, 0);
        xr[u] = make_uint4(v[0], v[1], v[2], v[3]);
    }
    __builtin_amdgcn_sched_barrier(0);  // the scheduler must not move the x loads behind the weights

    // this block's rows, dealt to its waves in turn
    const int bk = (int)blockIdx.x - a.block_begin;
    const int s0 = bk * a.rows_base + min(bk, a.rows_rem);
    const int nrows = a.rows_base + (bk < a.rows_rem ? 1 : 0);
    const int nrw = max(0, (nrows - wave + kW8Waves - 1) / kW8Waves);  // rows of this wave: at most 64
    const int total = nrw * nc;                                         // its stream of (row, chunk) loads

    // Loads: buffer descriptor + scalar offset (row, chunk; not range-checked by the hardware:
    // every address below is inside its tensor) + a lane offset that never changes.  Only the last
    // chunk of a row can run past K: a lane whose stretch does reads the first bytes and the first
    // group of that chunk instead (valid data; it meets zeros in x).  A chunk holds a whole number
    // of groups or a group a power-of-two number of chunks (host check), so a stretch's group is
    // (chunk part) + (lane part).
    const __amdgpu_buffer_rsrc_t rq = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint32_t*>(a.qw), 0, N * K, 0x00020000);
    const __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t*>(a.sc), 0, N * G * 2, 0x00020000);
    const int gpc = g < kW8ChunkK ? kW8ChunkK / g : 1;   // groups per chunk
    const int cpg = g < kW8ChunkK ? 1 : g / kW8ChunkK;   // chunks per group
    const int cpg_shift = __builtin_ctz(cpg), gpc_shift = __builtin_ctz(gpc);
    const int lgrp = g < kW8ChunkK ? (16 * lane) / g : 0;  // lane part of the group index
    const bool tail_out = (nc - 1) * kW8ChunkK + 16 * lane >= K;
    // (a wave without rows asks for offsets past the end of both tensors, which are below 2 GB: the
    // range check answers with zeros and fetches nothing.  Its loads are issued all the same: with
    // the ring's first loads behind a condition the compiler can no longer count the loads in
    // flight, and the staging of x below would wait for the weights as well)
    const int past = (int)0x80000000u;
    const int qlane = nrw == 0 ? past : lane * 16, qlane_last = (tail_out && nrw != 0) ? 0 : qlane;
    const int slane = nrw == 0 ? past : lgrp * 2, slane_last = (tail_out && nrw != 0) ? 0 : slane;

    uint4 q[kW8Ring];
    uint32_t sh[kW8Ring];  // fp16 bits as loaded (zero-extended): a conversion at the load would wait there
    auto issue = [&](int p, int ir, int ic) {
        const int row = s0 + wave + kW8Waves * ir;
        const bool last = ic == nc - 1;
        const int cg = (ic >> cpg_shift) << gpc_shift;
        const u32x4_t v = __builtin_amdgcn_raw_buffer_load_b128(rq, last ? qlane_last : qlane, row * K + ic * kW8ChunkK, 0);
        q[p] = make_uint4(v[0], v[1], v[2], v[3]);
        sh[p] = __builtin_amdgcn_raw_buffer_load_b16(rs, last ? slane_last : slane, row * (G * 2) + cg * 2, 0);
    };
    // next (row, chunk) of the stream; past its end the last load is repeated (and not consumed)
    auto advance = [&](int& rw, int& ch) {
        const bool last = ch == nc - 1;
        if (!(rw == nrw - 1 && last)) {
            ch = last ? 0 : ch + 1;
            rw += last ? 1 : 0;
        }
    };
    int ir = 0, ic = 0;
#pragma unroll
    for (int p = 0; p < kW8Ring; ++p) {
        issue(p, ir, ic);
        advance(ir, ic);
        __builtin_amdgcn_sched_barrier(0);  // program order = consumption order
    }

    // ---- stage x (whole block; one barrier)
    {
#pragma unroll
        for (int u = 0; u < kW8XRuns; ++u) {
            if (u * kW8Threads >= row_runs) break;  // block-uniform
            const int r = threadIdx.x + u * kW8Threads;
            const uint32_t w[4] = {xr[u].x, xr[u].y, xr[u].z, xr[u].w};
            float f[8];
            float amax = 0.f;
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                f[2 * t] = __builtin_bit_cast(float, w[t] << 16);
                f[2 * t + 1] = __builtin_bit_cast(float, w[t] & 0xFFFF0000u);
                amax = fmaxf(amax, fmaxf(fabsf(f[2 * t]), fabsf(f[2 * t + 1])));
            }
            amax = fmaxf(amax, dpp8_f<0xB1>(amax));  // the other run of the stretch
            // 2^-e with amax * 2^-e in [2^14, 2^15): exponent arithmetic on the bit pattern
            const int ex = (int)((__builtin_bit_cast(uint32_t, amax) >> 23) & 0xFF);
            int down = (amax > 0.f) ? (ex - 141) : 0;  // 141 = 127 + 14
            down = max(-126, min(113, down));           // keeps both exponent fields valid
            const float pre = __builtin_bit_cast(float, (uint32_t)(127 - down) << 23);
            _Float16 h[8];
            float sum = 0.f;
#pragma unroll
            for (int t = 0; t < 8; ++t) {
                h[t] = (_Float16)(f[t] * pre);
                sum += (float)h[t];  // the values the matrix cores will see
            }
            sum += dpp8_f<0xB1>(sum);
            if (r < row_runs) {
                auto pk = [](_Float16 lo, _Float16 hi) {
                    typedef __attribute__((ext_vector_type(2))) _Float16 h2;
                    const h2 v = {lo, hi};
                    return __builtin_bit_cast(uint32_t, v);
                };
                const int c = r / (kW8ChunkK / 8), rr = r % (kW8ChunkK / 8);
                const int L = rr >> 1, e = rr & 1;
                xl[(c * 2 + e) * kWave + L] = make_uint4(pk(h[0], h[1]), pk(h[2], h[3]), pk(h[4], h[5]), pk(h[6], h[7]));
                if (e == 0) {
                    const float P = __builtin_bit_cast(float, (uint32_t)(127 + down) << 23);  // exact factor
                    consts[c * kWave + L] = make_float2(P * (1152.f * sum), P);
                }
            }
        }
        // the part of the last chunk past K
        const int pad = nc * (kW8ChunkK / 8) - row_runs;
        for (int e0 = threadIdx.x; e0 < pad; e0 += kW8Threads) {
            const int r = row_runs + e0;
            const int c = r / (kW8ChunkK / 8), rr = r % (kW8ChunkK / 8);
            xl[(c * 2 + (rr & 1)) * kWave + (rr >> 1)] = make_uint4(0, 0, 0, 0);
            if ((rr & 1) == 0) consts[c * kWave + (rr >> 1)] = make_float2(0.f, 1.f);
        }
    }
    __syncthreads();
    if (total <= 0) return;

    // Results stay in registers (the wave's t-th row in lane t) and are stored once at the end: a
    // store between the loads would break the in-order completion that exact load waits rely on.
    float ykeep = 0.f;
    float acc = 0.f;
    const bool odd = lane & 1, hi = lane & 2;

    auto consume = [&](int p, int cc) {
        int xo = lane;
        asm volatile("" : "+v"(xo));  // keeps the LDS reads inside the loop
        const uint4 x0 = xl[(cc * 2) * kWave + xo], x1 = xl[(cc * 2 + 1) * kWave + xo];
        const float2 cst = consts[cc * kWave + xo];
        const uint32_t w[4] = {q[p].x, q[p].y, q[p].z, q[p].w};
        const uint2 xb[4] = {make_uint2(x0.x, x0.y), make_uint2(x0.z, x0.w), make_uint2(x1.x, x1.y), make_uint2(x1.z, x1.w)};
        f32x4_t d = {0.f, 0.f, 0.f, 0.f};  // one chain: the expansion between two MFMAs covers their latency
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            // bytes 0,1 and 2,3 of the word as fp16 pairs (1024 + u)
            const uint32_t p01 = __builtin_amdgcn_perm(0u, w[e], 0x0C010C00u) ^ 0x64806480u;
            const uint32_t p23 = __builtin_amdgcn_perm(0u, w[e], 0x0C030C02u) ^ 0x64806480u;
            d = __builtin_amdgcn_mfma_f32_4x4x4f16(__builtin_bit_cast(f16x4_t, make_uint2(p01, p23)),
                                                   __builtin_bit_cast(f16x4_t, xb[e]), d, 0, 0, 0);
        }
        // D[j][j] is register j = lane % 4
        const float e0 = odd ? d[1] : d[0], e1 = odd ? d[3] : d[2];
        const float dsel = hi ? e1 : e0;
        const float s = (float)__builtin_bit_cast(_Float16, (uint16_t)sh[p]);
        // s * 2^e * (D - 1152 * sum of the staged x)
        acc = fmaf(s, fmaf(cst.y, dsel, -cst.x), acc);
        asm volatile("" : "+v"(acc), "+v"(xo));
    };
    auto finish_row = [&](int cr) {
        const float v = wave_sum8(acc);
        ykeep = (lane == cr) ? v : ykeep;
        acc = 0.f;
        asm volatile("" ::: "memory");
    };

    int cr = 0, cc = 0;  // row and chunk being consumed
    int t = 0;
    for (; t + kW8Ring < total; t += kW8Ring) {
#pragma unroll
        for (int p = 0; p < kW8Ring; ++p) {
            consume(p, cc);
            if (__builtin_amdgcn_readfirstlane(cc == nc - 1)) finish_row(cr);
            advance(cr, cc);
            issue(p, ir, ic);
            advance(ir, ic);
            __builtin_amdgcn_sched_barrier(0);
        }
    }
#pragma unroll
    for (int p = 0; p < kW8Ring; ++p)
        if (t + p < total) {
            consume(p, cc);
            if (__builtin_amdgcn_readfirstlane(cc == nc - 1)) finish_row(cr);
            advance(cr, cc);
        }

    if (lane < nrw) a.y[s0 + wave + kW8Waves * lane] = f32_to_bf16_rne(ykeep);
}

}  // namespace

bool w8a16_stream_supports(const qail_wdesc& d, int M) {
    const int g = d.group_size;
    const bool pow2 = (g & (g - 1)) == 0;
    // a chunk of 1024 k holds a whole number of groups, or a group a power-of-two number of chunks
    const bool groups_ok = g % 16 == 0 && pow2 && (g <= kW8ChunkK || g % kW8ChunkK == 0);
    return M == 1 && d.K % 16 == 0 && d.K <= kW8MaxChunks * kW8ChunkK && groups_ok &&
           (unsigned long long)d.N * d.K < 0x80000000ull;  // 32-bit byte offsets in the kernel
}

hipError_t launch_w8a16_stream_batch(const qail_w8a16_item* items, int count, hipStream_t st) {
    for (int i0 = 0; i0 < count; i0 += kW8Batch) {
        const int n = count - i0 < kW8Batch ? count - i0 : kW8Batch;
        const qail_w8a16_item* its = items + i0;
        // blocks in proportion to the bytes, one or two blocks per CU in all; per linear fewer when there
        // are fewer than 16 rows for each block, more when a block would get more rows than its
        // waves can park results for (64 each)
        // two blocks of eight waves per CU when that leaves every wave three rows or more, else one
        // (as for the 4-bit stream: the second helping evens out the finish)
        long long rows_total = 0;
        for (int i = 0; i < n; ++i) rows_total += its[i].d.N;
        int cus = device_cu_count();
        if (rows_total >= 2LL * cus * kW8Waves * 3) cus *= 2;
        double total = 0;
        for (int i = 0; i < n; ++i) total += (double)its[i].d.N * its[i].d.K;
        W8Batch b;
        size_t lds = 0;
        int begin = 0;
        for (int i = 0; i < n; ++i) {
            const qail_wdesc& d = its[i].d;
            int blocks = (int)((double)d.N * d.K / total * cus + 0.5);
            if (blocks < 1) blocks = 1;
            const int by_rows = (d.N + kW8Waves - 1) / kW8Waves;
            if (blocks > by_rows) blocks = by_rows;
            const int need = (d.N + kW8Waves * kWave - 1) / (kW8Waves * kWave);
            if (blocks < need) blocks = need;
            const size_t nc = ((size_t)d.K + kW8ChunkK - 1) / kW8ChunkK;
            lds = std::max(lds, nc * kWave * (2 * 16 + 8));
            b.it[i] = W8Args{its[i].qweight, its[i].scales, its[i].x, its[i].y, d.N, d.K, d.group_size,
                             d.N / blocks, d.N % blocks, begin};
            begin += blocks;
        }
        for (int i = n; i < kW8Batch; ++i) b.it[i] = b.it[n - 1];
        b.count = n;
        hipLaunchKernelGGL(w8a16_stream_kernel, dim3(begin), dim3(kW8Threads), lds, st, b);
        const hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

hipError_t launch_w8a16_stream(const qail_wdesc& d, const uint32_t* qw, const uint16_t* sc, const uint16_t* x,
                               uint16_t* y, hipStream_t st) {
    const qail_w8a16_item it{d, qw, sc, x, y};
    return launch_w8a16_stream_batch(&it, 1, st);
}

}  // namespace qail
