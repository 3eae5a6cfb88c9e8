// W4A4 convolution as an implicit GEMM with exact int32 accumulation.
//
//   acc[(b,oh,ow)][n] = sum_{kh,kw,c} a[b][oh*s+kh-p][ow*s+kw-p][c] * w[n][kh][kw][c]
//
// Sec. 2.1 / Sec. 5.1: the driving policy's convolutions are compute-bound, so both
// GEMM operands are 4-bit integers.  CDNA4 has no 4-bit integer matrix
// instruction, so nibbles are widened to int8 in registers and fed to
// v_mfma_i32_16x16x64_i8 (int32 accumulate):
//   * unsigned activation codes:  w & 0x0F0F0F0F  and (w >> 4) & 0x0F0F0F0F
//     give the even and the odd codes of a word as bytes;
//   * signed weight codes are moved to the HIGH nibble of each byte,
//     (w << 4) & 0xF0F0F0F0 and w & 0xF0F0F0F0, which is the int8 value 16*code,
//     so no sign extension is needed; the accumulator is 16x the result and an
//     arithmetic shift by 4 restores it exactly.
// The two operands are permuted along k in the same way (even codes, then odd
// codes of each word), which leaves the sum unchanged.
//
// MFMA operand layout (16x16x64 int8, wave64): lane l supplies row (A) / column
// (B) l%16 and the 16 consecutive k starting at 16*(l/16); it receives
// D[4*(l/16)+r][l%16], r = 0..3.  A = activations (rows m), B = weights (columns n).
//
// Tiling: a block of 4 waves (2 x 2) owns a BM x BN output tile and walks K in
// steps of 128 codes (16 packed words per row; K is ordered (kh, kw, c), so a step
// is a run of channels of one or two filter taps).  Nibbles stay packed in LDS
// (half the LDS traffic of int8); global loads run several steps ahead in a register
// ring and are moved to one of two LDS buffers when they are due, one barrier per step.
// Zero padding costs nothing: code 0 of the unsigned activations is the value 0.
#include "qail_internal.h"

namespace qail {

namespace {

constexpr int kStepWords = 16;  // packed words per row per K step (128 codes)
constexpr int kPitchW = 18;     // words per LDS row: 8-byte aligned, conflict-free for the fragment reads

struct ConvGeom {
    int B, H, W, Cin, Cout, KH, KW, stride, pad, OH, OW, M;
};

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
};

// One output element of the fused epilogue (Sec. 5.1: every activation tensor of the driving
// encoder is 4-bit with one step per tensor, so the consumer's step is known here).  Each
// line is one correctly rounded fp32 operation; contraction to fma is switched off because
// the code is decided by these roundings and must equal the reference bit for bit.
__device__ __forceinline__ uint32_t fused_code(int acc, float scale, float bias, float r, float s_out) {
#pragma clang fp contract(off)
    float t = (float)acc * scale;
    t = t + bias;
    t = t + r;
    t = fmaxf(t, 0.f);
    const float q = __builtin_rintf(t / s_out);
    return (uint32_t)fminf(q, 15.f);
}

// 8 consecutive channels of one output pixel -> one packed word.
__device__ __forceinline__ uint32_t fused_word(const int (&acc)[8], const ConvOut& o, size_t m, int n0, int cout) {
    const float4 s0 = *reinterpret_cast<const float4*>(o.scale + n0), s1 = *reinterpret_cast<const float4*>(o.scale + n0 + 4);
    const float4 b0 = *reinterpret_cast<const float4*>(o.bias + n0), b1 = *reinterpret_cast<const float4*>(o.bias + n0 + 4);
    const float sc[8] = {s0.x, s0.y, s0.z, s0.w, s1.x, s1.y, s1.z, s1.w};
    const float bi[8] = {b0.x, b0.y, b0.z, b0.w, b1.x, b1.y, b1.z, b1.w};
    float r[8];
    if (o.res_u4) {
        const uint32_t rw = o.res_u4[m * (size_t)(cout / 8) + n0 / 8];
#pragma unroll
        for (int e = 0; e < 8; ++e) {
#pragma clang fp contract(off)
            r[e] = o.res_scale * (float)((rw >> (4 * e)) & 0xFu);
        }
    } else if (o.res_f32) {
        const float4 r0 = *reinterpret_cast<const float4*>(o.res_f32 + m * (size_t)cout + n0);
        const float4 r1 = *reinterpret_cast<const float4*>(o.res_f32 + m * (size_t)cout + n0 + 4);
        r[0] = r0.x; r[1] = r0.y; r[2] = r0.z; r[3] = r0.w; r[4] = r1.x; r[5] = r1.y; r[6] = r1.z; r[7] = r1.w;
    } else {
#pragma unroll
        for (int e = 0; e < 8; ++e) r[e] = 0.f;
    }
    uint32_t word = 0;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        // without a shortcut r is 0 and t + 0 == t (a -0 becomes +0; both end as code 0)
        word |= fused_code(acc[e], sc[e], bi[e], r[e], o.s_out) << (4 * e);
    }
    return word;
}

template <int BM, int BN, int kDepth>
__global__ __launch_bounds__(256, (BM * BN >= 128 * 128 ? 2 : 4)) void w4a4_conv_kernel(
    const ConvGeom gm, const uint32_t* __restrict__ a, const uint32_t* __restrict__ w, const ConvOut out) {
    int32_t* const acc_out = out.acc;
    const float* const scale = out.scale;
    const float* const bias = out.bias;
    float* const y_out = out.y;
    constexpr int kAR = BM / 64;   // A rows per thread
    constexpr int kBR = BN / 64;   // B rows per thread
    constexpr int kTM = BM / 32;   // MFMA tiles per wave along m
    constexpr int kTN = BN / 32;   // ... along n
    // [2][BM] activation rows, then [2][BN] weight rows, kPitchW words each; the fused epilogue
    // reuses the space as an int32 staging tile
    __shared__ __attribute__((aligned(16))) uint32_t smem[2 * (BM + BN) * kPitchW];
    uint32_t* const As0 = smem;
    uint32_t* const Bs0 = smem + 2 * BM * kPitchW;

    const int t = threadIdx.x;
    const int lane = t % kWave;
    const int wave = __builtin_amdgcn_readfirstlane(t / kWave);
    const int wm = wave / 2, wn = wave % 2;
    const int bm = blockIdx.y * BM, bn = blockIdx.x * BN;
    const int cw = gm.Cin / 8;                 // words per pixel
    const int kwords = gm.KH * gm.KW * cw;     // words per filter
    const int steps = (kwords + kStepWords - 1) / kStepWords;
    const int ntaps = gm.KH * gm.KW;

    const __amdgpu_buffer_rsrc_t ra = make_rsrc(a, (uint32_t)((size_t)gm.B * gm.H * gm.W * cw * 4));
    const __amdgpu_buffer_rsrc_t rw = make_rsrc(w, (uint32_t)((size_t)gm.Cout * kwords * 4));

    // Loader geometry: thread t loads words [4q, 4q+4) of a step for rows t/4 + 64*i: the four
    // lanes of a row fetch 64 contiguous bytes.
    const int q = t & 3, lrow = t >> 2;
    int abase[kAR];       // byte offset of (b, ih0, iw0, 0); may be negative at the border
    uint32_t amask[kAR];  // bit tap = the tap's pixel is inside the image
#pragma unroll
    for (int i = 0; i < kAR; ++i) {
        const int m = bm + lrow + 64 * i;
        abase[i] = 0;
        amask[i] = 0;
        if (m < gm.M) {
            const int b = m / (gm.OH * gm.OW);
            const int rem = m - b * (gm.OH * gm.OW);
            const int oh = rem / gm.OW, ow = rem - oh * gm.OW;
            const int ih0 = oh * gm.stride - gm.pad, iw0 = ow * gm.stride - gm.pad;
            abase[i] = ((b * gm.H + ih0) * gm.W + iw0) * cw * 4;
            for (int kh = 0; kh < gm.KH; ++kh)
                for (int kwi = 0; kwi < gm.KW; ++kwi)
                    if (ih0 + kh >= 0 && ih0 + kh < gm.H && iw0 + kwi >= 0 && iw0 + kwi < gm.W)
                        amask[i] |= 1u << (kh * gm.KW + kwi);
        }
    }
    uint32_t bbase[kBR];
#pragma unroll
    for (int i = 0; i < kBR; ++i) {
        const int n = bn + lrow + 64 * i;
        bbase[i] = n < gm.Cout ? (uint32_t)n * kwords * 4 : kOut;
    }

    // Register ring of kDepth K-steps of loads: a step's loads are issued kDepth steps before
    // they are needed (a step is only a few hundred MFMA cycles, far less than a cache
    // latency).  Nothing about a load is conditional, so the loads in flight at every wait are
    // known at compile time.
    u32x4_t ar[kDepth][kAR], br[kDepth][kBR];
    // position of the next step to issue (per thread: it depends on q), advanced without divisions
    int nkw0 = 4 * q, ncword = 4 * q, ntap = 0, ntapoff = 0, nkwi = 0;
    auto advance = [&](int words) {
        nkw0 += words;
        ncword += words;
        while (ncword >= cw) {
            ncword -= cw;
            ++ntap;
            ntapoff += cw * 4;
            if (++nkwi == gm.KW) { nkwi = 0; ntapoff += (gm.W - gm.KW) * cw * 4; }
        }
    };
    advance(0);
    auto issue = [&](int d) {
        const bool kin = ntap < ntaps;
        const int koff = ntapoff + ncword * 4;  // bytes from (ih0, iw0, 0) to this tap's words
#pragma unroll
        for (int i = 0; i < kAR; ++i) {
            const bool in = kin && ((amask[i] >> ntap) & 1u);
            ar[d][i] = __builtin_amdgcn_raw_buffer_load_b128(ra, in ? (uint32_t)(abase[i] + koff) : kOut, 0, 0);
        }
#pragma unroll
        for (int i = 0; i < kBR; ++i)
            br[d][i] = __builtin_amdgcn_raw_buffer_load_b128(rw, kin ? bbase[i] + (uint32_t)nkw0 * 4 : kOut, 0, 0);
        advance(kStepWords);
    };
    auto store_lds = [&](int d, int buf) {
#pragma unroll
        for (int i = 0; i < kAR; ++i) {
            uint2* dst = reinterpret_cast<uint2*>(&As0[buf * BM * kPitchW + (lrow + 64 * i) * kPitchW + 4 * q]);
            dst[0] = make_uint2(ar[d][i].x, ar[d][i].y);
            dst[1] = make_uint2(ar[d][i].z, ar[d][i].w);
        }
#pragma unroll
        for (int i = 0; i < kBR; ++i) {
            uint2* dst = reinterpret_cast<uint2*>(&Bs0[buf * BN * kPitchW + (lrow + 64 * i) * kPitchW + 4 * q]);
            dst[0] = make_uint2(br[d][i].x, br[d][i].y);
            dst[1] = make_uint2(br[d][i].z, br[d][i].w);
        }
    };

    i32x4_t acc[kTM][kTN];
#pragma unroll
    for (int i = 0; i < kTM; ++i)
#pragma unroll
        for (int j = 0; j < kTN; ++j) acc[i][j] = i32x4_t{0, 0, 0, 0};

#pragma unroll
    for (int d = 0; d < kDepth; ++d) {
        issue(d);  // steps past the end of K read nothing
        __builtin_amdgcn_sched_barrier(0);
    }

    for (int s0 = 0; s0 < steps; s0 += kDepth) {
#pragma unroll
        for (int d = 0; d < kDepth; ++d) {
            if (s0 + d >= steps) break;
            const int buf = d & 1;  // kDepth is even
            store_lds(d, buf);
            issue(d);
            __builtin_amdgcn_sched_barrier(0);
            __syncthreads();
#pragma unroll
            for (int sub = 0; sub < 2; ++sub) {  // two MFMA k-steps of 64 codes (8 words)
                i32x4_t af[kTM], bf[kTN];
#pragma unroll
                for (int i = 0; i < kTM; ++i) {
                    const uint2 p = *reinterpret_cast<const uint2*>(
                        &As0[buf * BM * kPitchW + (wm * (BM / 2) + i * 16 + (lane & 15)) * kPitchW + sub * 8 + (lane >> 4) * 2]);
                    af[i] = i32x4_t{(int)(p.x & 0x0F0F0F0Fu), (int)((p.x >> 4) & 0x0F0F0F0Fu),
                                    (int)(p.y & 0x0F0F0F0Fu), (int)((p.y >> 4) & 0x0F0F0F0Fu)};
                }
#pragma unroll
                for (int j = 0; j < kTN; ++j) {
                    const uint2 p = *reinterpret_cast<const uint2*>(
                        &Bs0[buf * BN * kPitchW + (wn * (BN / 2) + j * 16 + (lane & 15)) * kPitchW + sub * 8 + (lane >> 4) * 2]);
                    bf[j] = i32x4_t{(int)((p.x << 4) & 0xF0F0F0F0u), (int)(p.x & 0xF0F0F0F0u),
                                    (int)((p.y << 4) & 0xF0F0F0F0u), (int)(p.y & 0xF0F0F0F0u)};
                }
#pragma unroll
                for (int i = 0; i < kTM; ++i)
#pragma unroll
                    for (int j = 0; j < kTN; ++j)
                        acc[i][j] = __builtin_amdgcn_mfma_i32_16x16x64_i8(af[i], bf[j], acc[i][j], 0, 0, 0);
            }
        }
    }

    if (out.out_u4) {
        // Fused output: the accumulators of half the tile's rows at a time are staged in LDS
        // (pitch BN + 4 words: conflict-free for the writes below), then every thread turns 8
        // consecutive channels of a pixel into one packed word.
        constexpr int kSPitch = BN + 4;
        static_assert((BM / 2) * kSPitch <= 2 * (BM + BN) * kPitchW, "staging tile must fit");
        int32_t* const stage = reinterpret_cast<int32_t*>(smem);
        constexpr int kWordsPerRow = BN / 8;
#pragma unroll
        for (int pass = 0; pass < 2; ++pass) {
            __syncthreads();  // the operand tiles (or the previous pass) are no longer read
            if (wm == pass) {
#pragma unroll
                for (int i = 0; i < kTM; ++i)
#pragma unroll
                    for (int j = 0; j < kTN; ++j)
#pragma unroll
                        for (int r = 0; r < 4; ++r)
                            stage[(i * 16 + (lane >> 4) * 4 + r) * kSPitch + wn * (BN / 2) + j * 16 + (lane & 15)] =
                                acc[i][j][r] >> 4;  // exact: the accumulator is 16 * result
            }
            __syncthreads();
            for (int idx = t; idx < (BM / 2) * kWordsPerRow; idx += 256) {
                const int row = idx / kWordsPerRow, wd = idx % kWordsPerRow;
                const int m = bm + pass * (BM / 2) + row, n0 = bn + wd * 8;
                if (m >= gm.M || n0 >= gm.Cout) continue;
                const i32x4_t v0 = *reinterpret_cast<const i32x4_t*>(&stage[row * kSPitch + wd * 8]);
                const i32x4_t v1 = *reinterpret_cast<const i32x4_t*>(&stage[row * kSPitch + wd * 8 + 4]);
                const int av[8] = {v0[0], v0[1], v0[2], v0[3], v1[0], v1[1], v1[2], v1[3]};
                out.out_u4[(size_t)m * (gm.Cout / 8) + n0 / 8] = fused_word(av, out, (size_t)m, n0, gm.Cout);
            }
        }
        return;
    }

    // Epilogue through buffer stores: rows past M and columns past Cout get an offset past the
    // end and are dropped.
    const uint32_t out_bytes = (uint32_t)((size_t)gm.M * gm.Cout * 4);
    const __amdgpu_buffer_rsrc_t racc = make_rsrc(acc_out, acc_out ? out_bytes : 0);
    const __amdgpu_buffer_rsrc_t ry = make_rsrc(y_out, y_out ? out_bytes : 0);
    const int m0 = bm + wm * (BM / 2) + (lane >> 4) * 4;
    const int n0 = bn + wn * (BN / 2) + (lane & 15);
#pragma unroll
    for (int j = 0; j < kTN; ++j) {
        const int n = n0 + j * 16;
        const bool nin = n < gm.Cout;
        const float sc = (y_out && nin) ? scale[n] : 0.f;
        const float bi = (y_out && nin) ? bias[n] : 0.f;
#pragma unroll
        for (int i = 0; i < kTM; ++i)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int m = m0 + i * 16 + r;
                const uint32_t off = (nin && m < gm.M) ? (uint32_t)(m * gm.Cout + n) * 4 : kOut;
                const int v = acc[i][j][r] >> 4;  // exact: the accumulator is 16 * result
                if (acc_out) __builtin_amdgcn_raw_buffer_store_b32((uint32_t)v, racc, off, 0, 0);
                if (y_out) __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(uint32_t, fmaf((float)v, sc, bi)), ry, off, 0, 0);
            }
    }
}

// Any Cin % 8 == 0: one thread per output.  Slow; for shapes whose Cin is not a
// multiple of 32, more than 32 filter taps, or tensors of 4 GB and more.
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
    const int cw = gm.Cin / 8;
    int acc = 0;
    for (int kh = 0; kh < gm.KH; ++kh)
        for (int kwi = 0; kwi < gm.KW; ++kwi) {
            const int ih = oh * gm.stride + kh - gm.pad, iw = ow * gm.stride + kwi - gm.pad;
            if (ih < 0 || ih >= gm.H || iw < 0 || iw >= gm.W) continue;
            const uint32_t* ap = a + ((size_t)(b * gm.H + ih) * gm.W + iw) * cw;
            const uint32_t* wp = w + ((size_t)(n * gm.KH + kh) * gm.KW + kwi) * cw;
            for (int c = 0; c < cw; ++c) {
                const uint32_t av = ap[c], wv = wp[c];
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    const int qa = (av >> (4 * j)) & 0xF;
                    const int qw = (int)(((wv >> (4 * j)) & 0xFu) ^ 8u) - 8;
                    acc += qa * qw;
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

int conv_cus() {
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

template <int BM, int BN, int kDepth>
void launch_tiled(const ConvGeom& gm, const uint32_t* a, const uint32_t* w, const ConvOut& out, hipStream_t st) {
    dim3 grid((gm.Cout + BN - 1) / BN, (gm.M + BM - 1) / BM);
    hipLaunchKernelGGL((w4a4_conv_kernel<BM, BN, kDepth>), grid, dim3(256), 0, st, gm, a, w, out);
}

}  // namespace

namespace {
hipError_t launch_conv(const qail_conv_desc& d, const uint32_t* a, const uint32_t* w, const ConvOut& out,
                       hipStream_t st) {
    ConvGeom gm;
    gm.B = d.B; gm.H = d.H; gm.W = d.W; gm.Cin = d.Cin; gm.Cout = d.Cout;
    gm.KH = d.KH; gm.KW = d.KW; gm.stride = d.stride; gm.pad = d.pad;
    gm.OH = (d.H + 2 * d.pad - d.KH) / d.stride + 1;
    gm.OW = (d.W + 2 * d.pad - d.KW) / d.stride + 1;
    gm.M = d.B * gm.OH * gm.OW;
    const bool fits32 = (size_t)gm.B * gm.H * gm.W * (gm.Cin / 2) < 0xFFFFFFF0ull &&
                        (size_t)gm.Cout * gm.KH * gm.KW * (gm.Cin / 2) < 0xFFFFFFF0ull &&
                        (size_t)gm.M * gm.Cout * 4 < 0xFFFFFFF0ull;
    if (d.Cin % 32 == 0 && d.KH * d.KW <= 32 && fits32) {
        // the largest tile that still gives every CU about two blocks
        const long long want = 2LL * conv_cus();
        auto blocks = [&](int bm, int bn) {
            return (long long)((gm.M + bm - 1) / bm) * ((gm.Cout + bn - 1) / bn);
        };
        const bool wide = gm.Cout > 64;
        if (wide && blocks(128, 128) >= want) launch_tiled<128, 128, 2>(gm, a, w, out, st);
        else if (blocks(128, 64) >= want) launch_tiled<128, 64, 2>(gm, a, w, out, st);
        else if (wide && blocks(64, 128) >= want / 2) launch_tiled<64, 128, 2>(gm, a, w, out, st);
        else launch_tiled<64, 64, 2>(gm, a, w, out, st);
    } else if (out.out_u4) {
        const size_t words = (size_t)gm.M * (d.Cout / 8);
        hipLaunchKernelGGL(w4a4_generic_u4_kernel, dim3((unsigned)((words + 255) / 256)), dim3(256), 0, st, gm,
                           a, w, out);
    } else {
        const size_t outs = (size_t)gm.M * d.Cout;
        hipLaunchKernelGGL(w4a4_generic_kernel, dim3((unsigned)((outs + 255) / 256)), dim3(256), 0, st, gm,
                           a, w, out);
    }
    return hipGetLastError();
}
}  // namespace

hipError_t launch_w4a4_conv(const qail_conv_desc& d, const uint32_t* a, const uint32_t* w, int32_t* acc,
                            const float* scale, const float* bias, float* y, hipStream_t st) {
    const ConvOut out{acc, scale, bias, y, nullptr, nullptr, nullptr, 1.f, 0.f};
    return launch_conv(d, a, w, out, st);
}

hipError_t launch_w4a4_conv_u4(const qail_conv_desc& d, const uint32_t* a, const uint32_t* w, const float* scale,
                               const float* bias, float s_out, const uint32_t* res_u4, float res_scale,
                               const float* res_f32, uint32_t* out_u4, hipStream_t st) {
    const ConvOut out{nullptr, scale, bias, nullptr, out_u4, res_u4, res_f32, s_out, res_scale};
    return launch_conv(d, a, w, out, st);
}

}  // namespace qail
