// Host-side driver for the sanitizer test: calls the C ABI of a host-only, address- and
// undefined-behaviour-sanitized build of the library (no device code is linked in, so no kernel
// can run: a call that gets as far as a launch comes back as QAIL_ERR_HIP).  It walks the
// argument checks of every entry point, the size queries at extreme shapes, and the launchers'
// host logic (division of blocks among items, argument tables) on lists of every length.
// Exit status 0 = every expectation met; a sanitizer report aborts the process.
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <vector>

#include "qail.h"

static int failures = 0;
#define EXPECT(call, want)                                                                     \
    do {                                                                                       \
        const int got_ = (call);                                                               \
        if (got_ != (want)) {                                                                  \
            std::printf("line %d: %s = %d (%s), expected %d\n", __LINE__, #call, got_,         \
                        qail_status_string(got_), (int)(want));                                \
            ++failures;                                                                        \
        }                                                                                      \
    } while (0)
// a call that may be accepted or refused, but must do so without undefined behaviour
#define ANY(call)                                                                              \
    do {                                                                                       \
        const int got_ = (call);                                                               \
        if (got_ > 0 || got_ < QAIL_ERR_HIP) {                                                 \
            std::printf("line %d: %s = %d, not a status\n", __LINE__, #call, got_);            \
            ++failures;                                                                        \
        }                                                                                      \
    } while (0)
// reaches the launch (or a one-time attribute call) and fails there: the build has no device code
#define NO_DEVICE(call) EXPECT(call, QAIL_ERR_HIP)

template <typename T>
static T* fake(uintptr_t a) { return reinterpret_cast<T*>(a); }

int main() {
    // addresses that are never dereferenced on the host
    uint32_t* const u32 = fake<uint32_t>(0x10000);
    uint16_t* const u16 = fake<uint16_t>(0x20000);
    float* const f32 = fake<float>(0x30000);
    uint8_t* const u8 = fake<uint8_t>(0x40000);
    void* const ws = fake<void>(0x100000);
    uint32_t* const odd32 = fake<uint32_t>(0x10004);
    uint16_t* const odd16 = fake<uint16_t>(0x20002);

    EXPECT(qail_version() >= 100 ? 0 : 1, 0);
    for (int s = 1; s >= -8; --s) (void)qail_status_string(s);

    // ---- size queries, also where the products leave 32 bits
    size_t a = 0, b = 0, c = 0;
    const qail_wdesc d = {4096, 4096, 128, QAIL_W4_ASYM_GROUP};
    EXPECT(qail_packed_sizes(&d, &a, &b, &c), QAIL_OK);
    EXPECT(a == (size_t)4096 * 512 * 4 && b == (size_t)4096 * 32 * 2 && c == (size_t)4096 * 4 * 4 ? 0 : 1, 0);
    EXPECT(qail_packed_sizes(&d, nullptr, nullptr, nullptr), QAIL_OK);
    EXPECT(qail_packed_sizes(nullptr, &a, &b, &c), QAIL_ERR_NULL);
    const int32_t big = 0x7FFFFFF8;
    for (int scheme = 0; scheme <= 4; ++scheme) {
        const qail_wdesc h = {big, big, 8, scheme};
        ANY(qail_packed_sizes(&h, &a, &b, &c));
        const qail_wdesc h2 = {1, 8, 8, scheme};
        ANY(qail_packed_sizes(&h2, &a, &b, &c));
        for (int32_t M : {1, 2, 4, 5, 16, 17, 288, 65535, 65536, 0x7FFFFFFF}) {
            ANY(qail_w4a16_workspace(&h, M, &a));
            ANY(qail_w4a16_workspace(&h2, M, &a));
            ANY(qail_w8a16_workspace(&h, M, &a));
            ANY(qail_w8a16_workspace(&h2, M, &a));
        }
    }
    const qail_wdesc bad_k = {16, 12, 4, QAIL_W4_ASYM_GROUP}, bad_g = {16, 64, 48, QAIL_W4_ASYM_GROUP},
                     neg = {-1, 64, 64, QAIL_W4_ASYM_GROUP}, bad_scheme = {16, 64, 64, 77};
    for (const qail_wdesc* w : {&bad_k, &bad_g, &neg}) EXPECT(qail_packed_sizes(w, &a, &b, &c), QAIL_ERR_SHAPE);
    ANY(qail_packed_sizes(&bad_scheme, &a, &b, &c));
    EXPECT(qail_w4a16_workspace(&d, 0, &a), QAIL_ERR_SHAPE);
    EXPECT(qail_w4a16_workspace(&d, 1, nullptr), QAIL_ERR_NULL);
    EXPECT(qail_w4a16_workspace(nullptr, 1, &a), QAIL_ERR_NULL);
    EXPECT(qail_static_scratch_bytes(nullptr), QAIL_ERR_NULL);
    EXPECT(qail_static_scratch_bytes(&a), QAIL_OK);
    EXPECT(qail_lsq_backward_workspace(nullptr), QAIL_ERR_NULL);
    EXPECT(qail_lsq_backward_workspace(&a), QAIL_OK);

    // ---- quantisers
    EXPECT(qail_quantize_weights(&d, nullptr, u32, u16, u32, nullptr, nullptr), QAIL_ERR_NULL);
    EXPECT(qail_quantize_weights(&d, f32, u32, u16, nullptr, nullptr, nullptr), QAIL_ERR_NULL);
    EXPECT(qail_quantize_weights(&d, f32, odd32, u16, u32, nullptr, nullptr), QAIL_ERR_ALIGN);
    EXPECT(qail_quantize_weights(nullptr, f32, u32, u16, u32, nullptr, nullptr), QAIL_ERR_NULL);
    EXPECT(qail_quantize_weights(&bad_k, f32, u32, u16, u32, nullptr, nullptr), QAIL_ERR_SHAPE);
    EXPECT(qail_unpack_weights(&d, u32, nullptr, nullptr), QAIL_ERR_NULL);
    EXPECT(qail_act_scale_u4(f32, 8, nullptr, nullptr), QAIL_ERR_NULL);
    EXPECT(qail_quantize_act_u4(f32, 12, f32, u32, nullptr), QAIL_ERR_SHAPE);
    EXPECT(qail_quantize_act_u4(nullptr, 0, nullptr, nullptr, nullptr), QAIL_OK);
    EXPECT(qail_act_scale_s8(f32, 8, nullptr, nullptr), QAIL_ERR_NULL);
    EXPECT(qail_quantize_act_s8(f32, 6, f32, u32, nullptr), QAIL_ERR_SHAPE);
    EXPECT(qail_fake_quant_w4(&d, nullptr, f32, nullptr), QAIL_ERR_NULL);
    EXPECT(qail_lsq_forward(f32, 8, nullptr, -8, 7, f32, nullptr), QAIL_ERR_NULL);
    EXPECT(qail_lsq_forward(f32, 8, f32, 1, 7, f32, nullptr), QAIL_ERR_SHAPE);
    EXPECT(qail_lsq_backward(f32, f32, 8, f32, -8, 7, 1.f, f32, f32, nullptr, 0, nullptr), QAIL_ERR_WORKSPACE);
    EXPECT(qail_qbc_loss(f32, f32, 0, 8, f32, nullptr, ws, 1 << 20, nullptr), QAIL_ERR_SHAPE);
    EXPECT(qail_qbc_loss(f32, f32, 4, 8, f32, nullptr, nullptr, 0, nullptr), QAIL_ERR_WORKSPACE);

    // ---- W4A16: argument checks, then the launchers' host logic for lists of every length
    EXPECT(qail_w4a16_linear(&d, u32, u16, u32, u16, u16, 0, nullptr, 0, nullptr), QAIL_ERR_SHAPE);
    EXPECT(qail_w4a16_linear(&d, u32, u16, u32, nullptr, u16, 1, nullptr, 0, nullptr), QAIL_ERR_NULL);
    EXPECT(qail_w4a16_linear(&d, u32, u16, odd32, u16, u16, 1, nullptr, 0, nullptr), QAIL_ERR_ALIGN);
    EXPECT(qail_w4a16_linear_batch(nullptr, 0, 1, nullptr, 0, nullptr), QAIL_OK);
    EXPECT(qail_w4a16_linear_batch(nullptr, 2, 1, nullptr, 0, nullptr), QAIL_ERR_NULL);
    EXPECT(qail_w4a16_linear_batch(nullptr, -1, 1, nullptr, 0, nullptr), QAIL_ERR_SHAPE);
    const int32_t shapes[][3] = {{12288, 4096, 128}, {4096, 4096, 128}, {22016, 4096, 128}, {4096, 11008, 128},
                                 {8, 32, 32},        {40, 64, 64},      {301, 192, 64},     {4, 12288, 128},
                                 {128256, 4096, 128}, {16, 16384, 128}, {7, 40, 8},         {64, 256, 256}};
    const int nshapes = (int)(sizeof(shapes) / sizeof(shapes[0]));
    for (int count : {1, 2, 3, 4, 7, 8, 9, 15, 16, 17, 31, 32, 33, 40, 100}) {
        std::vector<qail_w4a16_item> items(count);
        std::vector<qail_w8a16_item> items8(count);
        std::vector<qail_lora> loras(count);
        for (int i = 0; i < count; ++i) {
            const int32_t* s = shapes[(i * 5 + count) % nshapes];
            items[i] = {{s[0], s[1], s[2], QAIL_W4_ASYM_GROUP}, u32, u16, u32, u16, u16};
            items8[i] = {{s[0], s[1], s[2], QAIL_W8_SYM_GROUP}, u32, u16, u16, u16};
            loras[i] = {u16, u16, 8 * (1 + i % 8), 0.5f};
        }
        for (int32_t M : {1, 2, 4, 5, 16, 17, 64, 288}) {
            size_t need = 0;
            EXPECT(qail_w4a16_batch_workspace(items.data(), count, M, &need), QAIL_OK);
            // a workspace is claimed but never touched by the host; with room enough the call reaches a launch
            NO_DEVICE(qail_w4a16_linear_batch(items.data(), count, M, ws, (size_t)1 << 40, nullptr));
            if (need) EXPECT(qail_w4a16_linear_batch(items.data(), count, M, ws, need - 1, nullptr), QAIL_ERR_WORKSPACE);
            ANY(qail_w8a16_batch_workspace(items8.data(), count, M, &need));
            ANY(qail_w8a16_linear_batch(items8.data(), count, M, ws, (size_t)1 << 40, nullptr));
            ANY(qail_w4a16_lora_workspace(items.data(), loras.data(), count, M, &need));
            ANY(qail_w4a16_linear_lora_batch(items.data(), loras.data(), count, M, ws, (size_t)1 << 40, nullptr));
            ANY(qail_w4a16_linear_lora_batch_static(items.data(), loras.data(), count, M, nullptr));
        }
        size_t need = 0;
        ANY(qail_w4a16_chain_workspace(items.data(), count, &need));
        ANY(qail_w4a16_linear_chain(items.data(), count, ws, (size_t)1 << 40, nullptr));
    }
    {
        qail_w4a16_item it = {d, u32, u16, u32, u16, u16};
        qail_lora lo = {u16, u16, 32, 1.f};
        EXPECT(qail_w4a16_linear_lora_batch(&it, nullptr, 1, 1, ws, 1 << 20, nullptr), QAIL_ERR_NULL);
        EXPECT(qail_w4a16_linear_lora_batch(&it, &lo, 1, 1, nullptr, 0, nullptr), QAIL_ERR_WORKSPACE);
        EXPECT(qail_w4a16_lora_workspace(&it, &lo, 1, 3, nullptr), QAIL_ERR_NULL);
        EXPECT(qail_w4a16_lora_workspace(&it, &lo, 1, 65536, &a), QAIL_ERR_UNSUPPORTED);
        lo.r = 7;
        EXPECT(qail_w4a16_linear_lora_batch(&it, &lo, 1, 1, ws, 1 << 20, nullptr), QAIL_ERR_SHAPE);
        lo.r = 32;
        lo.A = odd16;
        EXPECT(qail_w4a16_linear_lora_batch(&it, &lo, 1, 1, ws, 1 << 20, nullptr), QAIL_ERR_ALIGN);
        EXPECT(qail_w4a16_linear_chain(&it, 1, nullptr, 0, nullptr), QAIL_ERR_WORKSPACE);
        EXPECT(qail_w4a16_linear_chain(&it, 1, ws, 100, nullptr), QAIL_ERR_WORKSPACE);
        EXPECT(qail_w4a16_linear_chain(&it, -1, nullptr, 0, nullptr), QAIL_ERR_SHAPE);
        EXPECT(qail_w4a16_chain_workspace(nullptr, 1, &a), QAIL_ERR_NULL);
    }

    // ---- convolutions: every geometry check, then the launcher's tile choice and magic numbers
    const qail_conv_desc cv = {32, 56, 56, 64, 64, 3, 3, 1, 1};
    int32_t* const i32 = fake<int32_t>(0x50000);
    EXPECT(qail_w4a4_workspace(&cv, &a), QAIL_OK);
    EXPECT(qail_w4a4_workspace(nullptr, &a), QAIL_ERR_NULL);
    EXPECT(qail_w4a4_gemm(&cv, u32, u32, nullptr, nullptr, nullptr, nullptr, nullptr, 0, nullptr), QAIL_ERR_NULL);
    EXPECT(qail_w4a4_gemm(&cv, u32, u32, nullptr, nullptr, f32, f32, nullptr, 0, nullptr), QAIL_ERR_NULL);
    EXPECT(qail_w4a4_gemm(&cv, u32, odd32, i32, nullptr, nullptr, nullptr, nullptr, 0, nullptr), QAIL_ERR_ALIGN);
    EXPECT(qail_w4a4_conv_u4(&cv, u32, u32, f32, f32, 0.f, nullptr, 0.f, nullptr, u32, nullptr, 0, nullptr), QAIL_ERR_SHAPE);
    EXPECT(qail_w4a4_conv_u4(&cv, u32, u32, f32, f32, 0.5f, u32, 0.1f, f32, u32, nullptr, 0, nullptr), QAIL_ERR_SHAPE);
    EXPECT(qail_w4a4_conv_u4(&cv, u32, u32, f32, f32, 0.5f, u32, -1.f, nullptr, u32, nullptr, 0, nullptr), QAIL_ERR_SHAPE);
    EXPECT(qail_w4a4_conv_u4(&cv, u32, u32, f32, f32, 0.5f, nullptr, 0.f, nullptr, nullptr, nullptr, 0, nullptr), QAIL_ERR_NULL);
    const int32_t dims[] = {-1, 0, 1, 2, 3, 7, 8, 32, 56, 224, 1024, 46341, 0x7FFFFFFF};
    for (int32_t B : {1, 32, 0x7FFFFFFF})
        for (int32_t H : dims)
            for (int32_t C : {-8, 0, 4, 8, 32, 64, 520, 0x7FFFFFF8})
                for (int32_t k : {0, 1, 3, 7, 64})
                    for (int32_t st : {0, 1, 2, 5})
                        for (int32_t pad : {-1, 0, 1, 3, 100}) {
                            const qail_conv_desc g = {B, H, H, C, C, k, k, st, pad};
                            ANY(qail_w4a4_workspace(&g, &a));
                            ANY(qail_w4a4_gemm(&g, u32, u32, i32, f32, f32, f32, nullptr, 0, nullptr));
                            ANY(qail_w4a4_conv_u4(&g, u32, u32, f32, f32, 0.37f, u32, 0.1f, nullptr, u32, nullptr, 0, nullptr));
                            ANY(qail_w8a8_gemm(&g, u32, u32, i32, f32, f32, f32, nullptr, 0, nullptr));
                        }

    // ---- single linears that reach a launch
    for (const auto& s : shapes) {
        const qail_wdesc w = {s[0], s[1], s[2], QAIL_W4_ASYM_GROUP}, w8 = {s[0], s[1], s[2], QAIL_W8_SYM_GROUP};
        for (int32_t M : {1, 3, 9, 40}) {
            ANY(qail_w4a16_linear(&w, u32, u16, u32, u16, u16, M, ws, (size_t)1 << 40, nullptr));
            ANY(qail_w8a16_linear(&w8, u32, u16, u16, u16, M, ws, (size_t)1 << 40, nullptr));
        }
        ANY(qail_quantize_weights(&w, f32, u32, u16, u32, nullptr, nullptr));
        ANY(qail_unpack_weights(&w, u32, u8, nullptr));
        ANY(qail_fake_quant_w4(&w, f32, f32, nullptr));
    }
    ANY(qail_act_scale_u4(f32, (size_t)1 << 40, f32, nullptr));
    ANY(qail_quantize_act_u4(f32, (size_t)1 << 40, f32, u32, nullptr));
    ANY(qail_lsq_forward(f32, (size_t)1 << 40, f32, -8, 7, f32, nullptr));
    ANY(qail_lsq_backward(f32, f32, (size_t)1 << 40, f32, -8, 7, 1.f, f32, f32, ws, (size_t)1 << 40, nullptr));
    ANY(qail_qbc_loss(f32, f32, 0x7FFFFFFF, 0x7FFFFFFF, f32, f32, ws, (size_t)1 << 40, nullptr));

    if (failures) {
        std::printf("%d expectation(s) failed\n", failures);
        return 1;
    }
    std::printf("host sanitizer driver: ok\n");
    return 0;
}
