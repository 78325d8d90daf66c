// Calls the host-only part of the C ABI (size queries, the three plan builders, the bit allocator, status strings and
// the argument checks that return before any launch) with heap buffers of exactly the documented sizes.  The library's
// host code (csrc/aq_api.hip) is compiled into this program with -fsanitize=address,undefined on the host pass by
// tests/test_sanitizers.py; the kernels' launchers come from the ordinary libaq.so and are never reached: no call here
// gets past validation with pointers that a kernel would follow.  Needs no GPU.  Prints "ok" and exits 0.
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>
#include "aq.h"

#define CHECK(c) do { if (!(c)) { std::fprintf(stderr, "check failed at line %d: %s\n", __LINE__, #c); return 1; } } while (0)

int main()
{
    for (int s = 1; s >= -8; --s) CHECK(aq_status_string(s) != nullptr);
    CHECK(aq_packed_size(4096, 4096, 2, 32) == (size_t)4096 * 4096 * 5 / 16 + 256);
    CHECK(aq_packed_size(1, 32, 5, 32) == 0 && aq_packed_size(1, 33, 2, 32) == 0 && aq_packed_size(0, 32, 2, 32) == 0);
    CHECK(aq2_packed_size(4096, 4096, 2, 32) > 0 && aq2_packed_size(4096, 4096, 7, 32) == 0);
    CHECK(aq_qgemm_workspace_size(300, 4096, 4096, 2) > 0);
    CHECK(aq_hsic_workspace_size(513) > 0);

    // fake, aligned, never followed device addresses
    auto dev = [](uintptr_t i) { return reinterpret_cast<void*>((uintptr_t)0x7000000000ull + i * 0x1000000ull); };

    // decode list plans: sizes 1 .. 40 products of mixed shapes and widths, exact-size and one-byte-short buffers
    for (int count : {1, 3, 40}) {
        std::vector<aq_gemv_desc> d(count);
        for (int i = 0; i < count; ++i) {
            d[i].packed = dev(3 * i); d[i].x = dev(3 * i + 1); d[i].y = (float*)dev(3 * i + 2);
            d[i].N = 1 + 517 * (i % 5); d[i].K = 32 * (1 + 43 * (i % 4)); d[i].bits = 2 + i % 3;
            d[i].x_dtype = i % 2 ? AQ_BF16 : AQ_F16;
        }
        const size_t bytes = aq_qgemv_batch_plan_size(d.data(), count, 32);
        CHECK(bytes > 0);
        void* plan = std::malloc(bytes);
        CHECK(aq_qgemv_batch_plan(d.data(), count, 32, plan, bytes) == AQ_OK);
        CHECK(aq_qgemv_batch_plan(d.data(), count, 32, plan, bytes - 1) == AQ_ESIZE);
        CHECK(aq2_qgemv_batch_plan(d.data(), count, 32, plan, bytes) == AQ_OK);
        CHECK(aq_qgemv_batch(plan, nullptr, nullptr) == AQ_ENULL);
        d[count - 1].bits = 5;
        CHECK(aq_qgemv_batch_plan(d.data(), count, 32, plan, bytes) == AQ_EINVAL);
        std::memset(plan, 0, bytes);
        CHECK(aq_qgemv_batch(plan, dev(1), nullptr) != AQ_OK);          // not a plan image
        std::free(plan);
    }
    CHECK(aq_qgemv_batch_plan_size(nullptr, 1, 32) == 0);

    // prefill list plans
    for (int count : {1, 7}) {
        std::vector<aq_gemm_desc> d(count);
        for (int i = 0; i < count; ++i) {
            d[i].packed = dev(3 * i); d[i].X = dev(100 + i / 3); d[i].Y = (float*)dev(200 + i);
            d[i].N = 128 * (1 + i); d[i].K = 512; d[i].M = 300; d[i].ldx = 512; d[i].ldy = d[i].N; d[i].bits = 2 + i % 3;
            d[i].x_dtype = AQ_BF16;
        }
        const size_t bytes = aq_qgemm_batch_plan_size(count);
        void* plan = std::malloc(bytes);
        for (int flags : {AQ_GEMM_EXACT, AQ_GEMM_FAST}) {
            CHECK(aq_qgemm_batch_plan(d.data(), count, 32, flags, plan, bytes) == AQ_OK);
            CHECK(aq_qgemm_batch_workspace_size(plan) > 0);
        }
        CHECK(aq2_qgemm_batch_plan(d.data(), count, 32, AQ_GEMM_EXACT, plan, bytes) == AQ_OK);
        CHECK(aq2_qgemm_batch_plan(d.data(), count, 32, AQ_GEMM_FAST, plan, bytes) == AQ_OK);
        CHECK(aq_qgemm_batch_plan(d.data(), count, 32, 7, plan, bytes) == AQ_EINVAL);
        CHECK(aq_qgemm_batch_plan(d.data(), count, 32, AQ_GEMM_EXACT, plan, bytes - 1) == AQ_ESIZE);
        CHECK(aq_qgemm_batch(plan, nullptr, nullptr, 0, nullptr) == AQ_ENULL);
        std::memset(plan, 0, bytes);
        CHECK(aq_qgemm_batch_workspace_size(plan) == 0);
        std::free(plan);
    }

    // the layer step's plan
    {
        aq_block_shape shape = {256, 4, 2, 64, 512, AQ_ACT_SILU, 1e-5f};
        const int layers = 3;
        std::vector<aq_block_desc> blocks(layers);
        for (int l = 0; l < layers; ++l) {
            for (int j = 0; j < 7; ++j) { blocks[l].w[j] = dev(10 * l + j); blocks[l].bits[j] = 2 + (l + j) % 3; }
            blocks[l].norm_attn = (const float*)dev(500 + 2 * l);
            blocks[l].norm_mlp = (const float*)dev(501 + 2 * l);
        }
        const size_t pb = aq_decode_plan_size(layers), wb = aq_decode_workspace_size(&shape);
        CHECK(pb > 0 && wb > 0);
        void* plan = std::malloc(pb);
        CHECK(aq_decode_plan(&shape, blocks.data(), layers, 32, (float*)dev(900), (float*)dev(901), dev(902), wb, plan, pb) == AQ_OK);
        CHECK(aq_decode_plan(&shape, blocks.data(), layers, 32, (float*)dev(900), (float*)dev(901), dev(902), wb, plan, pb - 1) == AQ_ESIZE);
        CHECK(aq_decode_plan(&shape, blocks.data(), layers, 32, (float*)dev(900), (float*)dev(901), dev(902), wb - 1, plan, pb) == AQ_ESIZE);
        std::memset(plan, 0, pb);
        CHECK(aq_decode_step(plan, nullptr) != AQ_OK);
        std::free(plan);
    }

    // greedy bit allocation
    {
        const int L = 4, J = 7;
        std::vector<double> S(L * J);
        std::vector<int64_t> sizes(L * J);
        std::vector<int> bits(L * J);
        for (int i = 0; i < L * J; ++i) { S[i] = 1.0 + (i * 37 % 11) * 0.3; sizes[i] = 1000 + 4096 * (i % 3); }
        const int choices[3] = {2, 3, 4};
        CHECK(aq_allocate_bits(S.data(), sizes.data(), L, J, choices, 3, 2.5, bits.data()) == AQ_OK);
        for (int b : bits) CHECK(b >= 2 && b <= 4);
        CHECK(aq_allocate_bits(S.data(), sizes.data(), L, J, choices, 3, 1.5, bits.data()) == AQ_EINVAL);
        CHECK(aq_allocate_bits(S.data(), sizes.data(), L, J, choices, 3, 99.0, bits.data()) == AQ_OK);
        for (int b : bits) CHECK(b == 4);
    }

    // codebook variant: table analysis for every form, list plans with exact-size buffers
    {
        const float e2m1[16] = {0.f, .5f, 1.f, 1.5f, 2.f, 3.f, 4.f, 6.f, -0.f, -.5f, -1.f, -1.5f, -2.f, -3.f, -4.f, -6.f};
        const float sym3[8] = {-2.1f, -1.3f, -.7f, -.2f, .2f, .7f, 1.3f, 2.1f};
        const float gen2[4] = {-1.f, .1f, .2f, 5.f};
        int form = -1;
        float coef[16];
        CHECK(aqc_table_info(e2m1, 4, &form, coef) == AQ_OK && form == AQC_FORM_NATIVE);
        CHECK(aqc_table_info(sym3, 3, &form, coef) == AQ_OK && form == AQC_FORM_SIGNED);
        CHECK(aqc_table_info(gen2, 2, &form, coef) == AQ_OK && form == AQC_FORM_PLANES);
        CHECK(aqc_table_info(gen2, 2, nullptr, nullptr) == AQ_OK);
        std::vector<aqc_gemv_desc> d(5);
        const float* tabs[5] = {e2m1, sym3, gen2, e2m1, sym3};
        const int bits[5] = {4, 3, 2, 4, 3};
        for (int i = 0; i < 5; ++i) {
            d[i].product.packed = dev(3 * i); d[i].product.x = dev(3 * i + 1); d[i].product.y = (float*)dev(3 * i + 2);
            d[i].product.N = 1 + 300 * i; d[i].product.K = 32 * (1 + 100 * i); d[i].product.bits = bits[i];
            d[i].product.x_dtype = AQ_F16;
            d[i].levels = tabs[i];
        }
        const size_t bytes = aqc_qgemv_batch_plan_size(d.data(), 5, 32);
        CHECK(bytes > 0);
        void* plan = std::malloc(bytes);
        CHECK(aqc_qgemv_batch_plan(d.data(), 5, 32, plan, bytes) == AQ_OK);
        CHECK(aqc_qgemv_batch_plan(d.data(), 5, 32, plan, bytes - 1) == AQ_ESIZE);
        CHECK(aqc_qgemv_batch(plan, nullptr, nullptr) == AQ_ENULL);
        std::free(plan);
        CHECK(aqc_qgemm_workspace_size(300, 4096, 4096, 4) > aq_qgemm_workspace_size(300, 4096, 4096, 4));
        // a list of prefill products over codebook blobs: the base plan image, then one table per task
        std::vector<aqc_gemm_desc> gd(5);
        for (int i = 0; i < 5; ++i) {
            aq_gemm_desc& p = gd[i].product;
            p.packed = dev(3 * i); p.X = dev(3 * i + 1); p.Y = (float*)dev(3 * i + 2);
            p.N = 1 + 300 * i; p.K = 32 * (1 + 100 * i); p.M = 300; p.ldx = p.K + 8; p.ldy = p.N; p.bits = bits[i];
            p.x_dtype = AQ_BF16;
            gd[i].levels = tabs[i];
        }
        const size_t gbytes = aqc_qgemm_batch_plan_size(5);
        CHECK(gbytes == aq_qgemm_batch_plan_size(5) + 5 * 64 && aqc_qgemm_batch_plan_size(0) == 0);
        void* gplan = std::malloc(gbytes);
        CHECK(aqc_qgemm_batch_plan(gd.data(), 5, 32, gplan, gbytes) == AQ_OK);
        CHECK(aq_qgemm_batch_workspace_size(gplan) > 0);
        CHECK(aqc_qgemm_batch_plan(gd.data(), 5, 32, gplan, gbytes - 1) == AQ_ESIZE);
        CHECK(aqc_qgemm_batch_plan(gd.data(), 0, 32, gplan, gbytes) == AQ_EINVAL);
        gd[2].levels = nullptr;
        CHECK(aqc_qgemm_batch_plan(gd.data(), 5, 32, gplan, gbytes) == AQ_ENULL);
        std::free(gplan);
        CHECK(aqc_qgemm(dev(0), 64, 512, 2, 32, gen2, dev(1), 40, 512, AQ_F16, (float*)dev(2), 64, dev(3), 16, nullptr) == AQ_ESIZE);
        CHECK(aqc_qgemv(dev(0), 16, 64, 2, 32, nullptr, dev(1), AQ_F16, (float*)dev(2), nullptr) == AQ_ENULL);
    }

    // argument checks of the launching entry points: every call below must be turned away on the host
    CHECK(aq_qgemv(nullptr, 16, 32, 2, 32, dev(1), AQ_F16, (float*)dev(2), nullptr) == AQ_ENULL);
    CHECK(aq_qgemv(dev(0), 16, 33, 2, 32, dev(1), AQ_F16, (float*)dev(2), nullptr) == AQ_EINVAL);
    CHECK(aq_qgemv(dev(0), 16, 32, 2, 32, dev(1), 9, (float*)dev(2), nullptr) == AQ_EDTYPE);
    CHECK(aq_qgemv((char*)dev(0) + 4, 16, 32, 2, 32, dev(1), AQ_F16, (float*)dev(2), nullptr) == AQ_EALIGN);
    CHECK(aq_qgemm(dev(0), 16, 32, 2, 32, dev(1), 4, 32, AQ_F16, (float*)dev(2), 16, dev(3), 0, nullptr) == AQ_ESIZE);
    CHECK(aq_qgemm_fast(dev(0), 16, 32, 6, 32, dev(1), 4, 32, AQ_F16, (float*)dev(2), 16, dev(3), 1 << 20, nullptr) == AQ_EINVAL);
    CHECK(aq_qgemm_noalloc(dev(0), 16, 32, 2, 32, dev(1), 4, 16, AQ_F16, (float*)dev(2), 16, nullptr) == AQ_EINVAL);
    CHECK(aq_pack_weights(nullptr, nullptr, 16, 32, 2, 32, dev(0), 1 << 20, nullptr) == AQ_ENULL);
    CHECK(aq_optimize_scales(nullptr, nullptr, 16, 32, 2, 32, 4, nullptr, nullptr, nullptr) == AQ_ENULL);
    std::puts("ok");
    return 0;
}
