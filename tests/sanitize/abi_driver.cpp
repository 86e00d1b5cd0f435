// Host side of the C ABI under AddressSanitizer + UndefinedBehaviorSanitizer (host code only,
// no GPU needed): the AIFS index builder, the static scale, the tuning hook, and the argument
// validation of every device entry point, which must reject bad calls before anything is
// launched.  Host arrays handed to the library (spans, split indices and scales, linear
// descriptors) are exactly sized heap blocks, so a read past their end aborts the run.  Device
// pointers are fake non-NULL addresses that validation never dereferences.
// Built from the library's sources by tests/test_sanitizers.py.
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <vector>

#include "mquant.h"

#define CHECK(c) do { if (!(c)) { fprintf(stderr, "check failed: %s (line %d)\n", #c, __LINE__); exit(1); } } while (0)

int main()
{
    void *P = reinterpret_cast<void *>(0x1000), *Q = reinterpret_cast<void *>(0x2000);
    const int8_t *Pi8 = static_cast<const int8_t *>(P);
    const uint8_t *Pu8 = static_cast<const uint8_t *>(P);
    CHECK(mquant_version() >= 200);
    CHECK(mquant_build_id() != nullptr);
    for (int s = -7; s <= 0; ++s) CHECK(mquant_status_string(s) != nullptr);

    // ---- AIFS index vector: exact-size outputs, several layouts
    {
        struct Case { int32_t T; std::vector<mquant_span_t> spans; int32_t V; };
        std::vector<Case> cases = {{0, {}, 0}, {7, {{2, 3}}, 3}, {9, {{0, 9}}, 9}, {23, {{2, 3}, {9, 4}, {20, 3}}, 10},
                                   {16384, {{800, 3072}, {4704, 3072}, {8592, 3072}, {12488, 3072}}, 12288}};
        for (auto &c : cases) {
            int32_t *perm = static_cast<int32_t *>(malloc(sizeof(int32_t) * (c.T ? c.T : 1)));
            int32_t *inv = static_cast<int32_t *>(malloc(sizeof(int32_t) * (c.T ? c.T : 1)));
            mquant_span_t *sp = static_cast<mquant_span_t *>(malloc(sizeof(mquant_span_t) * (c.spans.size() ? c.spans.size() : 1)));
            for (size_t i = 0; i < c.spans.size(); ++i) sp[i] = c.spans[i];
            int32_t nv = -1;
            CHECK(mquant_aifs_build_perm(c.T, c.spans.empty() ? nullptr : sp, static_cast<int32_t>(c.spans.size()), perm, inv, &nv) == MQUANT_OK);
            CHECK(nv == c.V);
            for (int32_t i = 0; i < c.T; ++i) CHECK(inv[perm[i]] == i);
            CHECK(mquant_aifs_build_perm(c.T, c.spans.empty() ? nullptr : sp, static_cast<int32_t>(c.spans.size()), nullptr, nullptr, &nv) == MQUANT_OK);
            free(perm); free(inv); free(sp);
        }
        mquant_span_t bad[2] = {{2, 5}, {3, 1}};
        int32_t nv = 0;
        CHECK(mquant_aifs_build_perm(8, bad, 2, nullptr, nullptr, &nv) == MQUANT_ERR_BAD_SHAPE);
        CHECK(mquant_aifs_build_perm(4, bad, 1, nullptr, nullptr, &nv) == MQUANT_ERR_BAD_SHAPE);
        CHECK(mquant_aifs_build_perm(4, nullptr, 0, nullptr, nullptr, nullptr) == MQUANT_ERR_NULL);
    }
    // ---- Eq. (2) scale, tuning hook
    {
        float s = 0.0f;
        CHECK(mquant_static_scale_from_absmax(254.0f * 4.0f, 16, 8, &s) == MQUANT_OK && s == 2.0f);
        CHECK(mquant_static_scale_from_absmax(7.0f, 1, 4, &s) == MQUANT_OK && s == 1.0f);
        CHECK(mquant_static_scale_from_absmax(1.0f, 96, 8, &s) == MQUANT_ERR_UNSUPPORTED);
        CHECK(mquant_static_scale_from_absmax(-1.0f, 16, 8, &s) == MQUANT_ERR_BAD_SHAPE);
        CHECK(mquant_static_scale_from_absmax(1.0f, 16, 8, nullptr) == MQUANT_ERR_NULL);
        CHECK(mquant_tune_set(99, 0) == MQUANT_ERR_BAD_SHAPE);
        CHECK(mquant_tune_set(MQUANT_TUNE_GEMM_TILE, 5) == MQUANT_ERR_BAD_SHAPE);
        CHECK(mquant_tune_set(MQUANT_TUNE_GEMM_TILE, 2) == MQUANT_OK && mquant_tune_set(MQUANT_TUNE_GEMM_TILE, -1) == MQUANT_OK);
        CHECK(mquant_tune_set(MQUANT_TUNE_GEMV_VARIANT, 4) == MQUANT_ERR_BAD_SHAPE);
    }
    // ---- device entry points: rejected on the host, nothing launched
    CHECK(mquant_aifs_permute(nullptr, 64, Q, 64, static_cast<const int32_t *>(P), 4, 64, nullptr) == MQUANT_ERR_NULL);
    CHECK(mquant_aifs_permute(P, 64, P, 64, static_cast<const int32_t *>(P), 4, 64, nullptr) == MQUANT_ERR_BAD_SHAPE);
    CHECK(mquant_aifs_permute(P, 64, Q, 64, static_cast<const int32_t *>(P), 0, 64, nullptr) == MQUANT_OK);
    CHECK(mquant_aifs_remap_mask(nullptr, static_cast<uint8_t *>(P), static_cast<const int32_t *>(P), 8, nullptr) == MQUANT_ERR_NULL);
    CHECK(mquant_hadamard_quant_act(P, 512, nullptr, static_cast<int8_t *>(Q), 4, 512, 5, 1.0f, 1.0f, 512, nullptr) == MQUANT_ERR_BAD_SHAPE);
    CHECK(mquant_hadamard_quant_act(P, 512, nullptr, static_cast<int8_t *>(Q), 4, 512, 2, 1.0f, 1.0f, 96, nullptr) == MQUANT_ERR_UNSUPPORTED);
    CHECK(mquant_hadamard_quant_act_bits(P, 512, nullptr, static_cast<int8_t *>(Q), 4, 512, 2, 1.0f, 1.0f, 512, 9, nullptr) == MQUANT_ERR_UNSUPPORTED);
    CHECK(mquant_hadamard_absmax(P, 512, 4, 512, 512, nullptr, nullptr) == MQUANT_ERR_NULL);
    CHECK(mquant_hadamard_dynquant_act(P, 65536, nullptr, static_cast<int8_t *>(Q), static_cast<float *>(Q), 4, 65536, 512, nullptr) == MQUANT_ERR_UNSUPPORTED);
    CHECK(mquant_w4_prepacked_bytes(33, 64) == 2 * 1024);
    CHECK(mquant_w4_prepacked_bytes(32, 131072) == MQUANT_ERR_UNSUPPORTED);
    CHECK(mquant_w4_prepack(nullptr, static_cast<uint8_t *>(P), 32, 64, nullptr) == MQUANT_ERR_NULL);
    CHECK(mquant_w4a8_workspace_bytes(300, 520, 8192) > 0);
    CHECK(mquant_w4a8_workspace_bytes(16, 512, 100) == MQUANT_ERR_UNSUPPORTED);
    CHECK(mquant_w4a8_gemm(Pi8, Pu8, P, Q, 256, nullptr, 4, 512, 512, 0, 1.0f, 1.0f, nullptr, 0, nullptr) == MQUANT_ERR_BAD_SHAPE);
    CHECK(mquant_w4a8_gemm(Pi8, Pu8, P, Q, 520, nullptr, 300, 520, 8192, 0, 1.0f, 1.0f, nullptr, 0, nullptr) == MQUANT_ERR_WORKSPACE);
    CHECK(mquant_w4a8_gemm(nullptr, nullptr, nullptr, nullptr, 0, nullptr, 0, 512, 512, 0, 1.0f, 1.0f, nullptr, 0, nullptr) == MQUANT_OK);
    CHECK(mquant_w4a8_gemm_rowscale(Pi8, Pu8, P, nullptr, Q, 512, nullptr, 4, 512, 512, nullptr, 0, nullptr) == MQUANT_ERR_NULL);
    {
        // split-channel arrays: exact-size host blocks, every entry is read by the validation
        for (int n_split : {1, 2, 64}) {
            int32_t *idx = static_cast<int32_t *>(malloc(sizeof(int32_t) * n_split));
            float *sc = static_cast<float *>(malloc(sizeof(float) * n_split));
            for (int j = 0; j < n_split; ++j) { idx[j] = j * 3; sc[j] = 0.1f; }
            idx[n_split - 1] = 5000;                                   // out of range: found at the last entry
            CHECK(mquant_w4a8_gemm_rms(Pi8, Pu8, P, Q, 512, nullptr, 4, 512, 1024, 0, 1.0f, 1.0f, idx, Pi8, sc, n_split, nullptr, 0, nullptr) == MQUANT_ERR_BAD_SHAPE);
            free(idx); free(sc);
        }
        CHECK(mquant_w4a8_gemm_rms(Pi8, Pu8, P, Q, 512, nullptr, 4, 512, 1024, 0, 1.0f, 1.0f, nullptr, Pi8, nullptr, 65, nullptr, 0, nullptr) == MQUANT_ERR_BAD_SHAPE);
    }
    {
        const int64_t need = mquant_w4a8_linear_prefill_workspace_bytes(64, 512, 512);
        CHECK(need >= 64 * 512);
        CHECK(mquant_w4a8_linear_prefill(P, 512, nullptr, Pu8, P, Q, 512, 64, 512, 512, 48, 1.0f, 1.0f, 512, nullptr, 0, nullptr) == MQUANT_ERR_WORKSPACE);
        CHECK(mquant_w4a8_linear_prefill(P, 512, nullptr, Pu8, P, Q, 512, 64, 512, 512, 48, 1.0f, 1.0f, 96, P, need, nullptr) == MQUANT_ERR_UNSUPPORTED);
        CHECK(mquant_w4a8_linear_prefill_static(P, 29568, nullptr, Pu8, P, Q, 8192, 16384, 8192, 29568, 12288, 1.0f, 1.0f, 128, nullptr) == MQUANT_ERR_WORKSPACE);
        CHECK(mquant_w4a8_linear_decode(P, 512, Pu8, P, Q, 512, 5, 512, 512, 0, 1.0f, 1.0f, 512, nullptr) == MQUANT_ERR_UNSUPPORTED);
        CHECK(mquant_w4a8_linear_decode(P, 512, Pu8, P, Q, 512, 1, 512, 512, 2, 1.0f, 1.0f, 512, nullptr) == MQUANT_ERR_BAD_SHAPE);
    }
    {
        // grouped decode: the descriptor array is an exact-size host block
        for (int n : {1, 3, 4}) {
            mquant_linear_t *lin = static_cast<mquant_linear_t *>(malloc(sizeof(mquant_linear_t) * n));
            for (int i = 0; i < n; ++i) lin[i] = {Pu8, P, Q, 64, 64};
            lin[n - 1].ldy = 32;                                      // found at the last descriptor
            CHECK(mquant_w4a8_gemv_grouped(Pi8, 1, 128, 0, 1.0f, 1.0f, lin, n, nullptr) == MQUANT_ERR_BAD_SHAPE);
            lin[n - 1].ldy = 64;
            lin[n - 1].y_dev = nullptr;
            CHECK(mquant_w4a8_gemv_grouped(Pi8, 1, 128, 0, 1.0f, 1.0f, lin, n, nullptr) == MQUANT_ERR_NULL);
            CHECK(mquant_w4a8_gemv_grouped(Pi8, 0, 128, 0, 1.0f, 1.0f, lin, n, nullptr) == MQUANT_OK);
            CHECK(mquant_w4a8_linear_decode_grouped(P, 512, 1, 512, 0, 1.0f, 1.0f, 512, lin, n, nullptr) == MQUANT_ERR_NULL);
            lin[n - 1].y_dev = Q;
            lin[n - 1].ldy = 32;
            CHECK(mquant_w4a8_linear_decode_grouped(P, 512, 1, 512, 0, 1.0f, 1.0f, 512, lin, n, nullptr) == MQUANT_ERR_BAD_SHAPE);
            lin[n - 1].ldy = 64;
            CHECK(mquant_w4a8_linear_decode_grouped(P, 512, 0, 512, 0, 1.0f, 1.0f, 512, lin, n, nullptr) == MQUANT_OK);
            CHECK(mquant_w4a8_linear_decode_grouped(P, 512, 5, 512, 0, 1.0f, 1.0f, 512, lin, n, nullptr) == MQUANT_ERR_UNSUPPORTED);
            free(lin);
        }
        CHECK(mquant_w4a8_gemv_grouped(Pi8, 1, 128, 0, 1.0f, 1.0f, nullptr, 5, nullptr) == MQUANT_ERR_UNSUPPORTED);
    }
    CHECK(mquant_rope_apply(P, 1024, static_cast<const int32_t *>(P), 4, 8, 96, 10000.0, nullptr) == MQUANT_ERR_UNSUPPORTED);
    CHECK(mquant_aifs_attention_workspace_bytes(64, 4, 128) >= 64 * 4 * 128 * 2);
    CHECK(mquant_aifs_attention(P, 3584, P, 512, P, 512, Q, 3584, static_cast<const int32_t *>(P), 64, 28, 5, 128, P, 1 << 20, nullptr) == MQUANT_ERR_BAD_SHAPE);
    CHECK(mquant_w4g128_prepacked_bytes(64, 192) == MQUANT_ERR_UNSUPPORTED);
    CHECK(mquant_w4g128_prepack(nullptr, P, static_cast<uint8_t *>(P), 32, 128, nullptr) == MQUANT_ERR_NULL);
    CHECK(mquant_w4g128_gemm(P, 128, Pu8, Q, 64, 4, 64, 256, nullptr) == MQUANT_ERR_BAD_SHAPE);
    printf("abi host sanitizer run ok\n");
    return 0;
}
