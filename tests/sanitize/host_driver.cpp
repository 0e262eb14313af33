// Host-side checks of libconfu_verify's argument validation, launch planning and mask builder, meant to be
// built with AddressSanitizer and UndefinedBehaviorSanitizer (host code only; nothing here touches a GPU).
// Walks grids of descriptors through every host-only entry point and checks that return codes and sizes are sane.
#include <cstdint>
#include <cstdio>
#include <cstring>
#include <vector>

#include "confu_verify.h"

static int fails = 0;
#define CHECK(c) do { if (!(c)) { std::printf("FAILED %s:%d %s\n", __FILE__, __LINE__, #c); ++fails; } } while (0)

static tv_attn_desc attn(int dtype, int B, int M, int Hq, int Hkv, int D, int s, int P, int splits, int rb,
                         int64_t sum) {
    tv_attn_desc d;
    std::memset(&d, 0, sizeof d);
    d.struct_size = sizeof d; d.dtype = dtype; d.B = B; d.M = M; d.Hq = Hq; d.Hkv = Hkv; d.D = D;
    d.soft_len = s; d.max_prefix_len = P; d.softmax_scale = 0.088f; d.num_splits = splits; d.wg_row_blocks = rb;
    d.sum_prefix_len = sum;
    return d;
}

int main() {
    // ---- attention planner and workspace sizes
    const int Bs[] = {1, 2, 3, 8, 17, 64, 200}, Ps[] = {0, 1, 31, 100, 1024, 4096, 16384, 65536, 300000};
    const int Ms[] = {1, 9, 64, 120, 128}, splits[] = {0, 1, 3, 8, 64, 1000}, rbs[] = {0, 1, 2, 4};
    long planned = 0;
    for (int B : Bs) for (int P : Ps) for (int M : Ms) for (int sp : splits) for (int rb : rbs) {
        tv_attn_desc d = attn(TV_DTYPE_BF16, B, M, 32, 8, 128, P >= 16 ? 16 : 0, P, sp, rb, 0);
        int32_t wg = -1, n = -1;
        size_t bytes = (size_t)-1;
        const int rc = tv_attention_plan(&d, &wg, &n);
        const int rc2 = tv_attention_workspace_bytes(&d, &bytes);
        CHECK(rc == rc2);
        if (rc == TV_OK) {
            ++planned;
            CHECK(wg == 1 || wg == 2 || wg == 4);
            CHECK(n >= 1 && n <= 64);
            CHECK(rb == 0 || wg == rb);
            CHECK((n == 1) == (bytes == 0));
            CHECK(bytes % 256 == 0);
        } else {
            CHECK(rc == TV_ERR_INVALID_ARG || rc == TV_ERR_UNSUPPORTED);
        }
        if (B > 1 && P > 0) {      // with the caller's length hint
            d.sum_prefix_len = (int64_t)B * P / 2;
            CHECK(tv_attention_plan(&d, &wg, &n) == rc);
        }
    }
    CHECK(planned > 1000);
    {   // fp32 path, other head shapes, malformed descriptors
        tv_attn_desc d = attn(TV_DTYPE_F32, 1, 9, 8, 2, 64, 0, 128, 0, 0, 0);
        size_t bytes = 1;
        CHECK(tv_attention_workspace_bytes(&d, &bytes) == TV_OK && bytes == 0);
        d.D = 96;
        CHECK(tv_attention_workspace_bytes(&d, &bytes) == TV_ERR_UNSUPPORTED);
        d = attn(TV_DTYPE_BF16, 1, 64, 32, 8, 128, 0, 4096, 0, 0, 0);
        d.struct_size = 8;
        CHECK(tv_attention_workspace_bytes(&d, &bytes) == TV_ERR_INVALID_ARG);
        d = attn(TV_DTYPE_BF16, 1, 129, 32, 8, 128, 0, 4096, 0, 0, 0);
        CHECK(tv_attention_workspace_bytes(&d, &bytes) == TV_ERR_INVALID_ARG);
        d = attn(TV_DTYPE_BF16, 1, 64, 32, 5, 128, 0, 4096, 0, 0, 0);
        CHECK(tv_attention_workspace_bytes(&d, &bytes) == TV_ERR_INVALID_ARG);
        d = attn(TV_DTYPE_BF16, 1, 64, 32, 8, 128, 0, 4096, 0, 3, 0);
        CHECK(tv_attention_workspace_bytes(&d, &bytes) == TV_ERR_INVALID_ARG);
        CHECK(tv_attention_workspace_bytes(nullptr, &bytes) == TV_ERR_INVALID_ARG);
        CHECK(tv_attention_workspace_bytes(&d, nullptr) == TV_ERR_INVALID_ARG);
        // null device pointers are refused before anything is enqueued
        d = attn(TV_DTYPE_BF16, 1, 64, 32, 8, 128, 0, 4096, 0, 0, 0);
        CHECK(tree_verify_attention(&d, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr,
                                    nullptr, nullptr, nullptr, 0, nullptr) == TV_ERR_INVALID_ARG);
    }
    // ---- acceptance workspace sizes
    for (int B : {1, 8, 100}) for (int T : {1, 7, 60, 128}) for (int V : {1, 1000, 32000, 128256, 151936, 1000000})
        for (int rule = TV_RULE_GREEDY; rule <= TV_RULE_SAMPLE_MATCH; ++rule) {
            tv_accept_desc d;
            std::memset(&d, 0, sizeof d);
            d.struct_size = sizeof d; d.B = B; d.T = T; d.V = V; d.C = 4; d.rule = rule;
            d.temperature = rule == TV_RULE_GREEDY ? 0.f : 1.f;
            size_t bytes = 0;
            const int rc = tv_accept_workspace_bytes(&d, &bytes);
            CHECK(rc == TV_OK || rc == TV_ERR_INVALID_ARG || rc == TV_ERR_UNSUPPORTED);
            if (rc == TV_OK) CHECK(bytes > 0 && bytes % 256 == 0 && bytes < ((size_t)1 << 34));
            d.temperature = -1.f;
            if (rule != TV_RULE_GREEDY) CHECK(tv_accept_workspace_bytes(&d, &bytes) == TV_ERR_INVALID_ARG);
        }
    // ---- mask builder: random trees against a plain ancestor walk, and malformed trees
    uint32_t rng = 12345u;
    auto next = [&]() { rng = rng * 1664525u + 1013904223u; return rng >> 8; };
    for (int trial = 0; trial < 200; ++trial) {
        const int M = 1 + (int)(next() % TV_MAX_ROWS);
        std::vector<int32_t> parent(M);
        std::vector<uint8_t> kind(M, TV_KIND_NODE);
        parent[0] = -1;
        for (int i = 1; i < M; ++i) parent[i] = (int32_t)(next() % (uint32_t)i);
        for (int i = 1; i < M; ++i)       // leaves may be contemplate rows
            if (next() % 4 == 0) {
                bool leaf = true;
                for (int j = i + 1; j < M; ++j) leaf = leaf && parent[j] != i;
                if (leaf) kind[i] = TV_KIND_CONTEMPLATE;
            }
        std::vector<uint64_t> bits(2 * (size_t)M, ~0ull);
        CHECK(tv_build_mask_host(parent.data(), kind.data(), M, bits.data()) == TV_OK);
        for (int i = 0; i < M; ++i) {
            uint64_t w[2] = {0, 0};
            for (int j = i; j >= 0; j = parent[j]) w[j >> 6] |= (uint64_t)1 << (j & 63);
            CHECK(bits[2 * i] == w[0] && bits[2 * i + 1] == w[1]);
        }
        if (M >= 3) {
            std::vector<int32_t> bad = parent;
            bad[M - 1] = M - 1;                                   // its own parent
            CHECK(tv_build_mask_host(bad.data(), kind.data(), M, bits.data()) == -TV_STATUS_BAD_PARENT);
            std::vector<uint8_t> bk = kind;
            bk[1] = 7;
            CHECK(tv_build_mask_host(parent.data(), bk.data(), M, bits.data()) < 0);
        }
    }
    CHECK(tv_build_mask_host(nullptr, nullptr, 4, nullptr) == TV_ERR_INVALID_ARG);
    for (int code = -40; code < 10; ++code) CHECK(tv_error_string(code) != nullptr && tv_error_string(code)[0] != 0);
    CHECK(tv_version() > 0);
    if (fails) std::printf("host driver: %d check(s) failed\n", fails);
    else std::printf("host driver: ok (%ld plans)\n", planned);
    return fails ? 1 : 0;
}
