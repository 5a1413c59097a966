// Calls the host-side code of libmixllm_hip - argument validation, size accounting, the order of
// the concatenated rows, the launch plans of every path - from a build whose host objects carry
// -fsanitize=address,undefined.  No GPU is touched: every call either is pure host arithmetic or
// is refused by the validation before anything is launched.  Built and run by
// tests/test_sanitizers.py.
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <vector>

#include "mixllm.h"

#define CHECK(c)                                                                         \
    do {                                                                                 \
        if (!(c)) {                                                                      \
            std::fprintf(stderr, "host_driver: check failed at line %d: %s\n", __LINE__, #c); \
            return 1;                                                                    \
        }                                                                                \
    } while (0)

int main()
{
    const int Ks[] = {128, 384, 4096, 8192, 14336, 28672, 131072};
    const int Ns[] = {1, 16, 17, 100, 4096, 6144, 28672, 57344};
    const int Ms[] = {0, 1, 4, 16, 17, 32, 33, 64, 65, 128, 256, 512, 2048, 8192};
    long plans = 0;
    for (int K : Ks)
        for (int N : Ns)
            for (int share = 0; share <= 2; ++share)
                for (int M : Ms)
                    for (int gran = 0; gran < 3; ++gran) {
                        mixllm_desc d{M, K, N, share == 0 ? 0 : share == 1 ? N / 10 : N, MIXLLM_GROUP,
                                      gran == 1 ? MIXLLM_GROUP : K, gran >= 1 ? MIXLLM_GROUP : K};
                        mixllm_sizes s;
                        CHECK(mixllm_query_sizes(&d, &s) == MIXLLM_OK);
                        CHECK(s.workspace_bytes >= s.xq_bytes + s.xscale_bytes + s.linear_workspace_bytes);
                        if (M == 0) continue;
                        for (int path : {MIXLLM_PATH_DECODE_SPLIT, MIXLLM_PATH_MID, MIXLLM_PATH_PREFILL}) {
                            int32_t plan[16];
                            const int rc = mixllm_debug_work_split(&d, path, plan);
                            CHECK(rc == MIXLLM_OK || rc == MIXLLM_EUNSUPPORTED);
                            plans += rc == MIXLLM_OK;
                        }
                        // every data pointer null: refused before anything is launched, whatever the path
                        for (int path = MIXLLM_PATH_AUTO; path <= MIXLLM_PATH_PREFILL_128 + 1; ++path)
                            CHECK(mixllm_mixed_linear_path(&d, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr,
                                                           nullptr, nullptr, nullptr, 0, path, nullptr) < 0);
                        CHECK(mixllm_mixed_linear_fp16(&d, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr,
                                                       nullptr, 0, nullptr) == MIXLLM_EINVAL);
                        CHECK(mixllm_mixed_linear_fp16_static(&d, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr,
                                                              nullptr, nullptr) < 0);
                    }
    // the order of the concatenated rows, and what it refuses
    for (int N : {1, 2, 17, 1000}) {
        std::vector<int32_t> sal, perm((size_t)N);
        for (int c = N - 1; c >= 0; c -= 3) sal.push_back(c);
        CHECK(mixllm_build_feature_perm(N, (int32_t)sal.size(), sal.data(), perm.data()) == MIXLLM_OK);
        std::vector<char> seen((size_t)N, 0);
        for (int32_t c : perm) {
            CHECK(c >= 0 && c < N && !seen[(size_t)c]);
            seen[(size_t)c] = 1;
        }
        sal.push_back(sal[0]);
        CHECK(mixllm_build_feature_perm(N, (int32_t)sal.size(), sal.data(), perm.data()) == MIXLLM_EINVAL);
        sal.back() = N;
        CHECK(mixllm_build_feature_perm(N, (int32_t)sal.size(), sal.data(), perm.data()) == MIXLLM_EINVAL);
    }
    // the selection's host-side checks (layer list, T, workspace size)
    {
        const int L = 300;
        std::vector<int64_t> off((size_t)L + 1);
        for (int l = 0; l <= L; ++l) off[(size_t)l] = 10 * l;
        alignas(16) static unsigned char fake[64];
        CHECK(mixllm_select_salient_workspace(L) > 0);
        CHECK(mixllm_select_salient((const float *)fake, off.data(), L, 7, (int32_t *)fake, (int32_t *)fake, fake, 8, nullptr) ==
              MIXLLM_EWORKSPACE);
        CHECK(mixllm_select_salient((const float *)fake, off.data(), L, 10 * L + 1, (int32_t *)fake, (int32_t *)fake, fake,
                                    mixllm_select_salient_workspace(L), nullptr) == MIXLLM_EINVAL);
        off[5] = 1;
        CHECK(mixllm_select_salient((const float *)fake, off.data(), L, 7, (int32_t *)fake, (int32_t *)fake, fake,
                                    mixllm_select_salient_workspace(L), nullptr) == MIXLLM_EINVAL);
    }
    mixllm_desc bad{1, 4000, 64, 0, MIXLLM_GROUP, 4000, 4000};
    mixllm_sizes s;
    CHECK(mixllm_query_sizes(&bad, &s) == MIXLLM_EUNSUPPORTED);
    CHECK(mixllm_query_sizes(nullptr, &s) == MIXLLM_EINVAL);
    CHECK(mixllm_status_string(MIXLLM_EWORKSPACE) != nullptr && mixllm_abi_version() >= 2);
    std::printf("host_driver: ok (%ld launch plans)\n", plans);
    return 0;
}
