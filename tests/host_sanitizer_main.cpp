// The library's host half driven directly on random shapes (compiled with ASan/UBSan by test_host_sanitizers.py).
#include <cstdio>
#include <cstdlib>
#include <random>
#include <vector>
#include "etf_internal.h"

#define CK(x) do { int rc_ = (x); if (rc_ != ETF_OK) { printf("FAIL %s -> %d (%s)\n", #x, rc_, ctx.err.c_str()); return 1; } } while (0)

int main()
{
    std::mt19937 rng(7);
    for (int round = 0; round < 24; ++round) {
        etf_ctx ctx;
        const int Ms[] = {1, 2, 3, 4, 8, 16};
        const int M = Ms[rng() % 6];
        const int K = 1 + rng() % 256;
        const int ds = 1 + rng() % 5;
        const int d = M * ds;
        std::vector<float> cb((size_t)M * K * ds);
        for (auto &v : cb) v = (float)(rng() % 1000) / 100.f;
        CK(etf_pq_set_codebooks(&ctx, cb.data(), d, M, K));
        const int64_t N = 1 + rng() % 5000;
        std::vector<uint8_t> codes((size_t)N * M);
        const int spread = 1 + rng() % K;
        for (auto &c : codes) c = (uint8_t)(rng() % spread);
        std::vector<int32_t> ids(N);
        for (int64_t i = 0; i < N; ++i) ids[i] = (int32_t)(rng() % 100000);
        std::vector<int> divs;
        for (int t = 1; t <= M; ++t) if (M % t == 0) divs.push_back(t);
        const int T = divs[rng() % divs.size()];
        std::vector<int32_t> order(M);
        for (int j = 0; j < M; ++j) order[j] = j;
        std::shuffle(order.begin(), order.end(), rng);
        if (round % 3 == 0) CK(etf_index_set_chunk_order(&ctx, order.data()));
        ctx.opt.sample_min = 16 + rng() % 2000;
        CK(etf_index_build(&ctx, codes.data(), N, round % 2 ? ids.data() : nullptr, T, nullptr));
        etf_stats st;
        CK(etf_index_stats(&ctx, &st));
        etf_layout lay;
        CK(etf_index_layout(&ctx, &lay));
        std::vector<char> buf((size_t)etf_index_device_bytes(&ctx));
        CK(etf_index_export(&ctx, buf.data(), (int64_t)buf.size()));
        std::vector<int32_t> sug(M);
        int64_t a = 0, b = 0;
        CK(etf_suggest_chunk_order(&ctx, codes.data(), N, T, nullptr, sug.data(), &a, &b));
        if (b > a) { printf("FAIL suggestion worse\n"); return 1; }
        // unequal trees
        if (M >= 3) {
            std::vector<int32_t> cbeg = {0, 1, M};
            CK(etf_index_build(&ctx, codes.data(), N, nullptr, 2, cbeg.data()));
            CK(etf_index_stats(&ctx, &st));
        }
        // quantiser: train and encode
        const int64_t n = 50 + rng() % 300;
        std::vector<float> x((size_t)n * d);
        for (auto &v : x) v = (float)(rng() % 2000) / 100.f - 10.f;
        const int K2 = 1 + rng() % 16;
        CK(etf_pq_train(&ctx, x.data(), n, d, M, K2, 3, 11));
        std::vector<uint8_t> enc((size_t)n * M);
        CK(etf_pq_encode(&ctx, x.data(), n, enc.data()));
        printf("round %d ok: M=%d K=%d N=%lld T=%d Nd=%lld\n", round, M, K, (long long)N, T, (long long)st.n_distinct);
    }
    printf("host sanitizer run: ok\n");
    return 0;
}
