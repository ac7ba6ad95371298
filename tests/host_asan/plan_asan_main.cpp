// Host-side checks of the shard plan, the plan generators and the cost model, meant to be built with
// -fsanitize=address,undefined (see tests/test_host_sanitizers.py).  Every result is compared with a
// plain re-computation; the sanitizers watch the pointer arithmetic in between.
#include <algorithm>
#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <vector>
#include "../../include/cascade.h"

static int failures = 0;
#define CHECK(c)                                                        \
    do {                                                                \
        if (!(c)) { printf("FAIL %s:%d %s\n", __FILE__, __LINE__, #c); ++failures; } \
    } while (0)

static uint32_t rng_state = 12345u;
static uint32_t rnd() { rng_state = rng_state * 1664525u + 1013904223u; return rng_state >> 8; }

static void check_plan(int batch, int N, int S, const std::vector<int32_t> &a, const int32_t *pos) {
    cascade_plan *p = nullptr;
    CHECK(cascade_plan_create(&p, batch, N, S, a.data(), pos, CASCADE_MASK_CAUSAL) == CASCADE_OK);
    if (!p) return;
    const int32_t *perm, *inv, *off, *perm_d, *inv_d, *off_d;
    CHECK(cascade_plan_maps_host(p, &perm, &inv, &off) == CASCADE_OK);
    CHECK(cascade_plan_maps(p, &perm_d, &inv_d, &off_d) == CASCADE_OK);
    int r = 0;
    for (int j = 0; j < S; ++j) {                    // shards in id order, ascending token index inside
        CHECK(off[j] == r);
        for (int t = 0; t < N; ++t)
            if (a[t] == j) { CHECK(perm[r] == t); CHECK(inv[t] == r); CHECK(perm_d[r] == t); CHECK(inv_d[t] == r); ++r; }
    }
    CHECK(off[S] == N && off_d[S] == N && r == N);
    double ta = 0, tb = 0, tt = 0;
    CHECK(cascade_comm_time(p, 0, 0, 0, 2, 64, 12, 12, 1e-3, 1e9, &ta, &tb, &tt) == CASCADE_OK);
    int mx = 0;
    for (int j = 0; j < S; ++j) mx = std::max(mx, off[j + 1] - off[j]);
    CHECK(std::fabs(ta - (1e-3 + (double)S * 2 * 64 * 36 / 1e9 * mx)) < 1e-12);
    CHECK(std::fabs(tt - ta - tb) < 1e-15);
    cascade_plan_destroy(p);
}

int main() {
    // plans: equal, ragged, empty shards, more shards than tokens, one token, custom positions
    for (int trial = 0; trial < 40; ++trial) {
        const int N = 1 + rnd() % 700, S = 1 + rnd() % 40, batch = 1 + rnd() % 3;
        std::vector<int32_t> a(N), pos(N);
        for (int t = 0; t < N; ++t) { a[t] = (trial % 3 == 0) ? t % S : (int32_t)(rnd() % S); pos[t] = (int32_t)(rnd() % 100000) - 50; }
        check_plan(batch, N, S, a, trial % 2 ? pos.data() : nullptr);
    }
    {   // two partitions
        const int N = 333;
        std::vector<int32_t> a(N), kv(N);
        int32_t alpha = 0;
        CHECK(cascade_cdelta_assignment(N, 4, 20, a.data(), &alpha) == CASCADE_OK && alpha == 5);
        CHECK(cascade_m_split(N, alpha, a.data(), 3, kv.data()) == CASCADE_OK);
        std::vector<int> seen(alpha, 0);
        for (int t = 0; t < N; ++t) { CHECK(a[t] == (t % 20) / 4); CHECK(kv[t] == 3 * a[t] + seen[a[t]]++ % 3); }
        cascade_plan *p = nullptr;
        CHECK(cascade_plan_create_rs(&p, 2, N, alpha, a.data(), 3 * alpha, kv.data(), nullptr, CASCADE_MASK_NONE) == CASCADE_OK);
        int32_t nkv = 0;
        const int32_t *kperm, *koff, *k2r, *perm, *inv, *off;
        CHECK(cascade_plan_kv_maps_host(p, &nkv, &kperm, &koff, &k2r) == CASCADE_OK && nkv == 3 * alpha && k2r);
        CHECK(cascade_plan_maps_host(p, &perm, &inv, &off) == CASCADE_OK);
        for (int r = 0; r < N; ++r) CHECK(perm[k2r[r]] == kperm[r]);
        cascade_plan_destroy(p);
    }
    {   // error paths leave nothing behind
        std::vector<int32_t> a(16, 0);
        cascade_plan *p = (cascade_plan *)0x1;
        a[5] = 4;
        CHECK(cascade_plan_create(&p, 1, 16, 4, a.data(), nullptr, CASCADE_MASK_CAUSAL) == CASCADE_EASSIGN && p == nullptr);
        a[5] = -1;
        CHECK(cascade_plan_create(&p, 1, 16, 4, a.data(), nullptr, CASCADE_MASK_CAUSAL) == CASCADE_EASSIGN);
        a[5] = 0;
        CHECK(cascade_plan_create(&p, 0, 16, 4, a.data(), nullptr, CASCADE_MASK_CAUSAL) == CASCADE_EINVAL);
        CHECK(cascade_plan_create(&p, 1, 16, 4, nullptr, nullptr, CASCADE_MASK_CAUSAL) == CASCADE_EINVAL);
        CHECK(cascade_plan_create(&p, 1, 16, 4, a.data(), nullptr, 9) == CASCADE_EINVAL);
        CHECK(cascade_plan_create_rs(&p, 1, 16, 4, a.data(), 0, a.data(), nullptr, CASCADE_MASK_CAUSAL) == CASCADE_EINVAL);
        a[3] = 7;                                    // bad kv assignment after a good row assignment
        std::vector<int32_t> rows(16, 1);
        CHECK(cascade_plan_create_rs(&p, 1, 16, 4, rows.data(), 4, a.data(), nullptr, CASCADE_MASK_CAUSAL) == CASCADE_EASSIGN);
        CHECK(cascade_m_split(16, 2, a.data(), 2, rows.data()) == CASCADE_EASSIGN);
        CHECK(cascade_cdelta_assignment(16, 0, 4, rows.data(), nullptr) == CASCADE_EINVAL);
        CHECK(cascade_comm_time(nullptr, 4, 8, 8, 2, 64, 12, 12, -1.0, 1e9, nullptr, nullptr, nullptr) == CASCADE_EINVAL);
        CHECK(cascade_comm_time(nullptr, 4, 8, 8, 2, 64, 12, 12, 0.0, 0.0, nullptr, nullptr, nullptr) == CASCADE_EINVAL);
        cascade_plan_destroy(nullptr);
    }
    {   // cost model: Equation 1 halves and the rounds bound
        int64_t sa = 0, sb = 0, rd = 0;
        CHECK(cascade_comm_cost(4, 8, 0, 2, 64, 12, 12, 128, &sa, &sb, &rd) == CASCADE_OK);
        CHECK(sa == 8ll * 2 * 64 * 36 * 128 && sb == 8ll * 2 * 66 * 12 * 128 && rd == 2ll * 4 * 64);
        CHECK(cascade_comm_cost(4, 8, 1, 2, 64, 12, 12, 128, nullptr, nullptr, &rd) == CASCADE_OK && rd == 128);
    }
    printf(failures ? "FAILED %d\n" : "HOST_SANITIZER_OK\n", failures);
    return failures ? 1 : 0;
}
