// Driver for the host-only parts of the library (work scheduler, block pool, placement scheduler), meant to be
// built with -fsanitize=address,undefined by tests/test_host_sanitizers.py.  It feeds seeded random and edge-case
// inputs and checks structural properties; any sanitizer report or failed check ends it with a non-zero status.
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <random>
#include <vector>

#include "../include/distattn.h"
#include "../include/distattn_placement.h"
#include "../paper_2401_02669_amd/csrc/schedule.h"

#define CHECK(cond)                                                              \
    do {                                                                         \
        if (!(cond)) {                                                           \
            std::fprintf(stderr, "check failed: %s (line %d)\n", #cond, __LINE__); \
            std::exit(1);                                                        \
        }                                                                        \
    } while (0)

static da_problem problem(int B, int Hq, int Hkv, int T, int max_blocks, int q_len, int bf16)
{
    da_problem p{};
    p.batch = B; p.num_q_heads = Hq; p.num_kv_heads = Hkv; p.head_dim = 128; p.block_tokens = T;
    p.max_blocks_per_seq = max_blocks; p.num_phys_blocks = B * max_blocks; p.kv_dtype = bf16; p.q_dtype = bf16;
    p.scale = 0.088f; p.kv_token_stride = 128; p.kv_head_stride = 128 * (int64_t)T; p.kv_block_stride = 128 * (int64_t)T * Hkv;
    p.q_len = q_len;
    return p;
}

static void check_schedule(const da_problem &p, const std::vector<int32_t> &lens, const da_tuning &t, int cus)
{
    da::Schedule s;
    const da_status st = da::make_schedule(p, lens.data(), t, cus, s);
    CHECK(st == DA_OK);
    CHECK((int)s.nsplits.size() == p.batch);
    CHECK((int)s.range_start.size() == s.ranges + 1);
    CHECK(s.range_start.front() == 0 && s.range_start.back() == (int)s.entries.size());
    int64_t rows = 0;
    for (int r = 0; r < p.batch; ++r) {
        CHECK(s.nsplits[r] >= 1);
        CHECK(s.row_base[r] == rows);
        rows += (int64_t)s.nsplits[r] * p.num_q_heads * (p.q_len > 1 ? p.q_len : 1);
        // the splits of a request tile its tiles without gap or overlap
        int64_t next = 0;
        for (int j = 0; j < s.nsplits[r]; ++j) {
            const da::SplitEntry &e = s.entries[s.first_entry[r] + j];
            CHECK(e.r == r && e.j == j && e.t0 == next && e.t1 >= e.t0);
            next = e.t1;
        }
        CHECK(next >= s.ntiles[r]);
    }
    CHECK(rows == s.num_partials);
    for (int m = 0; m < s.ranges; ++m) CHECK(s.range_start[m] <= s.range_start[m + 1]);
}

int main()
{
    std::mt19937_64 rng(20240102);
    // ---- work scheduler ----
    for (int it = 0; it < 400; ++it) {
        const int B = 1 + (int)(rng() % (it % 7 == 0 ? 300 : 24));
        const int Hkv = 1 << (rng() % 4);
        const int G = (it % 3 == 0) ? 1 : (1 << (rng() % 4));
        const int T = 16 * (1 + (int)(rng() % 32));
        const int q_len = (it % 5 == 0) ? 1 + (int)(rng() % 8) : 1;
        const int max_len = (it % 11 == 0) ? 300000 : 5000;
        std::vector<int32_t> lens(B);
        for (int &L : lens) L = (rng() % 9 == 0) ? 0 : (int)(rng() % max_len);
        const int max_blocks = (max_len + T - 1) / T + 1;
        const da_problem p = problem(B, Hkv * G, Hkv, T, max_blocks, q_len, 1);
        da_tuning t{};
        t.blocks_per_split = (it % 4 == 0) ? 1 + (int)(rng() % 8) : 0;
        const int cus = (it % 13 == 0) ? 1 + (int)(rng() % 8) : 256;
        check_schedule(p, lens, t, cus);
    }
    {   // every request empty; one token; a length that ends exactly on a block
        check_schedule(problem(3, 8, 8, 64, 4, 1, 1), {0, 0, 0}, da_tuning{}, 256);
        check_schedule(problem(2, 64, 8, 256, 8, 1, 1), {1, 2048}, da_tuning{}, 256);
        da::Schedule s;
        std::vector<int32_t> bad = {5, -1};
        CHECK(da::make_schedule(problem(2, 8, 8, 64, 4, 1, 1), bad.data(), da_tuning{}, 256, s) == DA_ERR_INVALID_ARG);
        bad = {5, 64 * 4 + 1};
        CHECK(da::make_schedule(problem(2, 8, 8, 64, 4, 1, 1), bad.data(), da_tuning{}, 256, s) == DA_ERR_INVALID_ARG);
    }
    // ---- block pool ----
    {
        da_block_pool *pool = nullptr;
        CHECK(da_block_pool_create(64, &pool) == DA_OK);
        const int T = 16, max_blocks = 20;
        std::vector<std::vector<int32_t>> rows(6, std::vector<int32_t>(max_blocks, -1));
        std::vector<int> len(6, 0);
        for (int it = 0; it < 5000; ++it) {
            const int r = (int)(rng() % 6);
            if (rng() % 5 == 0) {
                CHECK(da_block_pool_release(pool, T, rows[r].data(), len[r]) == DA_OK);
                len[r] = 0;
            } else {
                const int add = 1 + (int)(rng() % 40);
                const int want = len[r] + add > T * max_blocks ? T * max_blocks : len[r] + add;
                const da_status st = da_block_pool_grow(pool, T, max_blocks, rows[r].data(), len[r], want);
                CHECK(st == DA_OK || st == DA_ERR_NO_SPACE);
                if (st == DA_OK) len[r] = want;
            }
            int32_t free_now = 0, held = 0;
            CHECK(da_block_pool_free_count(pool, &free_now) == DA_OK);
            for (int x = 0; x < 6; ++x) held += (len[x] + T - 1) / T;
            CHECK(free_now + held == 64);
        }
        CHECK(da_block_pool_grow(pool, T, max_blocks, rows[0].data(), len[0], T * max_blocks + 1) != DA_OK);
        CHECK(da_block_pool_destroy(pool) == DA_OK);
    }
    // ---- placement scheduler ----
    for (int it = 0; it < 300; ++it) {
        const int M = 1 + (int)(rng() % 40);
        const int T = 1 + (int)(rng() % 512);
        const int table = 2 + (int)(rng() % 64);
        std::vector<double> t_natn(table);
        for (int b = 1; b < table; ++b) t_natn[b] = 1e-4 + 1e-5 * b * (double)(rng() % 8);
        da_perf_model model{(int32_t)(1 + rng() % 80), T, it % 17 == 0 ? 1e300 : 1e5 + (double)(rng() % 1000000), t_natn.data(), table};
        std::vector<std::vector<int64_t>> toks(M);
        std::vector<std::vector<int32_t>> rem(M);
        std::vector<da_instance> inst(M);
        for (int i = 0; i < M; ++i) {
            const int beta = (int)(rng() % table);
            int64_t blocks = 0, remote = 0;
            for (int r = 0; r < beta; ++r) {
                const int64_t s = 1 + (int64_t)(rng() % (rng() % 4 == 0 ? 2000000 : 3000));
                const int64_t nb = (s + T - 1) / T;
                const int32_t rb = rng() % 3 == 0 ? (int32_t)(rng() % (nb + 1)) : 0;
                toks[i].push_back(s);
                rem[i].push_back(rb);
                blocks += nb;
                remote += rb;
            }
            inst[i].num_requests = beta;
            inst[i].req_tokens = toks[i].data();
            inst[i].req_remote_blocks = (i % 5 == 0) ? nullptr : rem[i].data();
            if (i % 5 == 0) remote = 0;
            inst[i].hosted_blocks = rng() % 4 == 0 ? (int32_t)(rng() % 100) : 0;
            const int64_t used = blocks - remote + inst[i].hosted_blocks;
            inst[i].capacity_blocks = (int32_t)(used + 1 + (int64_t)(rng() % 3 == 0 ? 0 : rng() % 4000));
            inst[i].waiting = (int32_t)(rng() % 50);
            inst[i].admit_blocks = (int32_t)(rng() % 10);
        }
        std::vector<da_move> moves((size_t)M * M + 1);
        int32_t n = -1;
        double before = 0, after = 0;
        const da_status st = da_placement_schedule(&model, inst.data(), M, (int32_t)(rng() % table), (double)(rng() % 100) / 99.0,
                                                   moves.data(), (int32_t)moves.size(), &n, &before, &after);
        CHECK(st == DA_OK && n >= 0 && n <= M * M);
        CHECK(before >= 0.0 && after >= 0.0);
        for (int x = 0; x < n; ++x) {
            const da_move &mv = moves[x];
            CHECK(mv.debtor >= 0 && mv.debtor < M && mv.creditor >= 0 && mv.creditor < M && mv.debtor != mv.creditor);
            CHECK(mv.request >= 0 && mv.request < inst[mv.debtor].num_requests && mv.blocks >= 1);
        }
        // a one-slot buffer still reports the full count
        int32_t n1 = -1;
        da_move one;
        const da_status st1 = da_placement_schedule(&model, inst.data(), M, 64, 0.7, &one, 1, &n1, nullptr, nullptr);
        CHECK((st1 == DA_OK && n1 <= 1) || (st1 == DA_ERR_WORKSPACE && n1 > 1));
    }
    std::puts("host sanitizer driver: ok");
    return 0;
}
