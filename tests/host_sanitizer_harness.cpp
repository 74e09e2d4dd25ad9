// Host entry points under AddressSanitizer / UBSan: pack, shard (all modes), streaming packer,
// latency prediction / selection, exact solver, with ordinary and degenerate inputs.
#include <cstdio>
#include <cstdlib>
#include <vector>
#include <random>
#include "wlb.h"
#define CHECK(x) do { wlb_status st_ = (x); if (st_ != WLB_OK) { printf("FAIL %s -> %d: %s\n", #x, (int)st_, wlb_last_error()); return 1; } } while (0)
#define EXPECT_ERR(x) do { wlb_status st_ = (x); if (st_ == WLB_OK) { printf("expected an error: %s\n", #x); return 1; } } while (0)
int main() {
    std::mt19937 rng(7);
    for (int trial = 0; trial < 200; ++trial) {
        const int n = 1 + rng() % 300;
        std::vector<int32_t> len(n);
        for (auto& x : len) x = 1 + (rng() % 10 == 0 ? rng() % 20000 : rng() % 700);
        const int N = 1 + rng() % 8;
        const int64_t lmax = 1000 + rng() % 40000;
        std::vector<int32_t> assign(n); std::vector<int64_t> mlen(N); std::vector<uint64_t> mcost(N);
        CHECK(wlb_pack(len.data(), n, N, lmax, 6, 640000, assign.data(), mlen.data(), mcost.data()));
        for (int cp : {1, 2, 3, 8}) for (int mode : {0, 1, 2}) {
            int64_t T = 0; for (auto x : len) T += x;
            if (mode == 1 && T % (2 * cp) != 0) continue;
            int64_t n_q = 0, n_seg = 0;
            const int rank = (int)(rng() % cp);
            CHECK(wlb_shard_size(len.data(), n, cp, rank, mode, &n_q, &n_seg));
            std::vector<int32_t> q(n_q), cuq(n_seg + 1), kb(n_seg), ke(n_seg), cuk(n + 1);
            int64_t pairs = 0;
            CHECK(wlb_shard(len.data(), n, cp, rank, mode, q.data(), cuq.data(), kb.data(), ke.data(), cuk.data(), &pairs));
        }
    }
    // streaming packer
    {
        wlb_packer* pk = nullptr;
        int64_t thr[2] = {3000, 9000};
        CHECK(wlb_packer_create(4, 20000, 6, 640000, thr, 2, &pk));
        for (int it = 0; it < 50; ++it) {
            const int n = rng() % 60;
            std::vector<int32_t> len(n); std::vector<int64_t> id(n);
            for (int i = 0; i < n; ++i) { len[i] = 1 + rng() % 12000; id[i] = it * 1000 + i; }
            std::vector<int64_t> out_id(4096); std::vector<int32_t> out_len(4096), out_mb(4096);
            int64_t n_out = 0;
            std::vector<int64_t> mlen(4); std::vector<uint64_t> mcost(4);
            CHECK(wlb_packer_step(pk, len.data(), id.data(), n, out_id.data(), out_len.data(), out_mb.data(), 4096, &n_out, mlen.data(), mcost.data()));
        }
        int64_t lo = 0, qd = 0;
        CHECK(wlb_packer_pending(pk, &lo, &qd));
        wlb_packer_destroy(pk);
    }
    // selection and the exact solver
    {
        int32_t ql[3] = {128, 1024, 8192}, kl[3] = {128, 4096, 65536};
        double tf[9] = {50, 80, 90, 200, 400, 500, 300, 700, 900};
        wlb_kernel_profile prof{3, 3, ql, kl, tf, 128, 128};
        for (int trial = 0; trial < 50; ++trial) {
            const int n = 1 + rng() % 40;
            std::vector<int32_t> len(n);
            int64_t T = 0;
            for (auto& x : len) { x = 1 + rng() % 9000; T += x; }
            len[0] += (int32_t)((16 - T % 16) % 16);
            double lat[8]; int32_t mode; double ls, ld;
            CHECK(wlb_predict_latency(len.data(), n, 8, 0, 32, 128, &prof, lat));
            CHECK(wlb_select_sharding(len.data(), n, 8, 32, 128, &prof, &mode, &ls, &ld));
        }
        for (int trial = 0; trial < 30; ++trial) {
            const int n = 1 + rng() % 12, N = 1 + rng() % 4;
            std::vector<int32_t> len(n);
            for (auto& x : len) x = 1 + rng() % 500;
            std::vector<int32_t> a(n); std::vector<int64_t> ml(N); std::vector<uint64_t> mc(N);
            uint64_t opt; int32_t proven;
            wlb_status st = wlb_pack_optimal(len.data(), n, N, 2000, 6, 640000, 200000, a.data(), ml.data(), mc.data(), &opt, &proven);
            (void)st;   // infeasible instances return INVALID_ARG
        }
    }
    // errors
    {
        int32_t bad[2] = {5, 0};
        int32_t a[2]; int64_t ml[2]; uint64_t mc[2];
        EXPECT_ERR(wlb_pack(bad, 2, 2, 100, 1, 1, a, ml, mc));
        EXPECT_ERR(wlb_pack(nullptr, 2, 2, 100, 1, 1, a, ml, mc));
        int64_t nq, ns;
        EXPECT_ERR(wlb_shard_size(bad, 2, 0, 0, 0, &nq, &ns));
    }
    printf("host entry points: ok\n");
    return 0;
}
