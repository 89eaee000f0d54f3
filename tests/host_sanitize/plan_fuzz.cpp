// host-only sanitizer run of the bucket plan and ready tracker
#include "bucket_plan.h"
#include <cstdio>
#include <random>
#include <utility>
int main() {
    std::mt19937_64 rng(1);
    for (int it = 0; it < 20000; ++it) {
        ddp::BucketPlan plan;
        int n = 1 + rng() % 60;
        plan.params.resize(n);
        for (auto& p : plan.params) { p.numel = rng() % 5000; p.dtype = rng() % 3; }
        uint64_t cap = (it % 7 == 0) ? UINT64_MAX : rng() % 40000;
        if (it % 3 == 0) {
            plan.assign(cap);
        } else {
            // a traced visit order: a random permutation, sometimes damaged on purpose
            std::vector<int32_t> order(n);
            for (int i = 0; i < n; ++i) order[i] = i;
            for (int i = n - 1; i > 0; --i) std::swap(order[i], order[rng() % (i + 1)]);
            bool bad = it % 11 == 0;
            if (bad) {
                switch (rng() % 3) {
                    case 0: order[rng() % n] = n + (int)(rng() % 5); break;     // out of range
                    case 1: order[rng() % n] = -1 - (int)(rng() % 5); break;    // negative
                    default: order.push_back(0); break;                          // too long / duplicate
                }
            }
            const bool ok = plan.assign(cap, &order);
            if (ok == bad) { printf("permutation check failed\n"); return 1; }
            if (!ok) continue;
            size_t k = 0;
            for (const auto& b : plan.buckets)
                for (int32_t p : b.params)
                    if (order[k++] != p) { printf("fill order differs from the visit order\n"); return 1; }
        }
        ddp::ReadyTracker tr; tr.reset(plan);
        for (int round = 0; round < 2; ++round) {
            std::vector<int32_t> launch;
            int marks = rng() % (n + 1);
            for (int k = 0; k < marks; ++k) { int p = (int)(rng() % (n + 4)) - 2; tr.mark(p, launch); }
            tr.drain(launch);
            if ((int)launch.size() != (int)plan.buckets.size()) { printf("bad launch count\n"); return 1; }
            for (size_t i = 0; i < launch.size(); ++i) if (launch[i] != (int)i) { printf("bad order\n"); return 1; }
            tr.new_iteration();
        }
    }
    printf("ok\n");
    return 0;
}
