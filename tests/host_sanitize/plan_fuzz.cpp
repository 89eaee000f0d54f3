// host-only sanitizer run of the bucket plan and ready tracker
#include "bucket_plan.h"
#include <cstdio>
#include <random>
int main() {
    std::mt19937_64 rng(1);
    for (int it = 0; it < 20000; ++it) {
        ddp::BucketPlan plan;
        int n = 1 + rng() % 60;
        plan.params.resize(n);
        for (auto& p : plan.params) { p.numel = rng() % 5000; p.dtype = rng() % 3; }
        uint64_t cap = (it % 7 == 0) ? UINT64_MAX : rng() % 40000;
        plan.assign(cap);
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
