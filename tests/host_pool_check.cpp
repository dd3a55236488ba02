#include "ngc_host_pool.h"
#include <atomic>
#include <cstdio>
int main() {
    for (int rep = 0; rep < 50; ++rep) {
        ngc_host_pool pool;
        long total = 0;
        for (int job = 0; job < 200; ++job) {
            const int cnt = 1 + (job * 7 + rep) % 9;
            std::atomic<long> sum(0);
            std::vector<int> hit(cnt + 1, 0);
            pool.start(cnt, [&](int tid) { hit[tid]++; sum.fetch_add(tid); });
            pool.wait();
            for (int t = 1; t <= cnt; ++t) if (hit[t] != 1) { printf("bad hit %d %d\n", t, hit[t]); return 1; }
            if (sum.load() != (long)cnt * (cnt + 1) / 2) { printf("bad sum\n"); return 1; }
            total += sum.load();
        }
        if (rep == 0) printf("total %ld\n", total);
    }
    { ngc_host_pool idle; }
    printf("ok\n");
    return 0;
}
