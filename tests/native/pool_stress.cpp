// Stress test of the host tier's thread pool, built with -fsanitize=thread by
// tests/test_pool_native.py.  It drives the pool the way the tiered lookup does:
// start a job, follow the completed prefix from the calling thread and consume
// the finished tasks' results while later tasks are still running, then wait.
#include <cstdio>
#include <cstdlib>
#include <vector>

#include "bgl_pool.h"

int main(int argc, char **argv)
{
    const int threads = argc > 1 ? atoi(argv[1]) : 4;
    const int rounds = argc > 2 ? atoi(argv[2]) : 300;
    bgl::Pool pool(threads);
    if (pool.threads() != (threads < 1 ? 1 : threads)) { printf("thread count %d\n", pool.threads()); return 1; }
    std::vector<long> out;
    unsigned long long seed = 12345;
    long checked = 0;
    for (int r = 0; r < rounds; ++r) {
        seed = seed * 6364136223846793005ull + 1442695040888963407ull;
        const long tasks = (long)((seed >> 33) % 97);          // includes 0 and 1
        const long per = 1 + (long)((seed >> 20) % 50);
        out.assign((size_t)(tasks * per), -1);
        bgl::Pool::Fn fn = [&](int64_t k) {
            for (long j = 0; j < per; ++j) out[(size_t)(k * per + j)] = (long)r * 1000003 + k * per + j;
        };
        if (r % 3 == 0) {
            pool.run(tasks, fn);                               // the caller works too
            for (long i = 0; i < tasks * per; ++i)
                if (out[(size_t)i] != (long)r * 1000003 + i) { printf("run: wrong value\n"); return 1; }
            checked += tasks * per;
            continue;
        }
        pool.start(tasks, fn);
        long seen = 0;
        while (seen < tasks) {
            const long done = (long)pool.done_prefix();
            if (done < seen) { printf("prefix went backwards\n"); return 1; }
            for (long i = seen * per; i < done * per; ++i)     // finished tasks are readable right away
                if (out[(size_t)i] != (long)r * 1000003 + i) { printf("start: wrong value\n"); return 1; }
            checked += (done - seen) * per;
            seen = done;
            if (r % 2 == 0) (void)pool.help_one();             // the caller takes a task between two looks
        }
        pool.wait();
        if (pool.done_prefix() != tasks) { printf("prefix after wait\n"); return 1; }
    }
    printf("ok %ld\n", checked);
    return 0;
}
