// Memory-safety check of the adapter slot manager's host logic (test infrastructure): a manager
// without parts owns no device memory and issues no copies, so its residency bookkeeping runs
// without a GPU.  Built by tests/test_slots_sanitize.py from csrc/slots.hip with the host pass under
// -fsanitize=address,undefined; the id and slot arrays are heap blocks of exactly n entries, so a
// read or write past either aborts the run.  The bookkeeping itself is compared with a model in
// tests/test_slots.py; here only invariants that hold for any correct manager are asserted.
// With -DPLANT_SHORT_OUTPUT the slot array is one entry short and the instrumented build must abort.
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <set>
#include <vector>

#include "../include/preft.h"

static uint64_t state = 42;
static int rnd(int n)
{
    state = state * 6364136223846793005ull + 1442695040888963407ull;
    return (int)((state >> 33) % (uint64_t)n);
}
static void fail(const char *what)
{
    std::fprintf(stderr, "slots_sanitize_driver: %s\n", what);
    std::exit(1);
}

static void exercise(int n_adapters, int n_slots, int max_batch)
{
    preft_slots_t *m = nullptr;
    if (preft_slots_create(&m, n_adapters, n_slots, 0, nullptr) != PREFT_OK || !m) fail("create");
    const int slots = n_slots < n_adapters ? n_slots : n_adapters;
    for (int step = 0; step < 400; ++step) {
        const int n = rnd(max_batch + 1);
        int32_t *ids = (int32_t *)std::malloc(sizeof(int32_t) * (n ? n : 1));
#ifdef PLANT_SHORT_OUTPUT                                          // the check of the check: one entry too few
        int32_t *out = (int32_t *)std::malloc(sizeof(int32_t) * (n > 1 ? n - 1 : 1));
#else
        int32_t *out = (int32_t *)std::malloc(sizeof(int32_t) * (n ? n : 1));
#endif
        std::set<int> distinct;
        for (int i = 0; i < n; ++i) {
            ids[i] = rnd(n_adapters + 3) - 1;                      // -1 and ids past the catalogue included
            if (ids[i] >= 0 && ids[i] < n_adapters) distinct.insert(ids[i]);
        }
        const int rc = preft_slots_acquire(m, ids, n, out, nullptr);
        if ((int)distinct.size() > slots) {
            if (rc != PREFT_ECAPACITY) fail("more distinct adapters than slots was not refused");
        } else {
            if (rc != PREFT_OK) fail("acquire");
            std::set<int> used;
            for (int i = 0; i < n; ++i) {
                const bool valid = ids[i] >= 0 && ids[i] < n_adapters;
                if (!valid && out[i] != -1) fail("an id outside the catalogue got a slot");
                if (valid) {
                    if (out[i] < 0 || out[i] >= slots) fail("slot out of range");
                    if (preft_slots_resident(m, ids[i]) != out[i]) fail("residency query disagrees");
                    used.insert(out[i]);
                }
            }
            if (used.size() != distinct.size()) fail("two adapters of one batch share a slot");
        }
        std::free(ids);
        std::free(out);
    }
    int64_t stats[5];
    if (preft_slots_stats(m, stats) != PREFT_OK || stats[4] != slots || stats[3] != 0) fail("stats");
    if (preft_slots_pool(m, 0) != nullptr) fail("a manager without parts has no pool");
    if (preft_slots_resident(m, -1) != -1 || preft_slots_resident(m, n_adapters) != -1) fail("resident(out of range)");
    if (preft_slots_store(m, 0, 0, nullptr, nullptr) == PREFT_OK) fail("store into a manager without parts");
    if (preft_slots_destroy(m) != PREFT_OK) fail("destroy");
}

int main()
{
    preft_slots_t *m = nullptr;
    if (preft_slots_create(nullptr, 4, 2, 0, nullptr) == PREFT_OK) fail("create(NULL)");
    if (preft_slots_create(&m, 0, 2, 0, nullptr) == PREFT_OK) fail("create(no adapters)");
    if (preft_slots_create(&m, 4, 0, 0, nullptr) == PREFT_OK) fail("create(no slots)");
    if (preft_slots_create(&m, 4, 2, PREFT_MAX_PARTS + 1, nullptr) == PREFT_OK) fail("create(too many parts)");
    exercise(40, 8, 6);
    exercise(512, 32, 40);       // batches that can exceed the slots
    exercise(5, 9, 4);           // more slots than adapters
    exercise(1, 1, 3);
    std::puts("slots_sanitize_driver: ok");
    return 0;
}
