// Drives the host-only scheduler of the C ABI through a long pseudo-random trace
// (valid and invalid submissions, moving free-block counts, service-time
// feedback, tiny and huge values) in a build with AddressSanitizer and
// UndefinedBehaviorSanitizer.  Prints a checksum of the decisions; the
// sanitizers abort on any finding.  Built and run by test_sched_sanitizers.py.
#include <cstdint>
#include <cstdio>
#include <vector>

#include "../include/fastcache.h"

static uint64_t rng_state = 0x9e3779b97f4a7c15ull;
static uint64_t next_u64() {  // splitmix64
  uint64_t z = (rng_state += 0x9e3779b97f4a7c15ull);
  z = (z ^ (z >> 30)) * 0xbf58476d1ce4e5b9ull;
  z = (z ^ (z >> 27)) * 0x94d049bb133111ebull;
  return z ^ (z >> 31);
}

int main() {
  uint64_t sum = 0;
  for (int round = 0; round < 40; ++round) {
    const int b_min = 1 + (int)(next_u64() % 4);
    const int b_max = b_min + (int)(next_u64() % 40);
    const int64_t max_wait = (int64_t)(next_u64() % 100000);
    fc_sched* s = nullptr;
    if (fc_sched_create(&s, b_min, b_max, max_wait) != FC_OK) return 2;
    // bad constructions are refused
    fc_sched* bad = nullptr;
    if (fc_sched_create(&bad, 0, 4, 10) == FC_OK || fc_sched_create(&bad, 5, 4, 10) == FC_OK ||
        fc_sched_create(&bad, 1, 4, -1) == FC_OK || fc_sched_create(nullptr, 1, 4, 1) == FC_OK)
      return 3;
    int64_t now = 0, id = 0;
    std::vector<int64_t> out(64);
    for (int step = 0; step < 3000; ++step) {
      const uint64_t r = next_u64();
      now += (int64_t)(r % 5000);
      switch (r >> 60) {
        case 0: {  // invalid submissions: time going back, bad budget, duplicate id
          sum += (uint64_t)fc_sched_submit(s, id + 1000000, now - 1 - (int64_t)(r % 7), 100, 50);
          sum += (uint64_t)fc_sched_submit(s, id + 1000001, now, 100, 0);
          sum += (uint64_t)fc_sched_submit(s, id + 1000002, now, 100, 101);
          if (id > 0) sum += (uint64_t)fc_sched_submit(s, id - 1, now, 100, 50);
          break;
        }
        case 1: case 2: case 3: case 4: case 5: case 6: {
          const int len = 1 + (int)((r >> 8) % 32768);
          const int budget = 1 + (int)((r >> 24) % (uint64_t)len);
          sum += (uint64_t)fc_sched_submit(s, id++, now, len, budget);
          break;
        }
        case 7: sum += (uint64_t)fc_sched_adjust(s, (int64_t)((r >> 8) % 200000)); break;
        case 8: sum += (uint64_t)fc_sched_adjust(s, (int64_t)1 << 50); break;  // absurdly slow batch
        default: {
          const int free_blocks = (int)((r >> 8) % 6000);
          const int cap = 1 + (int)((r >> 32) % 64);
          const int n = fc_sched_form_batch(s, now, free_blocks, out.data(), cap);
          if (n < 0) {
            sum += 7;  // capacity too small for the batch: nothing was taken
          } else {
            for (int i = 0; i < n; ++i) sum = sum * 1099511628211ull + (uint64_t)out[i];
          }
          sum += (uint64_t)fc_sched_pending(s) + (uint64_t)fc_sched_batch_target(s) +
                 (uint64_t)fc_sched_ready(s, now);
        }
      }
    }
    fc_sched_destroy(s);
  }
  fc_sched_destroy(nullptr);
  std::printf("%llu\n", (unsigned long long)sum);
  return 0;
}
