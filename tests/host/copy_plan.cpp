// Host-only unit test of the copy planning of the KV-swap library's engine: a move list is
// reordered (order_for_strided_copies) and cut into contiguous and 2-D strided copies
// (plan_copies).  The plan is applied here to plain byte arrays, in both directions, and must
// move exactly what the definition says: staging record k <-> the host record of move k.  Every
// byte outside the moved records must stay untouched, no byte may be written twice, and a
// strided copy may only be chosen where the library says it may (equal runs, constant positive
// pitch, rows not overlapping, chunk limit).
#include <stdio.h>
#include <string.h>

#include <set>

#include "../../paper_2411_18424_amd/csrc/kv_pool.hpp"

static int g_fail = 0;
#define EXPECT(c, ...)                                              \
  do {                                                              \
    if (!(c)) {                                                     \
      fprintf(stderr, "FAIL %s:%d: %s: ", __FILE__, __LINE__, #c);  \
      fprintf(stderr, __VA_ARGS__);                                 \
      fprintf(stderr, "\n");                                        \
      ++g_fail;                                                     \
    }                                                               \
  } while (0)

static uint64_t mix(uint64_t* s) {
  uint64_t z = (*s += 0x9E3779B97F4A7C15ull);
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
  return z ^ (z >> 31);
}

int main() {
  const int64_t R = 48;  // bytes per block record: small, so whole arenas can be compared
  uint64_t rng = 20241127;
  int64_t total_copies = 0, total_strided = 0, total_runs = 0;
  for (int trial = 0; trial < 3000; ++trial) {
    const int64_t arena = 40 + (int64_t)(mix(&rng) % 400);          // records
    const int density = 1 + (int)(mix(&rng) % 9);                   // tenths
    const int64_t chunk_records = 1 + (int64_t)(mix(&rng) % 40);    // copy_chunk in records
    kv_pool p;
    p.plan = true;
    p.R = R;
    p.copy_chunk = chunk_records * R;
    p.strided_copies = trial % 7 != 0;
    // the moved set: a random subset of the arena's records, in logical order ascending or, for
    // images in several extents, in two ascending pieces out of order
    std::vector<int64_t> recs;
    for (int64_t r = 0; r < arena; ++r)
      if ((int)(mix(&rng) % 10) < density) recs.push_back(r);
    if (trial % 5 == 0 && recs.size() > 4) std::rotate(recs.begin(), recs.begin() + (long)(recs.size() / 3), recs.end());
    std::vector<kvi::Move> mv;
    for (size_t k = 0; k < recs.size(); ++k) mv.push_back({recs[k] * R, (int32_t)(1000 + k)});
    std::vector<kvi::Move> before = mv;
    kvi::order_for_strided_copies(&p, mv);
    // a permutation of the same moves
    EXPECT(mv.size() == before.size(), "size");
    std::set<std::pair<int64_t, int32_t>> a, b;
    for (auto& m : before) a.insert({m.host_off, m.phys});
    for (auto& m : mv) b.insert({m.host_off, m.phys});
    EXPECT(a == b, "not a permutation");
    std::vector<kvi::CopyDesc> plan;
    kvi::plan_copies(mv.data(), (int64_t)mv.size(), R, p.copy_chunk, p.strided_copies, &plan);
    // device -> host: staging holds record k = bytes (phys_k, byte index); host starts as 0xEE
    std::vector<uint8_t> host((size_t)(arena * R), 0xEE), stag((size_t)(mv.size() * R));
    std::vector<uint8_t> written((size_t)(arena * R), 0);
    for (size_t k = 0; k < mv.size(); ++k)
      for (int64_t o = 0; o < R; ++o) stag[k * R + (size_t)o] = (uint8_t)(mv[k].phys * 7 + o);
    int64_t runs = mv.empty() ? 0 : 1;
    for (size_t k = 1; k < mv.size(); ++k)
      if (mv[k].host_off != mv[k - 1].host_off + R) ++runs;
    total_runs += runs;
    for (const kvi::CopyDesc& c : plan) {
      ++total_copies;
      EXPECT(c.width > 0 && c.rows >= 1 && c.width * c.rows <= std::max(p.copy_chunk, c.width), "copy larger than the chunk limit");
      if (c.rows > 1) {
        ++total_strided;
        EXPECT(p.strided_copies, "strided copy although switched off");
        EXPECT(c.pitch >= c.width && c.pitch <= kvi::KV_MAX_COPY_PITCH, "pitch %lld width %lld", (long long)c.pitch, (long long)c.width);
        EXPECT(c.width <= kvi::KV_MAX_STRIDED_WIDTH, "row of %lld bytes in a strided copy", (long long)c.width);
      }
      for (int64_t r = 0; r < c.rows; ++r) {
        const int64_t h0 = c.host_off + r * c.pitch, s0 = c.slot_off + r * c.width;
        EXPECT(h0 >= 0 && h0 + c.width <= arena * R && s0 >= 0 && s0 + c.width <= (int64_t)stag.size(), "copy out of bounds");
        if (h0 < 0 || h0 + c.width > arena * R || s0 < 0 || s0 + c.width > (int64_t)stag.size()) return 1;
        for (int64_t o = 0; o < c.width; ++o) {
          EXPECT(!written[(size_t)(h0 + o)], "host byte written twice");
          written[(size_t)(h0 + o)] = 1;
        }
        memcpy(&host[(size_t)h0], &stag[(size_t)s0], (size_t)c.width);
      }
    }
    std::vector<uint8_t> want((size_t)(arena * R), 0xEE);
    for (size_t k = 0; k < mv.size(); ++k) memcpy(&want[(size_t)mv[k].host_off], &stag[k * R], (size_t)R);
    EXPECT(host == want, "device-to-host plan moved the wrong bytes (trial %d)", trial);
    // host -> device with the same plan: staging must end up with the host records
    std::vector<uint8_t> stag2(stag.size(), 0x11);
    for (const kvi::CopyDesc& c : plan)
      for (int64_t r = 0; r < c.rows; ++r)
        memcpy(&stag2[(size_t)(c.slot_off + r * c.width)], &want[(size_t)(c.host_off + r * c.pitch)], (size_t)c.width);
    EXPECT(stag2 == stag, "host-to-device plan moved the wrong bytes (trial %d)", trial);
    if (!p.strided_copies) EXPECT((int64_t)plan.size() >= runs, "fewer copies than runs without strided copies");
  }
  EXPECT(total_strided > 1000, "strided copies were hardly ever chosen: %lld", (long long)total_strided);
  EXPECT(total_copies < total_runs, "strided copies should need fewer copies than runs: %lld vs %lld", (long long)total_copies, (long long)total_runs);
  printf("copy_plan: %d failures (%lld runs -> %lld copies, %lld of them strided)\n", g_fail, (long long)total_runs,
         (long long)total_copies, (long long)total_strided);
  return g_fail ? 1 : 0;
}
