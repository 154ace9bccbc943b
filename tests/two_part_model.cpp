// Host-threads model of the two-part copy inside a workgroup of the persistent kernel (options.overlap; Section 4.2 asks
// for useful work while the load stage is in flight).  TEST INFRASTRUCTURE: it shares no code with the HIP path; it
// restates the discipline so that it can be checked on the CPU, also under -fsanitize=thread.
//
// One thread plays one WAVEFRONT; W wavefronts form a workgroup and share a plain (non-atomic) array, the workgroup's LDS
// copy of the exchanged vector; std::atomic words play the exchange ring (4 slots, 0x80000000 = "not written yet", the
// same cross-workgroup protocol as in handoff_model.cpp, everyone reads everyone).  A step of a wavefront:
//   1. poll the ring words of the FIRST part that are its share of the copy, store them into LDS;
//   2. barrier A;  read all of the first part from LDS (the "early words");
//   3. poll its share of the SECOND part, store it into LDS (other wavefronts may still be reading the first part: the
//      two parts are disjoint, which is the whole point);
//   4. barrier B;  read all of the second part;
//   5. publish its own words of the new vector, re-arm the slot two steps ahead;
//   6. barrier C (nobody overwrites LDS while a wavefront of the workgroup still reads it).
// With plant = 1 the early words also read one word of the second part: the mistake this model is there to catch, which
// ThreadSanitizer reports as a data race (and which can show as a wrong value).
//
// usage: two_part_model G W E T plant seed      (E words per wavefront)
// exit 0 = every value matches the sequential reference, 1 = mismatch, 2 = a wait gave up.
#include <pthread.h>

#include <atomic>
#include <chrono>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <thread>
#include <vector>

namespace {
constexpr uint32_t kNotWritten = 0x80000000u;
constexpr int kSlots = 4;
uint32_t mix(uint64_t sum, uint32_t idx, uint32_t t) {
  const uint32_t v = (uint32_t)(sum * 2654435761ull) + idx * 40503u + t * 97u;
  return (v & 0x7fffffffu) | 1u;   // never the mark, never zero
}
}  // namespace

int main(int argc, char** argv) {
  if (argc < 7) { std::fprintf(stderr, "usage: %s G W E T plant seed\n", argv[0]); return 64; }
  const int G = std::atoi(argv[1]), W = std::atoi(argv[2]), E = std::atoi(argv[3]), T = std::atoi(argv[4]);
  const bool plant = std::atoi(argv[5]) != 0;
  const uint32_t seed = (uint32_t)std::atoi(argv[6]);
  const int n = G * W * E, half = n / 2;
  const long spin_limit = 200000000L;

  std::vector<std::vector<uint32_t>> ref(T + 1, std::vector<uint32_t>(n));
  for (int i = 0; i < n; ++i) ref[0][i] = mix(seed, (uint32_t)i, 0);
  for (int t = 1; t <= T; ++t) {
    uint64_t sum = 0;
    for (int i = 0; i < n; ++i) sum += ref[t - 1][i];
    for (int i = 0; i < n; ++i) ref[t][i] = mix(sum, (uint32_t)i, (uint32_t)t);
  }

  std::vector<std::atomic<uint32_t>> ring((size_t)kSlots * n);
  for (auto& w : ring) w.store(kNotWritten, std::memory_order_relaxed);
  for (int i = 0; i < n; ++i) ring[i].store(ref[0][i], std::memory_order_relaxed);
  std::vector<std::vector<uint32_t>> lds(G, std::vector<uint32_t>(n));   // plain memory: what the sanitizer watches
  std::vector<pthread_barrier_t> barrier(G);
  for (auto& b : barrier) pthread_barrier_init(&b, nullptr, (unsigned)W);
  std::vector<uint32_t> produced((size_t)T * n);
  std::atomic<int> gave_up{0};

  auto wavefront = [&](int g, int w) {
    uint32_t lcg = seed * 747796405u + (uint32_t)(g * W + w) * 2891336453u + 1u;
    auto hiccup = [&]() {
      lcg = lcg * 1664525u + 1013904223u;
      if ((lcg >> 28) == 0) std::this_thread::sleep_for(std::chrono::microseconds(30));
    };
    auto copy_share = [&](int slot, int lo, int hi) {   // this wavefront's share: words i with i % W == w
      for (int i = lo + ((w - lo % W) % W + W) % W; i < hi; i += W) {
        uint32_t v;
        long spins = 0;
        while ((v = ring[(size_t)slot * n + i].load(std::memory_order_acquire)) == kNotWritten) {
          if (++spins > spin_limit || gave_up.load(std::memory_order_relaxed)) { gave_up.store(1); break; }
          std::this_thread::yield();
        }
        lds[g][i] = v;
      }
    };
    for (int t = 1; t <= T; ++t) {
      const int prev = (t - 1) % kSlots, cur = t % kSlots, rearm = (t + 2) % kSlots;
      copy_share(prev, 0, half);
      hiccup();
      pthread_barrier_wait(&barrier[g]);                                  // A
      uint64_t sum = 0;
      for (int i = 0; i < half + (plant ? 1 : 0); ++i) sum += lds[g][i];  // early words
      hiccup();
      copy_share(prev, half, n);
      pthread_barrier_wait(&barrier[g]);                                  // B
      for (int i = half + (plant ? 1 : 0); i < n; ++i) sum += lds[g][i];
      hiccup();
      for (int e = 0; e < E; ++e) {
        const int i = (g * W + w) * E + e;
        const uint32_t v = mix(sum, (uint32_t)i, (uint32_t)t);
        produced[(size_t)(t - 1) * n + i] = v;
        ring[(size_t)cur * n + i].store(v, std::memory_order_release);
      }
      for (int e = 0; e < E; ++e) ring[(size_t)rearm * n + (g * W + w) * E + e].store(kNotWritten, std::memory_order_relaxed);
      pthread_barrier_wait(&barrier[g]);                                  // C
      if (gave_up.load(std::memory_order_relaxed)) {}                     // (keep stepping: the others wait at the barriers)
    }
  };

  std::vector<std::thread> threads;
  for (int g = 0; g < G; ++g)
    for (int w = 0; w < W; ++w) threads.emplace_back(wavefront, g, w);
  for (auto& th : threads) th.join();
  if (gave_up.load()) { std::puts("GAVE UP"); return 2; }
  long bad = 0;
  for (int t = 1; t <= T; ++t)
    for (int i = 0; i < n; ++i)
      if (produced[(size_t)(t - 1) * n + i] != ref[t][i]) ++bad;
  if (bad) { std::printf("MISMATCH %ld\n", bad); return 1; }
  std::puts("OK");
  return 0;
}
