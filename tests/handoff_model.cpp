// Host-threads model of the cross-workgroup hand-off of the persistent kernel (Section 4.2: Lamport-style validity
// carried by the data).  TEST INFRASTRUCTURE: one thread plays one workgroup, std::atomic words play the exchange
// ring.  It shares no code with the HIP path; it restates the protocol so that its logic can be checked on the CPU,
// also under -fsanitize=thread:
//
//   * the ring has 4 slots; slot t mod 4 holds step t; a word equal to 0x80000000 means "not written yet";
//   * step t of a workgroup: wait until every word it needs of slot (t - 1) mod 4 is written, compute, publish its own
//     words into slot t mod 4, then mark its own words of slot (t + 2) mod 4 as not written (re-arm); the re-arm is
//     ordered before the next publish;
//   * flow control: every workgroup also waits for one word of EVERY workgroup, whether it needs its value or not.
//     That keeps all workgroups within one step of each other, which is what makes re-arming two steps ahead (and
//     overwriting a slot four steps later) safe.  Without it a workgroup that needs nothing from a slow one runs
//     ahead and destroys words the slow one, or its readers, have not seen yet.
//
// usage: handoff_model G E T pattern flow slow seed [spin_limit]
//   G workgroups of E words, T steps; pattern 0 = everyone reads everyone, 1 = workgroup g reads workgroups <= g,
//   2 = workgroup g reads only itself and g - 1; flow 1 = with the flow-control words; slow = index of a workgroup that
//   pauses in every step (-1 none).  Exit 0 = every value matches the sequential reference, 1 = mismatch, 2 = a wait
//   gave up.
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

bool needs(int pattern, int reader, int producer) {
  if (pattern == 0) return true;
  if (pattern == 1) return producer <= reader;
  return producer == reader || producer == reader - 1;
}

}  // namespace

int main(int argc, char** argv) {
  if (argc < 8) { std::fprintf(stderr, "usage: %s G E T pattern flow slow seed\n", argv[0]); return 64; }
  const int G = std::atoi(argv[1]), E = std::atoi(argv[2]), T = std::atoi(argv[3]), pattern = std::atoi(argv[4]);
  const bool flow = std::atoi(argv[5]) != 0;
  const int slow = std::atoi(argv[6]);
  const uint32_t seed = (uint32_t)std::atoi(argv[7]);
  const long spin_limit = argc > 8 ? std::atol(argv[8]) : 200000000L;
  const int n = G * E;

  // sequential reference: value[t][i] for t = 0..T (value[0] is the initial state)
  std::vector<std::vector<uint32_t>> ref(T + 1, std::vector<uint32_t>(n));
  for (int i = 0; i < n; ++i) ref[0][i] = mix(seed, (uint32_t)i, 0);
  for (int t = 1; t <= T; ++t)
    for (int g = 0; g < G; ++g) {
      uint64_t sum = 0;
      for (int p = 0; p < G; ++p)
        if (needs(pattern, g, p)) for (int e = 0; e < E; ++e) sum += ref[t - 1][p * E + e];
      for (int e = 0; e < E; ++e) ref[t][g * E + e] = mix(sum, (uint32_t)(g * E + e), (uint32_t)t);
    }

  std::vector<std::atomic<uint32_t>> ring((size_t)kSlots * n);
  for (auto& w : ring) w.store(kNotWritten, std::memory_order_relaxed);
  for (int i = 0; i < n; ++i) ring[i].store(ref[0][i], std::memory_order_relaxed);   // step 0 lives in slot 0
  std::vector<std::vector<uint32_t>> produced(G, std::vector<uint32_t>((size_t)T * E));
  std::atomic<int> gave_up{0};

  auto workgroup = [&](int g) {
    uint32_t lcg = seed * 747796405u + (uint32_t)g * 2891336453u + 1u;
    for (int t = 1; t <= T && !gave_up.load(std::memory_order_relaxed); ++t) {
      const int prev = (t - 1) % kSlots, cur = t % kSlots, rearm = (t + 2) % kSlots;
      uint64_t sum = 0;
      for (int p = 0; p < G; ++p) {
        const bool wanted = needs(pattern, g, p);
        const int words = wanted ? E : (flow ? 1 : 0);       // flow control: one word of everybody else
        for (int e = 0; e < words; ++e) {
          uint32_t v;
          long spins = 0;
          while ((v = ring[(size_t)prev * n + p * E + e].load(std::memory_order_acquire)) == kNotWritten) {
            if (++spins > spin_limit || gave_up.load(std::memory_order_relaxed)) { gave_up.store(1); return; }
            std::this_thread::yield();
          }
          if (wanted) sum += v;
        }
      }
      if (g == slow) std::this_thread::sleep_for(std::chrono::microseconds(300));
      lcg = lcg * 1664525u + 1013904223u;
      if ((lcg >> 28) == 0) std::this_thread::sleep_for(std::chrono::microseconds(20));   // occasional hiccup anywhere
      for (int e = 0; e < E; ++e) {
        const uint32_t v = mix(sum, (uint32_t)(g * E + e), (uint32_t)t);
        produced[g][(size_t)(t - 1) * E + e] = v;
        ring[(size_t)cur * n + g * E + e].store(v, std::memory_order_release);        // publish
      }
      for (int e = 0; e < E; ++e)                                                     // re-arm two steps ahead;
        ring[(size_t)rearm * n + g * E + e].store(kNotWritten, std::memory_order_relaxed);   // ordered before the next publish (release)
    }
  };

  std::vector<std::thread> threads;
  for (int g = 0; g < G; ++g) threads.emplace_back(workgroup, g);
  for (auto& th : threads) th.join();
  if (gave_up.load()) { std::puts("GAVE UP"); return 2; }
  long bad = 0;
  for (int g = 0; g < G; ++g)
    for (int t = 1; t <= T; ++t)
      for (int e = 0; e < E; ++e)
        if (produced[g][(size_t)(t - 1) * E + e] != ref[t][g * E + e]) ++bad;
  if (bad) { std::printf("MISMATCH %ld\n", bad); return 1; }
  std::puts("OK");
  return 0;
}
