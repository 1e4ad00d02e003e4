// Exercises mts::CopyPool (the copy threads of the transfer pipeline) on its own, so that it can be
// built with -fsanitize=thread or -fsanitize=address,undefined on the CPU: copies of many sizes
// through pools of 1..6 threads, back to back (helpers polling) and after pauses (helpers
// asleep), from two pools at once, each result compared byte for byte.  Exit status 0 = all equal.
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

#include <chrono>
#include <thread>
#include <vector>

#include "../../paper_2604_22881_amd/csrc/mts_copy_pool.hpp"

static uint64_t next(uint64_t& s) {
  s ^= s << 13; s ^= s >> 7; s ^= s << 17;
  return s;
}

static int run(int threads, uint64_t seed, int rounds) {
  mts::CopyPool pool(threads);
  const size_t cap = 3u << 20;
  std::vector<unsigned char> src(cap), dst(cap);
  for (size_t i = 0; i < cap; ++i) src[i] = (unsigned char)(next(seed) >> 11);
  int bad = 0;
  for (int r = 0; r < rounds; ++r) {
    size_t n = (size_t)(next(seed) % cap);
    if (r % 5 == 0) n = (size_t)(next(seed) % 4096);           // short copies take the single-thread path
    const size_t off = (size_t)(next(seed) % (cap - n + 1));
    std::fill(dst.begin(), dst.end(), (unsigned char)0xEE);
    pool.copy(dst.data() + off, src.data() + off, n);
    for (size_t i = 0; i < cap; ++i) {
      const unsigned char want = (i >= off && i < off + n) ? src[i] : (unsigned char)0xEE;
      if (dst[i] != want) { ++bad; break; }
    }
    if (r % 7 == 3) std::this_thread::sleep_for(std::chrono::microseconds(300));   // lets the helpers fall asleep
  }
  return bad;
}

int main(int argc, char** argv) {
  const int rounds = argc > 1 ? atoi(argv[1]) : 40;
  int bad = 0;
  for (int threads = 1; threads <= 6; ++threads) bad += run(threads, 0x9E3779B97F4A7C15ull + threads, rounds);
  // two pools used from two threads at the same time (the onload and the offload worker each own one)
  int bad_a = 0, bad_b = 0;
  std::thread a([&] { bad_a = run(3, 77, rounds); });
  std::thread b([&] { bad_b = run(4, 78, rounds); });
  a.join();
  b.join();
  bad += bad_a + bad_b;
  for (int k = 0; k < 20; ++k) { mts::CopyPool p(1 + k % 5); }   // construction and teardown with idle helpers
  printf("copy pool check: %d mismatching copies\n", bad);
  return bad == 0 ? 0 : 1;
}
