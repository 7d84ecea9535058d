// Corrupted streams through every reader of the reference CPU codec, built with the address and
// undefined-behaviour sanitizers: whatever the bytes say, a call ends with a status, reads nothing
// outside the buffer it was given and writes nothing outside its output.  Exit status 0 = clean.
#include <cstdio>
#include <cstdlib>
#include <random>

#include "../../oracle/zcref.cpp"

int main() {
  std::mt19937_64 rng(20250218);
  unsigned long calls = 0, accepted = 0;
  for (int variant = 0; variant < 2; ++variant) {
    zcref_set_indexed(variant);
    for (int round = 0; round < 24; ++round) {
      const size_t n = size_t(rng() % 9000);
      std::vector<float> x(n);
      double v = 0.0;
      for (size_t i = 0; i < n; ++i) {
        v += double(int(rng() % 2001) - 1000) * 1e-3;
        if (rng() % 50 == 0) v += double(int(rng() % 2001) - 1000) * 1.0;      // now and then a wide block
        x[i] = float(v);
      }
      std::vector<uint8_t> good(zcref_compress_bound(n) + 64);
      size_t total = 0;
      const int st = zcref_compress(x.data(), n, 1e-3f, good.data(), good.size(), &total);
      if (st != OK && st != ERR_BOUND) return 2;
      for (int trial = 0; trial < 40; ++trial) {
        // the stream in a buffer of exactly its size, so that any read past it is caught
        size_t bytes = total;
        if (rng() % 6 == 0 && bytes) bytes = size_t(rng() % bytes);             // truncated
        std::vector<uint8_t> s(good.begin(), good.begin() + bytes);
        const int edits = int(rng() % 4);
        for (int e = 0; e < edits && bytes; ++e) {
          const size_t region = rng() % 3;                                       // header, tables, anywhere
          const size_t span = region == 0 ? 32 : region == 1 ? 32 + n / 4 + 64 : bytes;
          const size_t pos = size_t(rng() % (span < bytes ? span : bytes));
          s[pos] = (rng() % 2) ? uint8_t(rng()) : uint8_t(s[pos] ^ (1u << (rng() % 8)));
        }
        std::vector<float> y(n + 1);
        std::vector<uint8_t> out(zcref_compress_bound(n) + 64);
        size_t m = 0, ob = 0;
        int r = zcref_decompress(s.data(), s.size(), y.data(), n, &m);
        accepted += r == OK;
        r = zcref_decompress_average(s.data(), s.size(), y.data(), n, &m);
        r = zcref_decompress_range(s.data(), s.size(), 2048 * size_t(rng() % 6), size_t(rng() % 5000), y.data(), n, &m);
        r = zcref_inspect(s.data(), s.size(), nullptr, nullptr, nullptr);
        const void* chunks[2] = {good.data(), s.data()};
        const size_t sizes[2] = {total, s.size()};
        r = zcref_reduce(chunks, sizes, 2, out.data(), out.size(), &ob);
        r = zcref_reduce_op(chunks, sizes, 2, 1 + int(rng() % 2), out.data(), out.size(), &ob);
        r = zcref_reduce_step_op(s.data(), s.size(), x.data(), n, int(rng() % 3), out.data(), out.size(), &ob);
        (void)r;
        calls += 7;
      }
    }
  }
  std::printf("%lu calls, %lu streams still valid\n", calls, accepted);
  return 0;
}
