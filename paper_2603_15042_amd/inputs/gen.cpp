// Seeded synthetic-input generator shared by the tests, the oracle-side checks
// and the GPU harness.  It holds none of the method's arithmetic: it only turns
// (seed, tensor id, element index) into a value, so any element of any tensor
// can be regenerated in any order, by any number of threads, with equal bits.
//
//   z      = mix(seed, tensor, index, draw)          (splitmix64 finaliser)
//   unif   = (z >> 11 + 0.5) * 2^-53                 in (0,1)
//   normal = sqrt(-2 ln u1) cos(2 pi u2)             (Box-Muller, double)
//   stored = nearest bf16, ties to even
#include <cmath>
#include <cstdint>
#include <cstring>
#include <thread>
#include <vector>
#include <algorithm>

namespace {
inline uint64_t mix64(uint64_t z) {
  z += 0x9e3779b97f4a7c15ull;
  z = (z ^ (z >> 30)) * 0xbf58476d1ce4e5b9ull;
  z = (z ^ (z >> 27)) * 0x94d049bb133111ebull;
  return z ^ (z >> 31);
}
inline uint64_t draw(uint64_t seed, uint64_t tensor, uint64_t index, uint64_t which) {
  uint64_t s = mix64(seed * 0xd1342543de82ef95ull + tensor);
  return mix64(s ^ mix64(index * 2 + which));
}
inline double unit(uint64_t z) { return (static_cast<double>(z >> 11) + 0.5) * 0x1.0p-53; }

inline uint16_t to_bf16(double d) {
  float f = static_cast<float>(d);
  uint32_t u;
  std::memcpy(&u, &f, 4);
  // any deterministic rounding serves: whatever bf16 comes out IS the input
  uint32_t r = u + 0x7fffu + ((u >> 16) & 1u);
  return static_cast<uint16_t>(r >> 16);
}

template <class F>
void run(int64_t n, int threads, F&& f) {
  int t = static_cast<int>(std::max<int64_t>(1, std::min<int64_t>(threads, n / 4096 + 1)));
  if (t == 1) { f(0, n); return; }
  std::vector<std::thread> pool;
  for (int w = 0; w < t; ++w) pool.emplace_back([=, &f] { f(n * w / t, n * (w + 1) / t); });
  for (auto& th : pool) th.join();
}
}  // namespace

extern "C" {

// Elements [first, first+n) of the tensor are written to out[0..n).
void vte_gen_normal_bf16(uint64_t seed, uint64_t tensor, int64_t first, int64_t n,
                         double mean, double stddev, uint16_t* out, int threads) {
  run(n, threads, [=](int64_t lo, int64_t hi) {
    for (int64_t i = lo; i < hi; ++i) {
      double u1 = unit(draw(seed, tensor, first + i, 0)), u2 = unit(draw(seed, tensor, first + i, 1));
      double g = std::sqrt(-2.0 * std::log(u1)) * std::cos(6.283185307179586476925 * u2);
      out[i] = to_bf16(mean + stddev * g);
    }
  });
}

void vte_gen_uniform_bf16(uint64_t seed, uint64_t tensor, int64_t n, double lo_v,
                          double hi_v, uint16_t* out, int threads) {
  run(n, threads, [=](int64_t lo, int64_t hi) {
    for (int64_t i = lo; i < hi; ++i)
      out[i] = to_bf16(lo_v + (hi_v - lo_v) * unit(draw(seed, tensor, i, 0)));
  });
}

// Integers in [lo_i, hi_i] times 2^scale_pow2, exactly representable in bf16 when
// |integer| < 256: inputs on which every fp32 partial sum is exact.
void vte_gen_int_bf16(uint64_t seed, uint64_t tensor, int64_t n, int lo_i, int hi_i,
                      int scale_pow2, uint16_t* out, int threads) {
  run(n, threads, [=](int64_t lo, int64_t hi) {
    uint64_t span = static_cast<uint64_t>(hi_i - lo_i + 1);
    for (int64_t i = lo; i < hi; ++i) {
      int v = lo_i + static_cast<int>(draw(seed, tensor, i, 0) % span);
      out[i] = to_bf16(std::ldexp(static_cast<double>(v), scale_pow2));
    }
  });
}

void vte_gen_tokens(uint64_t seed, uint64_t tensor, int64_t n, int64_t vocab, int32_t* out) {
  for (int64_t i = 0; i < n; ++i)
    out[i] = static_cast<int32_t>(draw(seed, tensor, i, 0) % static_cast<uint64_t>(vocab));
}

}  // extern "C"
