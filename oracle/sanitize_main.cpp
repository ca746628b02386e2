// Sanitizer driver for the CPU oracle (test infrastructure only): includes the oracle's source,
// calls every entry point on small curves of every size from 1 to 70 samples, every dtype, one to
// three rows, broadcast operands and counts up to four, and prints a checksum.  Built by
// tests/test_oracle_hygiene.py with -fsanitize=address,undefined: an access outside an array or
// an undefined operation in any loop of the oracle ends the run with a report and a non-zero
// exit status.  Inputs come from a small linear congruential generator (inputs only; none of the
// curve algebra lives here).
#include "rtc_oracle.cpp"

#include <cstdio>
#include <vector>

namespace {

uint64_t g_state = 0x9E3779B97F4A7C15ull;
uint32_t next_u32() {
  g_state = g_state * 6364136223846793005ull + 1442695040888963407ull;
  return (uint32_t)(g_state >> 33);
}

template <typename T> void fill_monotone(std::vector<T>& v, int64_t rows, int64_t n, int max_inc) {
  v.resize((size_t)(rows * n));
  for (int64_t b = 0; b < rows; ++b) {
    T run = (T)(next_u32() % 6);
    for (int64_t i = 0; i < n; ++i) {
      run = run + (T)(next_u32() % (uint32_t)(max_inc + 1));
      v[(size_t)(b * n + i)] = run;
    }
  }
}

template <typename T> double checksum(const std::vector<T>& v) {
  double s = 0;
  for (size_t i = 0; i < v.size(); ++i) s += (double)v[i] * (double)(1 + i % 7);
  return s;
}

template <typename T> double exercise(int dt) {
  double sum = 0;
  for (int64_t n = 1; n <= 70; ++n) {
    const int64_t batch = 1 + n % 3, m = 1 + (n * 7) % 40, k = 1 + (n * 5) % 50, count = 1 + n % 4;
    std::vector<T> f, g, one, out((size_t)(batch * n)), out2((size_t)(batch * n)), tmp((size_t)(batch * n));
    fill_monotone(f, batch, n, 9);
    fill_monotone(g, batch, n, 5);
    fill_monotone(one, 1, n, 4);
    oracle_minplus_conv(f.data(), g.data(), out.data(), batch, n, n, n, dt); sum += checksum(out);
    oracle_maxplus_deconv(f.data(), g.data(), out.data(), batch, n, n, n, dt); sum += checksum(out);
    oracle_maxplus_conv(f.data(), one.data(), out.data(), batch, n, n, 0, dt); sum += checksum(out);
    oracle_minplus_deconv(one.data(), g.data(), out.data(), batch, n, 0, n, dt); sum += checksum(out);
    std::vector<int64_t> idx = {0, n - 1, n / 2};
    std::vector<T> at(idx.size());
    oracle_product_at(f.data(), g.data(), n, idx.data(), (int64_t)idx.size(), at.data(), 0, dt); sum += checksum(at);
    oracle_product_at(f.data(), g.data(), n, idx.data(), (int64_t)idx.size(), at.data(), 1, dt); sum += checksum(at);
    std::vector<T> x;
    fill_monotone(x, batch, m, 11);
    std::vector<int32_t> inv((size_t)(batch * m));
    for (int mode = 0; mode < 2; ++mode) {
      oracle_pseudo_inverse(f.data(), n, x.data(), m, inv.data(), batch, mode, dt);
      sum += checksum(inv);
    }
    std::vector<T> outer;
    fill_monotone(outer, batch, k, 6);
    std::vector<int32_t> inner((size_t)(batch * n));
    for (size_t i = 0; i < inner.size(); ++i) inner[i] = (int32_t)(next_u32() % (uint32_t)(k + 4)) - 2;   // some out of range
    int32_t flags = 0;
    oracle_compose(outer.data(), k, inner.data(), n, out.data(), batch, dt, &flags); sum += checksum(out) + flags;
    oracle_gpc_step(f.data(), g.data(), one.data(), out.data(), out2.data(), tmp.data(), 1, n, dt);   // one row
    sum += checksum(out) + checksum(out2);
    oracle_gpc_step(f.data(), g.data(), f.data(), out.data(), out2.data(), tmp.data(), batch, n, dt);
    sum += checksum(out) + checksum(out2);
    oracle_gpc_step_lower(g.data(), f.data(), g.data(), out.data(), out2.data(), tmp.data(), batch, n, dt);
    sum += checksum(out) + checksum(out2);
    if (n <= 24) {
      std::vector<T> scratch((size_t)(3 * n));
      flags = 0;
      oracle_closure(f.data(), out.data(), scratch.data(), batch, n, 0, dt, &flags); sum += checksum(out) + flags;
      oracle_closure(f.data(), out.data(), scratch.data(), batch, n, 1, dt, &flags); sum += checksum(out) + flags;
    }
    std::vector<T> curves, chain((size_t)(batch * n)), line((size_t)n);
    fill_monotone(curves, count * batch, n, 7);
    oracle_conv_chain(curves.data(), count, chain.data(), line.data(), batch, n, dt); sum += checksum(chain);
    std::vector<int32_t> h((size_t)batch);
    std::vector<T> v((size_t)batch);
    flags = 0;
    oracle_max_hdev(f.data(), g.data(), h.data(), batch, n, dt, &flags); sum += checksum(h) + flags;
    oracle_max_vdev(f.data(), g.data(), v.data(), batch, n, dt); sum += checksum(v);
  }
  return sum;
}

}  // namespace

int main() {
  const double a = exercise<int32_t>(0), b = exercise<int64_t>(1), c = exercise<double>(2);
  std::printf("oracle sanitizer run ok: checksums %.6g %.6g %.6g, threads %d, overflow counter %lld\n", a, b, c,
              oracle_num_threads(), oracle_overflow_count(0));
  return 0;
}
