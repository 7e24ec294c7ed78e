// Host-side check of the multiply-shift division that the launchers prepare for the kernels'
// item -> (segment, head, block) mapping: fast_div / fast_mod must equal n / d and n % d for every
// 0 <= n < 2^31 and every divisor the launchers can produce.  Prints "ok <cases>" or the first
// mismatch.  Pure host code: needs no GPU.
#include <cstdio>
#include <cstdlib>

#include "segattn_internal.h"

int main() {
  using namespace segattn;
  unsigned long long state = 0x9e3779b97f4a7c15ull;
  auto rnd = [&]() {
    state ^= state << 13;
    state ^= state >> 7;
    state ^= state << 17;
    return state;
  };
  long long cases = 0;
  auto check = [&](long long d) {
    const FastDiv f = fast_div_by(d);
    if (f.d == 0) {
      printf("divisor %lld rejected\n", d);
      exit(1);
    }
    const long long probes[] = {0, 1, d - 1, d, d + 1, 2 * d - 1, 2 * d, 3 * d + 1, (1ll << 31) - 1, (1ll << 31) - 2,
                                (1ll << 30), (1ll << 30) - 1};
    auto one = [&](long long n) {
      if (n < 0 || n >= (1ll << 31)) return;
      const int q = fast_div((int)n, f), r = fast_mod((int)n, f);
      if (q != (int)(n / d) || r != (int)(n % d)) {
        printf("mismatch: %lld / %lld = %d rem %d\n", n, d, q, r);
        exit(1);
      }
      ++cases;
    };
    for (long long n : probes) one(n);
    for (int i = 0; i < 64; ++i) one((long long)(rnd() % (1ull << 31)));
    // multiples of d near the top of the range, where the product mul * n is largest
    const long long top = ((1ll << 31) - 1) / d;
    for (long long k = top; k >= 0 && k > top - 4; --k) {
      one(k * d);
      one(k * d + d - 1);
      one(k * d - 1);
    }
  };
  for (long long d = 1; d <= 70000; ++d) check(d);
  for (int s = 1; s < 31; ++s)
    for (long long e = -2; e <= 2; ++e) {
      const long long d = (1ll << s) + e;
      if (d >= 1 && d < (1ll << 31)) check(d);
    }
  for (int i = 0; i < 200000; ++i) check((long long)(rnd() % ((1ull << 31) - 1)) + 1);
  if (fast_div_by(0).d != 0 || fast_div_by(1ll << 31).d != 0 || fast_div_by(-3).d != 0) {
    printf("an unusable divisor was accepted\n");
    return 1;
  }
  printf("ok %lld\n", cases);
  return 0;
}
