// Host-side brute-force check of the stream share map used by the attention kernels:
// shares tile the stream, none is empty when there are at least as many blocks as
// wavefronts, and share_owner inverts share_start.
// Compiled and run by tests/test_share_map.py (host code only, no GPU).
#include "pkv_kernels.h"
#include <cstdio>
int main() {
  using namespace pkv;
  long bad = 0;
  for (int64_t T : {1LL, 5LL, 2047LL, 2048LL, 2049LL, 4095LL, 4096LL, 4097LL, 31744LL, 147520LL,
                    494040LL, 1000003LL, 2147483647LL}) {
    const int64_t W = T < kStreamWaves ? T : kStreamWaves;   // as both kernels choose it
    if (share_start(0, T, W) != 0 || share_start(W, T, W) != T) { printf("T=%lld ends wrong\n", (long long)T); bad++; }
    int64_t minlen = (int64_t)1 << 40, maxlen = 0;
    for (int64_t w = 0; w < W; ++w) {
      const int64_t a = share_start(w, T, W), b = share_start(w + 1, T, W);
      if (b - a < minlen) minlen = b - a;
      if (b - a > maxlen) maxlen = b - a;
      if (b <= a) { bad++; continue; }
      if (share_owner(a, T, W) != w || share_owner(b - 1, T, W) != w) {
        if (bad < 10) printf("T=%lld w=%lld owner mismatch %d %d\n", (long long)T, (long long)w,
                             share_owner(a, T, W), share_owner(b - 1, T, W));
        bad++;
      }
    }
    printf("T=%lld W=%lld share len %lld..%lld\n", (long long)T, (long long)W, (long long)minlen, (long long)maxlen);
    if (maxlen - minlen > 1) bad++;
  }
  printf("bad=%ld\n", bad);
  return bad != 0;
}
