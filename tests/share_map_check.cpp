// Host-side brute-force check of the stream share map used by the attention kernels:
// shares tile the stream, none is empty when there are at least as many blocks as
// wavefronts, and share_owner inverts share_start.
// Then the record slots: walking every wavefront's share block by block (as the
// stream pass does), slot = segment + wavefront is unique, stays below the bound
// the workspace is sized for, and the slots of a segment are exactly the range
// the merge pass computes from the owners of its first and last block.
// Compiled and run by tests/test_share_map.py (host code only, no GPU).
#include "pkv_kernels.h"
#include <cstdio>
#include <set>
#include <vector>

static long check_slots(const std::vector<int>& nblk, int Hkv) {
  using namespace pkv;
  const int S = (int)nblk.size();
  std::vector<int64_t> cumB(S + 1, 0);
  for (int s = 0; s < S; ++s) cumB[s + 1] = cumB[s] + nblk[s];
  const int64_t T = (int64_t)Hkv * cumB[S];
  if (T == 0) return 0;
  const int64_t W = T < kStreamWaves ? T : kStreamWaves;
  long bad = 0;
  std::set<int64_t> used;
  std::vector<std::set<int64_t>> of_seg((size_t)S * Hkv);
  for (int64_t w = 0; w < W; ++w) {
    int64_t prev_seg = -1;
    for (int64_t pos = share_start(w, T, W); pos < share_start(w + 1, T, W); ++pos) {
      int s = 0;
      while (!((int64_t)Hkv * cumB[s] <= pos && pos < (int64_t)Hkv * cumB[s + 1])) ++s;
      const int kvh = (int)((pos - Hkv * cumB[s]) / nblk[s]);
      const int64_t seg = (int64_t)s * Hkv + kvh;
      if (seg == prev_seg) continue;
      prev_seg = seg;
      const int64_t slot = seg + w;
      if (!used.insert(slot).second) bad++;          // two (wavefront, segment) pairs share a slot
      if (slot >= (int64_t)S * Hkv + kStreamWaves) bad++;
      of_seg[(size_t)seg].insert(slot);
    }
  }
  for (int s = 0; s < S; ++s)
    for (int kvh = 0; kvh < Hkv; ++kvh) {
      const int64_t seg = (int64_t)s * Hkv + kvh;
      if (nblk[s] == 0) { if (!of_seg[(size_t)seg].empty()) bad++; continue; }
      const int64_t pos_a = (int64_t)Hkv * cumB[s] + (int64_t)kvh * nblk[s];
      const int64_t first = seg + share_owner(pos_a, T, W);
      const int64_t last = seg + share_owner(pos_a + nblk[s] - 1, T, W);
      std::set<int64_t> want;
      for (int64_t x = first; x <= last; ++x) want.insert(x);
      if (want != of_seg[(size_t)seg]) bad++;
    }
  return bad;
}

int main() {
  using namespace pkv;
  long bad = 0;
  {
    // seeded batches: short, empty and long requests mixed, several head counts
    uint64_t x = 20260211;
    auto rnd = [&]() { x = x * 6364136223846793005ULL + 1442695040888963407ULL; return (uint32_t)(x >> 33); };
    long slot_bad = 0;
    for (int trial = 0; trial < 24; ++trial) {
      const int S = 1 + (int)(rnd() % 97);
      const int Hkv = 1 + (int)(rnd() % 8);
      std::vector<int> nblk(S);
      for (int s = 0; s < S; ++s) {
        const uint32_t k = rnd() % 8;
        nblk[s] = k == 0 ? 0 : k < 4 ? 1 + (int)(rnd() % 4) : k < 7 ? 1 + (int)(rnd() % 200) : 1 + (int)(rnd() % 2048);
      }
      slot_bad += check_slots(nblk, Hkv);
    }
    slot_bad += check_slots(std::vector<int>(64, 32), 8);      // shares and segments end together
    slot_bad += check_slots(std::vector<int>(2048, 1), 1);     // one block per wavefront
    slot_bad += check_slots(std::vector<int>(3, 1), 2);        // fewer blocks than wavefronts
    printf("slot check bad=%ld\n", slot_bad);
    bad += slot_bad;
  }
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
