// Host-side check of the workgroup -> (head slot, query block) mapping: for a list of head
// lists, K/V group sizes and block counts, every hardware workgroup id of the launch is decoded
// and every (slot, block) pair must come out exactly once.  Built and run by
// tests/test_sched_host.py (no GPU needed: the mapping is plain integer arithmetic).
#include <cstdio>
#include <cstring>
#include <vector>

#include "minf_internal.h"

using namespace minf;

static int check(const std::vector<int> &heads, int group, int n_blk) {
  HeadList hl;
  memset(&hl, 0, sizeof(hl));
  hl.n = (int)heads.size();
  for (int i = 0; i < hl.n; ++i) hl.h[i] = heads[i];
  const Sched s = make_sched(hl, group, n_blk);
  std::vector<int> seen((size_t)hl.n * n_blk, 0);
  long long items = 0;
  for (int hw = 0; hw < s.per_xcd * 8; ++hw) {
    int slot = -1, blk = -1;
    if (!decode_item(s, hw, slot, blk)) continue;
    if (slot < 0 || slot >= hl.n || blk < 0 || blk >= n_blk) {
      printf("FAIL out of range: hw %d -> slot %d blk %d\n", hw, slot, blk);
      return 1;
    }
    ++seen[(size_t)slot * n_blk + blk];
    ++items;
  }
  for (size_t i = 0; i < seen.size(); ++i)
    if (seen[i] != 1) {
      printf("FAIL heads %d group %d n_blk %d: item %zu seen %d times\n", hl.n, group, n_blk, i, seen[i]);
      return 1;
    }
  // chunks never mix K/V heads and never exceed the cap
  for (int i = 0; i < hl.n; ++i) {
    const int c0 = s.cstart[i], cs = s.csize[i];
    if (cs < 1 || cs > SCHED_MAX_CHUNK || i < c0 || i >= c0 + cs || hl.h[c0] / group != hl.h[i] / group) {
      printf("FAIL chunk of slot %d\n", i);
      return 1;
    }
  }
  printf("ok heads %d group %d n_blk %d items %lld grid %d\n", hl.n, group, n_blk, items, s.per_xcd * 8);
  return 0;
}

int main() {
  int bad = 0;
  const int blocks[] = {1, 2, 7, 8, 9, 63, 64, 65, 513, 2048, 16384};
  for (int nb : blocks) {
    bad |= check({0}, 4, nb);
    bad |= check({0, 1, 2, 3}, 4, nb);
    bad |= check({0, 1, 2, 4, 5, 6, 7, 9, 13}, 4, nb);
    bad |= check({5, 1, 12, 3}, 8, nb);
    bad |= check({0, 1, 2, 3, 4, 5, 6, 7, 8, 9, 10, 11, 12, 13, 14, 15, 16}, 16, nb);
  }
  std::vector<int> all;
  for (int i = 0; i < MINF_MAX_HEADS; ++i) all.push_back(i);
  bad |= check(all, 4, 300);
  bad |= check(all, 1, 33);
  return bad;
}
