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

// Two head lists in one launch (decode_mixed): every item of both lists exactly once, the XCD of an
// item (low three bits of its position in its own launch order) equal to the XCD of the workgroup id.
static int check_mixed(const std::vector<int> &ha, const std::vector<int> &hb, int group, int n_blk) {
  HeadList la, lb;
  memset(&la, 0, sizeof(la));
  memset(&lb, 0, sizeof(lb));
  la.n = (int)ha.size();
  lb.n = (int)hb.size();
  for (int i = 0; i < la.n; ++i) la.h[i] = ha[i];
  for (int i = 0; i < lb.n; ++i) lb.h[i] = hb[i];
  const Sched sa = make_sched(la, group, n_blk), sb = make_sched(lb, group, n_blk);
  std::vector<int> seen_a((size_t)la.n * n_blk, 0), seen_b((size_t)lb.n * n_blk, 0);
  const int grid = 40 * mixed_groups(sa, sb);
  int run_a = 0, worst_a = 0;
  for (int w = 0; w < grid; ++w) {
    int kind = -1, slot = -1, blk = -1;
    const bool has = decode_mixed(sa, sb, w, kind, slot, blk);
    if (kind == 0) { ++run_a; if (run_a > worst_a) worst_a = run_a; } else run_a = 0;
    if (!has) continue;
    const int n = kind == 0 ? la.n : lb.n;
    if (kind < 0 || kind > 1 || slot < 0 || slot >= n || blk < 0 || blk >= n_blk) {
      printf("FAIL mixed out of range: w %d -> kind %d slot %d blk %d\n", w, kind, slot, blk);
      return 1;
    }
    ++(kind == 0 ? seen_a : seen_b)[(size_t)slot * n_blk + blk];
  }
  for (size_t i = 0; i < seen_a.size(); ++i)
    if (seen_a[i] != 1) { printf("FAIL mixed: first list item %zu seen %d times\n", i, seen_a[i]); return 1; }
  for (size_t i = 0; i < seen_b.size(); ++i)
    if (seen_b[i] != 1) { printf("FAIL mixed: second list item %zu seen %d times\n", i, seen_b[i]); return 1; }
  if (worst_a > 32) { printf("FAIL mixed: %d ids of the first kind in a row\n", worst_a); return 1; }
  printf("ok mixed heads %d + %d n_blk %d grid %d\n", la.n, lb.n, n_blk, grid);
  return 0;
}

int main() {
  int bad = 0;
  for (int nb : {1, 7, 64, 513, 16384}) {
    bad |= check_mixed({0, 1, 2, 4, 5, 6}, {3, 7}, 4, nb);
    bad |= check_mixed({9}, {0, 1, 2, 3, 4, 5, 6, 7, 8}, 4, nb);
    bad |= check_mixed({0, 1, 2, 4, 5, 6, 8, 9, 10, 12, 13, 14, 16, 17, 18, 20, 21, 22, 24, 25, 26, 28, 29, 30},
                       {3, 7, 11, 15, 19, 23}, 4, nb);
  }
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
