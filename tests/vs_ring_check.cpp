// Host-side check of the step schedule of the shared-tile Vertical-Slash kernel
// (paper_2407_02490_amd/csrc/vs_ring_sched.h): for seeded run lists, sequence lengths and
// workgroup positions, the four waves' schedules are enumerated and compared with a
// brute-force cover of the slash runs (App. C.4.2: block at q0 may attend key q0 - t for every
// offset t of a run, 0 <= key <= query row).  Built and run by tests/test_sched_host.py.
#include <cstdio>
#include <cstdlib>
#include <vector>

#define MINF_HD
#include "vs_ring_sched.h"

using namespace minf;

struct Fetch {
  const std::vector<int> &r;   // t0, t1 pairs
  bool operator()(int iv, int &a, int &b) const {
    if (iv < 0 || 2 * iv + 1 >= (int)r.size()) return false;
    a = r[2 * iv]; b = r[2 * iv + 1];
    return true;
  }
};

static long long g_steps = 0, g_loads = 0;

static int check_wg(const std::vector<int> &runs, int N, int q0w) {
  std::vector<RStep> s[4];
  for (int w = 0; w < 4; ++w) {
    Fetch f{runs};
    VsRingGen<Fetch> gen(f, q0w, w, N);
    RStep d;
    int guard = 0;
    while (gen.next(d)) {
      s[w].push_back(d);
      if (++guard > 10000000) { printf("FAIL endless schedule\n"); return 1; }
    }
  }
  for (int w = 1; w < 4; ++w)
    if (s[w].size() != s[0].size()) { printf("FAIL step counts differ\n"); return 1; }
  const int T = (int)s[0].size();
  for (int g = 0; g < T; ++g)
    for (int w = 0; w < 4; ++w) {
      const RStep &d = s[w][g];
      if (d.kbase < 0 || d.kbase > N - 32) { printf("FAIL kbase %d out of range\n", d.kbase); return 1; }
      if (d.src < 0 || d.src > w) { printf("FAIL src\n"); return 1; }
      const RStep &l = s[d.src][g];
      if (d.src != w) {
        if (d.load || !l.load || l.src != d.src || l.kbase != d.kbase) {
          printf("FAIL follower/leader mismatch N %d q0w %d g %d wave %d\n", N, q0w, g, w);
          return 1;
        }
      } else if (!d.load && d.work) {
        printf("FAIL a step with work reads rows nobody fetched\n");
        return 1;
      }
      if (d.load) ++g_loads;
      if (d.load || d.src != w) ++g_steps;
    }
  // attended keys per wave against the brute-force cover, for the first and the last row
  for (int w = 0; w < 4; ++w) {
    const int q0 = q0w + 64 * w;
    if (q0 >= N) continue;
    for (int row : {q0, q0 + 31, q0 + 63}) {
      std::vector<int> want(N, 0), got(N, 0);
      for (size_t i = 0; i + 1 < runs.size(); i += 2)
        for (int t = runs[i]; t < runs[i + 1]; ++t) {
          const int key = q0 - t;
          if (key >= 0 && key <= row) want[key] = 1;
        }
      for (int g = 0; g < T; ++g) {
        const RStep &d = s[w][g];
        int n_att = 0;
        for (int key = d.kbase; key < d.kbase + 32; ++key)
          if (key >= d.lo && key < d.hi && key <= row) { ++got[key]; ++n_att; }
        if (!d.work && n_att) { printf("FAIL a step without work attends keys\n"); return 1; }
        if (d.work && !d.mask && n_att != 32) { printf("FAIL unmasked step is not full (row %d)\n", row); return 1; }
        if (d.mask && !d.work) { printf("FAIL mask without work\n"); return 1; }
      }
      for (int key = 0; key < N; ++key)
        if (want[key] != got[key]) {
          printf("FAIL N %d q0w %d wave %d row %d key %d: want %d got %d\n", N, q0w, w, row, key, want[key], got[key]);
          return 1;
        }
    }
    // work means some row attends something
    for (int g = 0; g < T; ++g) {
      const RStep &d = s[w][g];
      bool any = false;
      for (int key = d.kbase; key < d.kbase + 32 && !any; ++key) any = key >= d.lo && key < d.hi && key <= q0 + 63;
      if (any != d.work) { printf("FAIL work flag/emptiness mismatch\n"); return 1; }
    }
  }
  return 0;
}

static unsigned rnd_state = 12345u;
static int rnd(int n) {
  rnd_state = rnd_state * 1664525u + 1013904223u;
  return (int)((rnd_state >> 8) % (unsigned)n);
}

// ascending disjoint runs; kind 0: unions of 64-wide slash tiles (what the builder produces),
// kind 1: arbitrary widths >= 1 (a caller may fill the index itself)
static std::vector<int> make_runs(int N, int n_slash, int kind) {
  std::vector<char> cov(N + 64, 0);
  for (int i = 0; i < n_slash; ++i) {
    const int o = rnd(N), wdt = kind == 0 ? 64 : 1 + rnd(100);
    for (int t = o - wdt + 1; t <= o; ++t) cov[t + 64 < 0 ? 0 : t + 64] = 1;
  }
  std::vector<int> r;
  for (int t = -63; t <= N; ++t) {
    const bool in = t < N && cov[t + 64], prev = t > -63 && cov[t + 63];
    if (in && !prev) r.push_back(t);
    if (!in && prev) r.push_back(t);
  }
  return r;
}

int main() {
  int bad = 0, cases = 0;
  const int Ns[] = {64, 128, 320, 1024, 4160};
  for (int N : Ns)
    for (int kind = 0; kind < 2; ++kind)
      for (int n_slash : {0, 1, 3, 17, 200}) {
        const std::vector<int> runs = make_runs(N, n_slash, kind);
        for (int q0w = 0; q0w < N; q0w += 256) { bad |= check_wg(runs, N, q0w); ++cases; }
      }
  // dense limits and the main diagonal alone
  for (int N : {64, 256, 1088}) {
    bad |= check_wg({-63, N}, N, 0);
    bad |= check_wg({-63, N}, N, (N / 256) * 256 == N ? N - 256 : (N / 256) * 256);
    bad |= check_wg({-63, 1}, N, 0);
    cases += 3;
  }
  printf("%s cases %d steps %lld fetched %lld\n", bad ? "FAIL" : "ok", cases, g_steps, g_loads);
  return bad;
}
