// Step schedule of the shared-tile Vertical-Slash attention kernel.  Plain
// integer arithmetic, compiled for the device and for the host (a test
// enumerates it against a brute-force cover).
//
// A workgroup is four waves = four consecutive 64-row query blocks of one head
// (wave w owns the block whose first row is q0w + 64 w).  A slash run [t0, t1)
// of the head (App. C.4.2: the union of the 64 x 64 tiles of neighbouring kept
// slashes, in offset space t = q0 - key) gives the block at q0 the keys
// (q0 - t1, q0 - t0]: the same key sequence for every block, shifted by the
// block's first row.  All four waves therefore walk ONE common schedule of
// 32-key steps (run r, step j), wave w's step starting at key
//     q0w - t1 + 1 + 64 w + 32 j,
// and wave w runs the schedule two steps behind wave w - 1.  At any moment the
// waves that are inside the same run then need the same 32 keys: wave w's step
// (r, j) is wave (w-1)'s step (r, j + 2).  Only the first wave of such a group
// (the "leader": the one whose predecessor has already left the run) fetches
// the keys, into its own ring in LDS; the others read that ring.  A run of n
// steps is fetched n + 6 times per workgroup instead of 4 n times.
//
// Every wave yields the same number of steps (2 w idle steps first, 6 - 2 w idle
// steps last), so the four waves can meet at a barrier every step.
#ifndef MINF_VS_RING_SCHED_H_
#define MINF_VS_RING_SCHED_H_

#ifndef MINF_HD
#define MINF_HD __host__ __device__
#endif

namespace minf {

// One 32-key step of a wave.  Keys kbase .. kbase+31 are the rows held in LDS
// (kbase is clamped into [0, N - 32]); the wave attends key j of them iff
// lo <= j < hi and j <= query row.  work: some element is attended (else the wave
// still runs the step, with P = 0); mask: some element of a step with work is not
// attended (the element mask must be applied).  src: the wave whose ring holds
// the rows; load: this wave fetches them.
struct RStep {
  int kbase, lo, hi, src;
  bool work, mask, load;
};

// RunFetch: bool operator()(int iv, int &t0, int &t1) -- run iv of the head, false past the last.
template <class RunFetch>
struct VsRingGen {
  RunFetch &fetch;
  int q0w, wave, N;        // first row of wave 0's block; this wave; sequence length
  int lead, tail;          // idle steps still to yield before / after the schedule
  int iv, j, n, t0, t1;    // next run; next step of the current run and its step count
  bool ended;

  MINF_HD VsRingGen(RunFetch &f, int q0w_, int wave_, int N_)
      : fetch(f), q0w(q0w_), wave(wave_), N(N_), lead(2 * wave_), tail(6 - 2 * wave_), iv(0), j(0), n(0),
        t0(0), t1(0), ended(false) {}

  MINF_HD void idle(RStep &d) const {
    d.kbase = 0; d.lo = 0; d.hi = 0; d.src = wave; d.work = false; d.mask = false; d.load = false;
  }

  MINF_HD bool next(RStep &d) {
    if (lead > 0) { --lead; idle(d); return true; }
    while (j >= n) {
      if (!ended) {
        int a, b;
        // runs ascend; the last wave's block (first row q0w + 192) reaches the furthest back
        if (fetch(iv, a, b) && a <= q0w + 192) {
          ++iv;
          t0 = a; t1 = b;
          n = (t1 - t0 + 31) >> 5;
          // first step that holds a key >= 0 for the last wave (earlier ones are empty for all four)
          const int x = t1 - q0w - 224;
          j = x > 0 ? (x + 31) >> 5 : 0;
          continue;
        }
        ended = true;
      }
      if (tail > 0) { --tail; idle(d); return true; }
      return false;
    }
    const int q0 = q0w + 64 * wave;
    const int kb = q0 - t1 + 1 + 32 * j;              // first key of the step (may lie outside [0, N))
    const int ks = q0 - t1 + 1 > 0 ? q0 - t1 + 1 : 0;
    const int ke = q0 - t0 + 1 < N ? q0 - t0 + 1 : N;
    d.lo = kb > ks ? kb : ks;
    d.hi = kb + 32 < ke ? kb + 32 : ke;
    d.kbase = kb < 0 ? 0 : (kb > N - 32 ? N - 32 : kb);
    // the wave ahead is two steps further into the same run, if the run is that long
    const int ahead = (n - 1 - j) >> 1;
    const int f = wave < ahead ? wave : ahead;
    d.src = wave - f;
    d.load = f == 0;
    d.work = d.lo < d.hi && d.lo <= q0 + 63;
    d.mask = d.work && !(d.kbase == kb && d.lo == kb && d.hi == kb + 32 && kb + 31 <= q0);
    ++j;
    return true;
  }
};

}  // namespace minf
#endif
