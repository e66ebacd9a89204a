// Exhaustive cross-check of the oracle evaluator against the sequence
// simulator on a tiny DAG.  TEST INFRASTRUCTURE ONLY.
//
// Enumerates every assignment (a, s, e) with C = 2, copy 0 active and
// well-formed, copy 1 either inactive or well-formed, over T = 2n positions,
// evaluates each with orc_eval, and for every assignment without violations
// decodes the rematerialisation sequence (nodes in increasing order of their
// live starts -- Section 1's seq(G) read off the intervals of Section 2) and
// runs bf_simulate on it.  Checked per assignment: the sequence is valid, its
// duration equals the assignment's objective (Eq. (1)), and its minimal
// footprint does not exceed the assignment's peak (Eq. (4) with the intervals
// as given, which may retain longer than needed).
#include <algorithm>
#include <cstdint>
#include <thread>
#include <vector>

extern "C" {
int orc_result_fields();
void orc_eval(int32_t n, const int32_t* in_ptr, const int32_t* in_idx, const int32_t* size,
              const int32_t* dur, int64_t budget, int32_t C, int32_t T, int64_t B,
              const int32_t* starts, const int32_t* ends, const uint8_t* active, int64_t* out);
int bf_simulate(int32_t n, const int32_t* in_ptr, const int32_t* in_idx, const int32_t* size,
                const int32_t* dur, int32_t L, const int32_t* seq, int64_t* peak, int64_t* duration);
}

namespace {

struct State { int32_t s0, e0, s1, e1; uint8_t a1; };

struct Tally {
  int64_t evaluated = 0, clean = 0, bad_decode = 0;
  std::vector<int64_t> min_peak;
};

}  // namespace

extern "C" {

// counts = {assignments evaluated, assignments without violations, failed checks};
// min_peak[mask] = smallest peak over violation-free assignments whose set of
// nodes with an active copy 1 is `mask` (-1 if there is none).  n <= 4.
void orc_exhaustive_c2(int32_t n, const int32_t* in_ptr, const int32_t* in_idx, const int32_t* size,
                       const int32_t* dur, int32_t n_threads, int64_t* counts, int64_t* min_peak) {
  const int C = 2, T = 2 * n, K = 2 * n;
  std::vector<State> states;
  for (int s0 = 0; s0 < T; ++s0)
    for (int e0 = s0; e0 < T; ++e0) {
      states.push_back({s0, e0, 0, 0, 0});
      for (int s1 = 0; s1 < T; ++s1)
        for (int e1 = s1; e1 < T; ++e1) states.push_back({s0, e0, s1, e1, 1});
    }
  const int64_t S = (int64_t)states.size();
  int64_t total = 1;
  for (int v = 0; v < n; ++v) total *= S;
  const int F = orc_result_fields();
  if (n_threads < 1) n_threads = 1;
  std::vector<Tally> tallies(n_threads);
  std::vector<std::thread> pool;
  for (int w = 0; w < n_threads; ++w) {
    pool.emplace_back([&, w]() {
      Tally& t = tallies[w];
      t.min_peak.assign((size_t)1 << n, -1);
      std::vector<int32_t> s(K), e(K), seq;
      std::vector<uint8_t> a(K);
      std::vector<int64_t> res(F);
      std::vector<std::pair<int32_t, int32_t>> ev;
      for (int64_t id = w; id < total; id += n_threads) {
        int64_t rest = id;
        int mask = 0;
        for (int v = 0; v < n; ++v) {
          const State& st = states[rest % S];
          rest /= S;
          s[2 * v] = st.s0; e[2 * v] = st.e0; a[2 * v] = 1;
          s[2 * v + 1] = st.s1; e[2 * v + 1] = st.e1; a[2 * v + 1] = st.a1;
          if (st.a1) mask |= 1 << v;
        }
        orc_eval(n, in_ptr, in_idx, size, dur, INT64_MAX, C, T, 1, s.data(), e.data(), a.data(),
                 res.data());
        ++t.evaluated;
        if (res[2] != 0) continue;   // violations
        ++t.clean;
        ev.clear();
        for (int k = 0; k < K; ++k)
          if (a[k]) ev.push_back({s[k], k / C});
        std::sort(ev.begin(), ev.end());
        seq.clear();
        for (auto& x : ev) seq.push_back(x.second);
        int64_t pk = 0, du = 0;
        const int ok = bf_simulate(n, in_ptr, in_idx, size, dur, (int32_t)seq.size(), seq.data(), &pk, &du);
        if (!ok || du != res[1] || pk > res[0]) ++t.bad_decode;
        if (t.min_peak[mask] < 0 || res[0] < t.min_peak[mask]) t.min_peak[mask] = res[0];
      }
    });
  }
  for (auto& th : pool) th.join();
  counts[0] = counts[1] = counts[2] = 0;
  for (int mk = 0; mk < (1 << n); ++mk) min_peak[mk] = -1;
  for (auto& t : tallies) {
    counts[0] += t.evaluated; counts[1] += t.clean; counts[2] += t.bad_decode;
    for (int mk = 0; mk < (1 << n); ++mk)
      if (t.min_peak[mk] >= 0 && (min_peak[mk] < 0 || t.min_peak[mk] < min_peak[mk]))
        min_peak[mk] = t.min_peak[mk];
  }
}

}  // extern "C"
