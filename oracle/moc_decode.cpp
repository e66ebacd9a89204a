// From an assignment back to a rematerialisation sequence, and that sequence's
// own footprint.  TEST INFRASTRUCTURE ONLY; shares no code with the other
// oracle files nor with the HIP sources.
//
// Section 2 of the paper (arXiv 2304.14463): the start of an active interval
// is the event at which its node is computed, so reading the active copies in
// order of their starts gives the sequence the solution stands for.  Section 1
// (problem statement) says what makes a sequence valid -- every node occurs,
// and the outputs of all predecessors of a node are in memory when it is
// computed -- and what it costs: the summed duration and the peak footprint.
//
// Readings taken here (the paper gives no procedure):
//   - only starts and active flags are read; ends play no part, the footprint
//     is the sequence's own: a use is served by the most recent earlier
//     computation of the producer, and an output is held from the step that
//     computes it through the last step it serves (its own step if none);
//   - two active copies with the same start, or an active copy whose start is
//     outside [0, T), make the assignment undecodable (status -1): Eq. (6) and
//     Eq. (8) forbid both, and no order of the steps follows from them.
//
// Pinned in tests/test_oracle_decode.py against the sequence enumerator of
// moc_bruteforce.cpp (separate code: round trip sequence -> canonical
// assignment -> sequence, and its simulated footprint), against the interval
// evaluator of moc_oracle.cpp (a violation-free assignment decodes to a valid
// sequence of the same duration and no larger footprint), and by hand-counted
// cases.
#include <algorithm>
#include <cstdint>
#include <utility>
#include <vector>

extern "C" {

// One candidate.  s, a: [n*C].  seq: [T], receives the nodes in order, then -1.
// out[4] = status, length, peak, duration.  status 1: a valid sequence; 0: decoded but not
// valid (peak = duration = 0); -1: not decodable (length = peak = duration = 0, seq all -1).
void dec_decode(int32_t n, const int32_t* in_ptr, const int32_t* in_idx, const int32_t* size,
                const int32_t* dur, int32_t C, int32_t T, const int32_t* s, const uint8_t* a,
                int32_t* seq, int64_t* out) {
  const int K = n * C;
  for (int t = 0; t < T; ++t) seq[t] = -1;
  out[0] = -1; out[1] = 0; out[2] = 0; out[3] = 0;

  std::vector<std::pair<int, int>> steps;   // (start, node) of every active copy
  for (int k = 0; k < K; ++k) {
    if (!a[k]) continue;
    if (s[k] < 0 || s[k] >= T) return;
    steps.push_back({s[k], k / C});
  }
  std::sort(steps.begin(), steps.end());
  for (size_t p = 1; p < steps.size(); ++p)
    if (steps[p].first == steps[p - 1].first) return;

  const int L = (int)steps.size();
  for (int p = 0; p < L; ++p) seq[p] = steps[p].second;
  out[0] = 0;
  out[1] = L;

  // validity, and for each step the last step its output serves
  std::vector<int> held_to(L);
  std::vector<char> occurs(n, 0);
  for (int p = 0; p < L; ++p) held_to[p] = p;
  for (int p = 0; p < L; ++p) {
    const int v = seq[p];
    occurs[v] = 1;
    for (int x = in_ptr[v]; x < in_ptr[v + 1]; ++x) {
      int q = p - 1;
      while (q >= 0 && seq[q] != in_idx[x]) --q;
      if (q < 0) return;          // predecessor not computed yet
      held_to[q] = p;             // p only grows
    }
  }
  for (int v = 0; v < n; ++v)
    if (!occurs[v]) return;

  int64_t peak = 0, total = 0;
  for (int p = 0; p < L; ++p) {
    int64_t held = 0;
    for (int q = 0; q <= p; ++q)
      if (held_to[q] >= p) held += size[seq[q]];
    peak = std::max(peak, held);
    total += dur[seq[p]];
  }
  out[0] = 1;
  out[2] = peak;
  out[3] = total;
}

}  // extern "C"
