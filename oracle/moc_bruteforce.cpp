// Brute force over rematerialisation sequences, with an independent liveness
// simulation.  TEST INFRASTRUCTURE ONLY; it exists to pin moc_oracle.cpp and
// shares no code with it (nor with the HIP sources).
//
// It works on the problem as stated in Section 1 of the paper (arXiv
// 2304.14463): a rematerialisation sequence is an ordered list of nodes that
// contains every node at least once; the outputs of all predecessors of a
// node must be in memory when it is computed; the cost is the summed duration
// and the constraint is on the peak memory footprint.  Here a node may occur
// at most C times (Section 2, parameter C_v).
//
// Liveness rule used to give a sequence its (minimal) footprint: every use of
// an output is served by the most recent earlier computation of the producer,
// and each computation is kept from its own step through the last use it
// serves (its own step only, if it serves none).  The footprint of a step
// counts the output being computed and everything kept across that step --
// the paper's example: recomputing node 1 while node 3's output is retained
// costs m_1 + m_3 (Section 2, paragraph on compute events).
#include <cstdint>
#include <vector>

namespace {

struct Dag {
  int n;
  const int32_t* in_ptr;
  const int32_t* in_idx;
  const int32_t* size;
  const int32_t* dur;
};

// Simulate a sequence.  Returns false if a node is used before any computation
// of one of its predecessors, or some node never occurs.  keep_until[p] = last
// step served by the computation at step p.
bool simulate(const Dag& g, const std::vector<int>& seq, int64_t* peak, int64_t* duration,
              std::vector<int>* keep_until_out) {
  const int L = (int)seq.size();
  std::vector<int> latest(g.n, -1);   // step of the most recent computation of each node
  std::vector<int> keep_until(L);
  *duration = 0;
  for (int p = 0; p < L; ++p) {
    const int v = seq[p];
    for (int q = g.in_ptr[v]; q < g.in_ptr[v + 1]; ++q) {
      const int u = g.in_idx[q];
      if (latest[u] < 0) return false;
      keep_until[latest[u]] = p;      // steps increase, so this is the last use so far
    }
    latest[v] = p;
    keep_until[p] = p;
    *duration += g.dur[v];
  }
  for (int v = 0; v < g.n; ++v)
    if (latest[v] < 0) return false;
  int64_t worst = 0;
  for (int p = 0; p < L; ++p) {
    int64_t in_use = 0;
    for (int q = 0; q <= p; ++q)
      if (keep_until[q] >= p) in_use += g.size[seq[q]];
    if (in_use > worst) worst = in_use;
  }
  *peak = worst;
  if (keep_until_out) *keep_until_out = keep_until;
  return true;
}

struct Enumerator {
  Dag g;
  int C;
  int max_len;
  int64_t cap;
  int64_t count = 0;
  std::vector<int> seq, times;
  int32_t* seq_len;
  int32_t* seqs;
  int64_t* peak;
  int64_t* duration;
  int32_t* s;
  int32_t* e;
  uint8_t* a;

  void emit() {
    int64_t pk, du;
    std::vector<int> keep;
    if (!simulate(g, seq, &pk, &du, &keep)) return;
    if (count < cap) {
      const int K = g.n * C;
      seq_len[count] = (int32_t)seq.size();
      for (int p = 0; p < K; ++p) seqs[count * K + p] = p < (int)seq.size() ? seq[p] : -1;
      peak[count] = pk;
      duration[count] = du;
      // canonical candidate: the i-th occurrence of v at step p is copy i = [p, keep[p]]
      for (int k = 0; k < K; ++k) { s[count * K + k] = 0; e[count * K + k] = 0; a[count * K + k] = 0; }
      std::vector<int> seen(g.n, 0);
      for (int p = 0; p < (int)seq.size(); ++p) {
        const int k = seq[p] * C + seen[seq[p]]++;
        s[count * K + k] = p;
        e[count * K + k] = keep[p];
        a[count * K + k] = 1;
      }
    }
    ++count;
  }

  void extend(int distinct) {
    if (distinct == g.n) emit();
    if ((int)seq.size() == max_len) return;
    for (int v = 0; v < g.n; ++v) {
      if (times[v] == C) continue;
      bool ready = true;
      for (int q = g.in_ptr[v]; q < g.in_ptr[v + 1]; ++q)
        if (times[g.in_idx[q]] == 0) ready = false;
      if (!ready) continue;
      ++times[v];
      seq.push_back(v);
      extend(distinct + (times[v] == 1));
      seq.pop_back();
      --times[v];
    }
  }
};

}  // namespace

extern "C" {

// Simulate one sequence of length L.  Returns 1 and fills peak/duration if it
// is a valid rematerialisation sequence, 0 otherwise.
int bf_simulate(int32_t n, const int32_t* in_ptr, const int32_t* in_idx, const int32_t* size,
                const int32_t* dur, int32_t L, const int32_t* seq, int64_t* peak, int64_t* duration) {
  Dag g{n, in_ptr, in_idx, size, dur};
  std::vector<int> sq(seq, seq + L);
  for (int x : sq)
    if (x < 0 || x >= n) return 0;
  return simulate(g, sq, peak, duration, nullptr) ? 1 : 0;
}

// Enumerate every valid sequence with at most C occurrences per node and
// length <= n + max_extra.  For each (up to cap) writes its length, the
// sequence (padded with -1 to n*C), its simulated peak and duration and its
// canonical candidate (s, e, a as [n*C]).  Returns the number of sequences.
int64_t bf_enumerate(int32_t n, const int32_t* in_ptr, const int32_t* in_idx, const int32_t* size,
                     const int32_t* dur, int32_t C, int32_t max_extra, int64_t cap, int32_t* seq_len,
                     int32_t* seqs, int64_t* peak, int64_t* duration, int32_t* s, int32_t* e,
                     uint8_t* a) {
  Enumerator en;
  en.g = Dag{n, in_ptr, in_idx, size, dur};
  en.C = C;
  en.max_len = n + max_extra < n * C ? n + max_extra : n * C;
  en.cap = cap;
  en.times.assign(n, 0);
  en.seq_len = seq_len; en.seqs = seqs; en.peak = peak; en.duration = duration;
  en.s = s; en.e = e; en.a = a;
  en.extend(0);
  return en.count;
}

}  // extern "C"
