// CPU oracle for the batched candidate evaluator.  TEST INFRASTRUCTURE ONLY:
// it is what the HIP library is checked against, it is never on the product
// path, and it shares no code with the HIP sources.
//
// It evaluates the retention-interval model of Moccasin (arXiv 2304.14463,
// Section 2.1, Eq. (1)-(8)) on a given assignment of the variables
// (a, s, e) -- the plain definitions written out, single-threaded, int64.
//
// Notation: node v in [0,n), copy i in [0,C), copy index k = v*C + i,
// positions (the paper's event domain D, Eq. (8) and the display after it,
// shifted to 0-based) t in [0,T).  T is an explicit argument so that the
// worked example of Section 2 (drawn on 10 events for 4 nodes x 2 copies)
// can be evaluated as printed; the HIP library always uses T = n*C.
//
// Readings taken where the paper leaves a choice (all listed in the design
// notes): an inactive copy is ignored by every constraint (Section 2.1, first
// paragraph); intervals are closed, [s, e] (Eq. (4)); precedence is Eq. (5)
// literally, s_u + 1 <= s_v <= e_u; "all starts different" (Eq. (6) and the
// sentence after Eq. (8) on it) covers all live copies, same node included;
// an active copy with s > e or a position outside [0,T) is malformed: it is
// one violation of Eq. (2)/(8), is skipped by everything else, and still
// counts in the objective (Eq. (1) depends on a only).
//
// Parity pins (tests/test_oracle_*.py): the worked example's printed values,
// hand-counted single-violation cases, closed forms, exhaustive enumeration
// of rematerialisation sequences on tiny DAGs against an independent liveness
// simulation (moc_bruteforce.cpp), the no-remat liveness invariant.  The
// neighbourhood scorer re-evaluates every move through the pinned evaluator;
// its numbering of the moves, the rule for moves that do not apply and the
// order of the best move are pinned on hand-counted cases and against
// candidates edited by the test itself (tests/test_oracle_neighbours.py, as
// is the descent by such moves put together in oracle/__init__.py); the move
// set itself is this library's, not the paper's.
#include <cstdint>
#include <cstring>
#include <vector>

namespace {

struct Problem {
  int32_t n;
  const int32_t* in_ptr;  // [n+1] predecessors of v: in_idx[in_ptr[v] .. in_ptr[v+1])
  const int32_t* in_idx;  // [m]
  const int32_t* size;    // [n]  m_v
  const int32_t* dur;     // [n]  w_v
  int64_t budget;         // M
  int32_t C;
  int32_t T;
};

// fields of one result row (int64 each)
enum { R_PEAK, R_DURATION, R_VIOLATIONS, R_FEASIBLE, R_FORM, R_FIRST, R_ORDER, R_START, R_PREC, R_FIELDS };

struct Scratch {
  std::vector<char> live;
  std::vector<int64_t> profile;
  std::vector<int32_t> cnt;
};

// Eq. (2) and the domain of Eq. (8): an active copy is usable iff 0 <= s <= e <= T-1.
inline bool well_formed(const Problem& p, int32_t s, int32_t e, uint8_t a) {
  return a != 0 && 0 <= s && s <= e && e <= p.T - 1;
}

// in_domain (may be null: every position of [0,T) is allowed): per copy, whether its start is a
// value the variable may take at all (Section 2.3 restricts the starts to particular events).
// A start outside its domain is treated like one outside [0,T): the copy is not usable.
void evaluate(const Problem& p, const int32_t* s, const int32_t* e, const uint8_t* a, Scratch& w,
              int64_t* out, int64_t* profile_out, const char* in_domain = nullptr) {
  const int K = p.n * p.C;
  w.live.assign(K, 0);
  int64_t v_form = 0, v_first = 0, v_order = 0, v_start = 0, v_prec = 0, duration = 0;

  for (int k = 0; k < K; ++k) {
    w.live[k] = well_formed(p, s[k], e[k], a[k]) && (!in_domain || in_domain[k]);
    if (a[k] != 0 && !w.live[k]) ++v_form;          // Eq. (2), Eq. (8)
    if (a[k] != 0) duration += p.dur[k / p.C];      // Eq. (1)
  }
  for (int v = 0; v < p.n; ++v)
    if (a[v * p.C] == 0) ++v_first;                 // Eq. (7)

  // Eq. (3): a live copy must end no later than the next live copy of its node starts.
  for (int v = 0; v < p.n; ++v)
    for (int i = 0; i < p.C; ++i) {
      if (!w.live[v * p.C + i]) continue;
      for (int j = i + 1; j < p.C; ++j)
        if (w.live[v * p.C + j]) {
          if (e[v * p.C + i] > s[v * p.C + j]) ++v_order;
          break;
        }
    }

  // Eq. (6): compute events do not coincide.
  w.cnt.assign(p.T > 0 ? p.T : 0, 0);
  for (int k = 0; k < K; ++k)
    if (w.live[k]) ++w.cnt[s[k]];
  for (int t = 0; t < p.T; ++t)
    if (w.cnt[t] > 1) v_start += w.cnt[t] - 1;

  // Eq. (5): every input of every live copy is covered by a live copy of the producer.
  for (int v = 0; v < p.n; ++v)
    for (int q = p.in_ptr[v]; q < p.in_ptr[v + 1]; ++q) {
      const int u = p.in_idx[q];
      for (int i = 0; i < p.C; ++i) {
        if (!w.live[v * p.C + i]) continue;
        const int64_t sv = s[v * p.C + i];
        bool covered = false;
        for (int j = 0; j < p.C; ++j) {
          const int ku = u * p.C + j;
          if (w.live[ku] && (int64_t)s[ku] + 1 <= sv && sv <= (int64_t)e[ku]) covered = true;
        }
        if (!covered) ++v_prec;
      }
    }

  // Eq. (4): memory in use at every position, closed intervals; peak = max over positions.
  w.profile.assign(p.T > 0 ? p.T : 0, 0);
  for (int k = 0; k < K; ++k)
    if (w.live[k])
      for (int t = s[k]; t <= e[k]; ++t) w.profile[t] += p.size[k / p.C];
  int64_t peak = 0;
  for (int t = 0; t < p.T; ++t)
    if (w.profile[t] > peak) peak = w.profile[t];
  if (profile_out)
    for (int t = 0; t < p.T; ++t) profile_out[t] = w.profile[t];

  const int64_t violations = v_form + v_first + v_order + v_start + v_prec;
  out[R_PEAK] = peak;
  out[R_DURATION] = duration;
  out[R_VIOLATIONS] = violations;
  out[R_FEASIBLE] = (violations == 0 && peak <= p.budget) ? 1 : 0;
  out[R_FORM] = v_form;
  out[R_FIRST] = v_first;
  out[R_ORDER] = v_order;
  out[R_START] = v_start;
  out[R_PREC] = v_prec;
}

}  // namespace

extern "C" {

int orc_result_fields() { return R_FIELDS; }

// Evaluate B candidates; starts/ends/active are [B][n*C]; out is [B][R_FIELDS] int64.
void orc_eval(int32_t n, const int32_t* in_ptr, const int32_t* in_idx, const int32_t* size,
              const int32_t* dur, int64_t budget, int32_t C, int32_t T, int64_t B,
              const int32_t* starts, const int32_t* ends, const uint8_t* active, int64_t* out) {
  Problem p{n, in_ptr, in_idx, size, dur, budget, C, T};
  Scratch w;
  const int64_t K = (int64_t)n * C;
  for (int64_t b = 0; b < B; ++b)
    evaluate(p, starts + b * K, ends + b * K, active + b * K, w, out + b * R_FIELDS, nullptr);
}

// One candidate; also returns the memory profile (Eq. (4) left-hand side) per position.
void orc_profile(int32_t n, const int32_t* in_ptr, const int32_t* in_idx, const int32_t* size,
                 const int32_t* dur, int64_t budget, int32_t C, int32_t T, const int32_t* starts,
                 const int32_t* ends, const uint8_t* active, int64_t* out, int64_t* profile) {
  Problem p{n, in_ptr, in_idx, size, dur, budget, C, T};
  Scratch w;
  evaluate(p, starts, ends, active, w, out, profile);
}

// Stage-restricted domain (Section 2.3, "Complexity Reduction by Enforcing an Initial
// Topological Ordering").  Events are grouped into n stages, stage j (0-based) holding the
// j + 1 positions j(j+1)/2 .. j(j+1)/2 + j, so that the domain has n(n+1)/2 positions.  With
// index[v] = k the place of node v in the given topological order, v may be computed only at
// event k of a stage (0-based slot k, which exists in stages j >= k), and its first interval
// starts at slot k of stage k, the last position of that stage: a fixed value, not a variable.
// Readings: a start that is not one of these values is outside the variable's domain, as a
// position outside [0,T) is in the plain model: the copy counts as one violation of Eq. (8),
// takes part in nothing else and still counts in Eq. (1).  Ends may be any position of the
// domain.  Eq. (6) is kept as it is evaluated elsewhere (copies of one node can still share
// an event); everything else is Eq. (1)-(8) on T = n(n+1)/2 positions.
static int stage_of(int64_t pos) {   // the stage whose positions include pos >= 0
  int j = 0;
  while ((int64_t)(j + 1) * (j + 2) / 2 <= pos) ++j;
  return j;
}

// Evaluate B candidates in the stage-restricted domain; index[v] in [0,n) is a permutation that
// orders the nodes topologically.  starts/ends/active are [B][n*C]; out is [B][R_FIELDS].
void orc_eval_staged(int32_t n, const int32_t* in_ptr, const int32_t* in_idx, const int32_t* size,
                     const int32_t* dur, int64_t budget, int32_t C, const int32_t* index, int64_t B,
                     const int32_t* starts, const int32_t* ends, const uint8_t* active, int64_t* out) {
  const int64_t D = (int64_t)n * (n + 1) / 2;
  Problem p{n, in_ptr, in_idx, size, dur, budget, C, (int32_t)D};
  Scratch w;
  const int64_t K = (int64_t)n * C;
  std::vector<char> in_domain(K);
  for (int64_t b = 0; b < B; ++b) {
    const int32_t* s = starts + b * K;
    for (int v = 0; v < n; ++v)
      for (int i = 0; i < C; ++i) {
        const int64_t pos = s[v * C + i];
        bool ok = false;
        if (pos >= 0 && pos < D) {
          const int j = stage_of(pos);
          const int64_t slot = pos - (int64_t)j * (j + 1) / 2;
          ok = slot == index[v] && (i > 0 || j == index[v]);
        }
        in_domain[v * C + i] = ok;
      }
    evaluate(p, s, ends + b * K, active + b * K, w, out + b * R_FIELDS, nullptr, in_domain.data());
  }
}

// Neighbourhood of one candidate by full re-evaluation.  Move index
// q = ((k*2 + field)*2R + d), field 0 = start, 1 = end, delta = d-R for d < R,
// d-R+1 otherwise (so delta runs -R..-1, +1..+R).  A move is not applicable if
// the copy is inactive or the moved field would leave [0,T): score (-1,-1).
// Otherwise the score is (violations, peak) of the candidate with that one
// field changed.  n_moves == 0: score every move, moves == NULL; else score
// only the listed move indices.  scores is [count][2] int64.
// best (may be NULL) receives {move, violations, peak} of the applicable move
// that minimises (violations, max(peak, M), peak, q) lexicographically -- the
// Phase-1 objective of Section 2.4 as tie-break after the violation count --
// over the moves scored by this call; move = -1 if none was applicable.
void orc_neighbours(int32_t n, const int32_t* in_ptr, const int32_t* in_idx, const int32_t* size,
                    const int32_t* dur, int64_t budget, int32_t C, int32_t T, const int32_t* starts,
                    const int32_t* ends, const uint8_t* active, int32_t R, int64_t n_moves,
                    const int64_t* moves, int64_t* scores, int64_t* best) {
  Problem p{n, in_ptr, in_idx, size, dur, budget, C, T};
  Scratch w;
  const int K = n * C;
  std::vector<int32_t> s(starts, starts + K), e(ends, ends + K);
  const int64_t total = (int64_t)K * 4 * R;
  const int64_t count = n_moves ? n_moves : total;
  int64_t best_move = -1, best_v = 0, best_peak = 0;
  int64_t res[R_FIELDS];
  for (int64_t idx = 0; idx < count; ++idx) {
    const int64_t q = n_moves ? moves[idx] : idx;
    const int d = (int)(q % (2 * R));
    const int field = (int)((q / (2 * R)) % 2);
    const int k = (int)(q / (4 * R));
    const int delta = d < R ? d - R : d - R + 1;
    int32_t& var = field == 0 ? s[k] : e[k];
    const int64_t moved = (int64_t)var + delta;
    if (active[k] == 0 || moved < 0 || moved >= T) {
      scores[2 * idx] = -1;
      scores[2 * idx + 1] = -1;
      continue;
    }
    const int32_t keep = var;
    var = (int32_t)moved;
    evaluate(p, s.data(), e.data(), active, w, res, nullptr);
    var = keep;
    scores[2 * idx] = res[R_VIOLATIONS];
    scores[2 * idx + 1] = res[R_PEAK];
    const int64_t key_mem = res[R_PEAK] > budget ? res[R_PEAK] : budget;
    const int64_t best_mem = best_peak > budget ? best_peak : budget;
    if (best_move < 0 || res[R_VIOLATIONS] < best_v ||
        (res[R_VIOLATIONS] == best_v &&
         (key_mem < best_mem || (key_mem == best_mem && res[R_PEAK] < best_peak)))) {
      // moves are visited in increasing q within a call that scores all of them,
      // so strict improvement keeps the smallest q among equals
      best_move = q; best_v = res[R_VIOLATIONS]; best_peak = res[R_PEAK];
    }
  }
  if (best) {
    best[0] = best_move;
    best[1] = best_move < 0 ? 0 : best_v;
    best[2] = best_move < 0 ? 0 : best_peak;
  }
}

// Scores of the K = n*C candidates that differ from the given one in one active flag
// (starts and ends stay): scores[3k..3k+2] = (violations, peak, duration) of the candidate
// with active[k] flipped, by full re-evaluation.  Dropping a copy or activating a spare one
// are the moves that change the objective, Eq. (1).
void orc_toggles(int32_t n, const int32_t* in_ptr, const int32_t* in_idx, const int32_t* size, const int32_t* dur,
                 int64_t budget, int32_t C, int32_t T, const int32_t* starts, const int32_t* ends,
                 const uint8_t* active, int64_t* scores) {
  Problem p{n, in_ptr, in_idx, size, dur, budget, C, T};
  Scratch w;
  const int K = n * C;
  std::vector<uint8_t> a(active, active + K);
  int64_t res[R_FIELDS];
  for (int k = 0; k < K; ++k) {
    a[k] = a[k] ? 0 : 1;
    evaluate(p, starts, ends, a.data(), w, res, nullptr);
    a[k] = active[k];
    scores[3 * k] = res[R_VIOLATIONS];
    scores[3 * k + 1] = res[R_PEAK];
    scores[3 * k + 2] = res[R_DURATION];
  }
}

// The cut-and-recompute move for in-edge x = (u, v) (CSR order) and copy i of the consumer v,
// applied to s, e, a in place.  Not part of the paper's text as a procedure: it is the edit that
// turns "keep u's output until v needs it" into "recompute u just before v", the trade of
// duration for memory the formulation exists for (Section 1; Eq. (1) against Eq. (4)).
//   t  = start of the consumer copy, which must be live;
//   k  = the live copy of u with s_k < t <= e_k that starts last (lowest index among equals);
//   j  = the lowest copy of u that is not active;
//   p  = the last position in (s_k, t) at which no live copy starts and the outputs of all
//        predecessors of u are held (Eq. (5) for the new computation);
//   e' = the last start, in (s_k, p), of a live copy of a consumer of u; s_k if there is none.
// Copy k keeps [s_k, e'], copy j becomes active with [p, e_k].  Returns 0 (nothing changed) if
// the consumer copy is not live or k, j or p does not exist.
// mode 1 (keep the inputs instead of looking for a place where they are held): p is the last
// position in (s_k, t) at which no live copy starts and every predecessor w of u is either held
// (a live copy with s_w < p <= e_w) or has a live copy that ends before p; for each predecessor
// that is not held, its live copy with the largest end below p (the highest index among equals)
// is kept until p.  Small inputs are then carried across the stretch on which the large output
// is dropped.
static int apply_cut(const Problem& p, int x, int i, int32_t* s, int32_t* e, uint8_t* a, int mode = 0) {
  const int C = p.C, T = p.T;
  auto live = [&](int c) { return a[c] && s[c] >= 0 && s[c] <= e[c] && e[c] <= T - 1; };
  int v = 0;
  while (p.in_ptr[v + 1] <= x) ++v;
  const int u = p.in_idx[x];
  const int c = v * C + i;
  if (!live(c)) return 0;
  const int t = s[c];
  int k = -1, j = -1;
  for (int q = 0; q < C; ++q) {
    const int cu = u * C + q;
    if (live(cu) && s[cu] < t && t <= e[cu] && (k < 0 || s[cu] > s[k])) k = cu;
    if (!a[cu] && j < 0) j = cu;
  }
  if (k < 0 || j < 0) return 0;
  std::vector<char> taken(T, 0);
  for (int q = 0; q < p.n * C; ++q)
    if (live(q)) taken[s[q]] = 1;
  auto inputs_held = [&](int at) {   // every predecessor of u has a live copy with s < at <= e
    for (int y = p.in_ptr[u]; y < p.in_ptr[u + 1]; ++y) {
      bool held = false;
      for (int q = 0; q < C; ++q) {
        const int cw = p.in_idx[y] * C + q;
        if (live(cw) && s[cw] < at && at <= e[cw]) held = true;
      }
      if (!held) return false;
    }
    return true;
  };
  auto held_at = [&](int w, int at) {
    for (int q = 0; q < C; ++q) {
      const int cw = w * C + q;
      if (live(cw) && s[cw] < at && at <= e[cw]) return true;
    }
    return false;
  };
  auto copy_to_keep = [&](int w, int at) {   // live copy of w with the largest end below at, -1 if none
    int best = -1;
    for (int q = 0; q < C; ++q) {
      const int cw = w * C + q;
      if (live(cw) && e[cw] < at && (best < 0 || e[cw] >= e[best])) best = cw;
    }
    return best;
  };
  auto inputs_can_be_had = [&](int at) {
    for (int y = p.in_ptr[u]; y < p.in_ptr[u + 1]; ++y)
      if (!held_at(p.in_idx[y], at) && copy_to_keep(p.in_idx[y], at) < 0) return false;
    return true;
  };
  int pos = t - 1;
  if (mode == 0)
    while (pos > s[k] && (taken[pos] || !inputs_held(pos))) --pos;
  else
    while (pos > s[k] && (taken[pos] || !inputs_can_be_had(pos))) --pos;
  if (pos <= s[k]) return 0;
  if (mode == 1)
    for (int y = p.in_ptr[u]; y < p.in_ptr[u + 1]; ++y) {
      const int w = p.in_idx[y];
      if (!held_at(w, pos)) e[copy_to_keep(w, pos)] = pos;   // a predecessor listed twice is held the second time
    }
  int last_use = s[k];
  for (int w = 0; w < p.n; ++w)
    for (int y = p.in_ptr[w]; y < p.in_ptr[w + 1]; ++y)
      if (p.in_idx[y] == u)
        for (int q = 0; q < C; ++q) {
          const int cw = w * C + q;
          if (live(cw) && s[cw] > s[k] && s[cw] < pos && s[cw] > last_use) last_use = s[cw];
        }
  a[j] = 1;
  s[j] = pos;
  e[j] = e[k];
  e[k] = last_use;
  return 1;
}

// One cut applied to a copy of the candidate: out_s, out_e, out_a [n*C].  Returns 1 if the move
// is applicable, 0 otherwise (outputs = inputs).
int orc_cut_apply(int32_t n, const int32_t* in_ptr, const int32_t* in_idx, const int32_t* size, const int32_t* dur,
                  int32_t C, int32_t T, const int32_t* starts, const int32_t* ends, const uint8_t* active,
                  int32_t x, int32_t i, int32_t* out_s, int32_t* out_e, uint8_t* out_a, int32_t mode) {
  Problem p{n, in_ptr, in_idx, size, dur, 0, C, T};
  const int K = n * C;
  std::copy(starts, starts + K, out_s);
  std::copy(ends, ends + K, out_e);
  std::copy(active, active + K, out_a);
  return apply_cut(p, x, i, out_s, out_e, out_a, mode);
}

// Number of positions at which a profile reaches at least `level`.
static int64_t positions_at(const std::vector<int64_t>& prof, int T, int64_t level) {
  int64_t c = 0;
  for (int t = 0; t < T; ++t) c += prof[t] >= level ? 1 : 0;
  return c;
}

// Scores of all m*C cuts of one candidate: scores[4q..4q+3] = (violations, peak, duration,
// positions at which the edited candidate's memory still reaches the peak of the candidate as
// given) by full re-evaluation, q = x*C + i; (-1, -1, 0, 0) where not applicable.
void orc_cuts(int32_t n, const int32_t* in_ptr, const int32_t* in_idx, const int32_t* size, const int32_t* dur,
              int64_t budget, int32_t C, int32_t T, const int32_t* starts, const int32_t* ends,
              const uint8_t* active, int64_t* scores, int32_t mode) {
  Problem p{n, in_ptr, in_idx, size, dur, budget, C, T};
  Scratch w;
  const int K = n * C, m = in_ptr[n];
  std::vector<int32_t> s(K), e(K);
  std::vector<uint8_t> a(K);
  std::vector<int64_t> prof(T);
  int64_t res[R_FIELDS];
  evaluate(p, starts, ends, active, w, res, nullptr);
  const int64_t base_peak = res[R_PEAK];
  for (int x = 0; x < m; ++x)
    for (int i = 0; i < C; ++i) {
      std::copy(starts, starts + K, s.begin());
      std::copy(ends, ends + K, e.begin());
      std::copy(active, active + K, a.begin());
      int64_t* out = scores + 4 * ((int64_t)x * C + i);
      if (!apply_cut(p, x, i, s.data(), e.data(), a.data(), mode)) {
        out[0] = -1; out[1] = -1; out[2] = 0; out[3] = 0;
        continue;
      }
      evaluate(p, s.data(), e.data(), a.data(), w, res, prof.data());
      out[0] = res[R_VIOLATIONS];
      out[1] = res[R_PEAK];
      out[2] = res[R_DURATION];
      out[3] = positions_at(prof, T, base_peak);
    }
}

// Greedy descent by cuts, one candidate, in place: up to max_steps times, score every cut by
// full re-evaluation, take the first minimum of (violations, peak, positions left at the
// present peak) among the applicable ones, and apply it if it lowers
// (violations, max(peak, M)) against the candidate as it stands or, above the budget with both
// unchanged, leaves fewer positions at the peak; stop at the first step that does not.
// Returns the number of cuts applied.
int orc_search_cuts(int32_t n, const int32_t* in_ptr, const int32_t* in_idx, const int32_t* size, const int32_t* dur,
                    int64_t budget, int32_t C, int32_t T, int32_t* starts, int32_t* ends, uint8_t* active,
                    int32_t max_steps, int32_t mode) {
  Problem p{n, in_ptr, in_idx, size, dur, budget, C, T};
  Scratch w;
  const int K = n * C, m = in_ptr[n];
  std::vector<int32_t> s(K), e(K);
  std::vector<uint8_t> a(K);
  std::vector<int64_t> prof(T);
  int64_t res[R_FIELDS];
  int applied = 0;
  for (int step = 0; step < max_steps; ++step) {
    evaluate(p, starts, ends, active, w, res, prof.data());
    const int64_t now_v = res[R_VIOLATIONS], now_peak = res[R_PEAK], now_p = std::max(now_peak, budget);
    const int64_t now_at = positions_at(prof, T, now_peak);
    int64_t best_v = 0, best_p = 0, best_at = 0;
    int best_x = -1, best_i = -1;
    for (int x = 0; x < m; ++x)
      for (int i = 0; i < C; ++i) {
        std::copy(starts, starts + K, s.begin());
        std::copy(ends, ends + K, e.begin());
        std::copy(active, active + K, a.begin());
        if (!apply_cut(p, x, i, s.data(), e.data(), a.data(), mode)) continue;
        evaluate(p, s.data(), e.data(), a.data(), w, res, prof.data());
        const int64_t at = positions_at(prof, T, now_peak);
        if (best_x < 0 || res[R_VIOLATIONS] < best_v ||
            (res[R_VIOLATIONS] == best_v && (res[R_PEAK] < best_p || (res[R_PEAK] == best_p && at < best_at)))) {
          best_v = res[R_VIOLATIONS];
          best_p = res[R_PEAK];
          best_at = at;
          best_x = x;
          best_i = i;
        }
      }
    if (best_x < 0) break;
    const int64_t then_p = std::max(best_p, budget);
    const bool better = best_v < now_v ||
                        (best_v == now_v && (then_p < now_p || (then_p == now_p && now_peak > budget && best_at < now_at)));
    if (!better) break;
    apply_cut(p, best_x, best_i, starts, ends, active, mode);
    ++applied;
  }
  return applied;
}

}  // extern "C"
