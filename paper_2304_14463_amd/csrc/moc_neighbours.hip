// moc_eval_neighbours: scores every single-field move (start or end of one copy
// by -R..-1, +1..+R positions) of a batch of base candidates.  The move set is
// this library's (the neighbourhood a local search over the variables of the
// paper's Section 2.1 would scan); each score is, by definition, what
// moc_eval_batch returns for the candidate with that one field changed.
//
// One workgroup per base candidate.  It evaluates the base once and keeps in
// LDS what a move needs: the packed intervals of all copies, the memory profile
// (Eq. (4) left-hand side per position) with its prefix and suffix maxima, and
// two bitmaps of start positions occupied once / more than once (Eq. (6)).
// A move of copy k = (v, i) changes only
//   - whether copy k is well formed                           Eq. (2), (8)
//   - the ordering among the copies of v                      Eq. (3)
//   - the start collision of copy k                           Eq. (6)
//   - the inputs of copy k (in-edges of v)                    Eq. (5), k as consumer
//   - the consumers of v (out-edges of v, all their copies)   Eq. (5), v as provider
//   - the profile on the positions gained or lost             Eq. (4)
// so violations' = violations - f(old copy) + f(new copy) + start-collision delta,
// with f = the first, second, fourth and fifth items counted around node v,
// and peak' = max(prefix max before, suffix max after, shifted profile inside)
// over the changed positions (at most R of them unless the copy was outside
// the domain before the move).
// Pass 1 stores f(old copy) per copy and lists the active copies.  Pass 2 runs
// one lane per move of an active copy: 64 consecutive moves of the list per
// wave, so the lanes of one copy walk the same edges together, inactive copies
// cost nothing, and a wave writes its scores as whole 128-byte lines.  A third
// pass fills the scores of the inactive copies (not applicable).  The adjacency
// lists are kept in LDS when they fit beside the five T-word arrays.
#include "moc_internal.h"

namespace {

constexpr int kNT = 1024;
constexpr int kNW = kNT / kWave;

struct NbLayout {
  int T_pad;      // T rounded up to 4
  int bit_words;  // ceil(T / 32)
  int adj_off;    // word offset of the graph's adjacency lists in LDS, 0 if they stay in global memory
  int bytes;
};

NbLayout nb_layout(int T, int n, int m, int max_lds) {
  NbLayout l;
  l.T_pad = (T + 3) & ~3;
  l.bit_words = (T + 31) / 32;
  // profile, prefix max, suffix max, packed, f(old) + two bitmaps + scratch
  const int words = 5 * l.T_pad + 2 * l.bit_words + 8 * kNW + 16;
  l.adj_off = 0;
  l.bytes = 4 * words;
  // the CSR lists both ways, if that costs no resident workgroup (two of 16 waves fit a CU):
  // every move walks the edges of its node
  const int with_adj = 4 * (words + 2 * (n + 1) + 2 * m);
  if (with_adj <= max_lds && std::min(max_lds / with_adj, 2) >= std::min(max_lds / l.bytes, 2)) {
    l.adj_off = words;
    l.bytes = with_adj;
  }
  return l;
}

// The graph's adjacency, by in-edges and by out-edges (CSR), in LDS or in global memory.
struct Adj {
  const int32_t* in_ptr;
  const int32_t* in_idx;
  const int32_t* out_ptr;
  const int32_t* out_idx;
};

struct NbLds {
  int32_t* profile;
  int32_t* pmax;
  int32_t* smax;
  uint32_t* packed;
  uint16_t* fold;   // [2k]: f(old copy k), below 2^15 for any T this call accepts
  uint16_t* list;   // [2j]: j-th entry of the copy lists (the other half of the same words)
  uint32_t* occ1;
  uint32_t* occ2;
  int32_t* scratch;   // 8 * kNW + 16
};

__device__ __forceinline__ bool live_of(uint32_t p) { return (p & 0xFFFFu) != 0xFFFFu; }
__device__ __forceinline__ bool covers1(uint32_t pu, uint32_t x) { return (pu & 0xFFFFu) < x && (pu >> 16) >= x; }
__device__ __forceinline__ uint32_t pack_copy(bool live, int s, int e) {
  return live ? ((uint32_t)s | ((uint32_t)e << 16)) : MOC_DEAD;
}
__device__ __forceinline__ bool bit_at(const uint32_t* bits, int t) { return (bits[t >> 5] >> (t & 31)) & 1u; }

struct AddOp { static __device__ int id() { return 0; } static __device__ int op(int a, int b) { return a + b; } };
struct MaxOp { static __device__ int id() { return 0; } static __device__ int op(int a, int b) { return max(a, b); } };

// Inclusive scan of dst[idx(0..T-1)] <- src, in place allowed; REV scans from the top.
template <typename Op, bool REV>
__device__ void block_scan(const int32_t* src, int32_t* dst, int T, int32_t* scratch, int tid) {
  const int lane = tid & (kWave - 1), wave = tid / kWave;
  const int L = (T + kNT - 1) / kNT;
  const int lo = tid * L, hi = min(lo + L, T);
  auto at = [&](int i) { return REV ? T - 1 - i : i; };
  int acc = Op::id();
  for (int i = lo; i < hi; ++i) acc = Op::op(acc, src[at(i)]);
  int inc = acc;
#pragma unroll
  for (int off = 1; off < kWave; off <<= 1) {
    const int o = __shfl_up(inc, off);
    if (lane >= off) inc = Op::op(inc, o);
  }
  if (lane == kWave - 1) scratch[wave] = inc;
  __syncthreads();
  int before = Op::id();
  for (int w = 0; w < wave; ++w) before = Op::op(before, scratch[w]);
  const int prev = __shfl_up(inc, 1);
  int run = Op::op(before, lane == 0 ? Op::id() : prev);
  for (int i = lo; i < hi; ++i) {
    run = Op::op(run, src[at(i)]);
    dst[at(i)] = run;
  }
  __syncthreads();
}

// The part of the violation count that depends on copy i of node v: copy i with the
// given values (all other copies as staged in `packed`).
//   form  : copy i active but not well formed
//   order : Eq. (3) among the live copies of v
//   cons  : in-edges of v not covered at the start of copy i
//   prov  : (out-edge (v,w), live copy of w) pairs not covered by any live copy of v
__device__ __forceinline__ int node_part(const Adj& g, int C, const uint32_t* __restrict__ packed, int v, int i,
                                         bool active, bool live, int s, int e) {
  const uint32_t mine = pack_copy(live, s, e);
  int count = (active && !live) ? 1 : 0;
  // Eq. (3): each live copy against the next live copy
  int prev_end = -1;
  bool have_prev = false;
  for (int j = 0; j < C; ++j) {
    const uint32_t p = j == i ? mine : packed[v * C + j];
    if (!live_of(p)) continue;
    if (have_prev && prev_end > (int)(p & 0xFFFFu)) ++count;
    prev_end = (int)(p >> 16);
    have_prev = true;
  }
  // Eq. (5), copy i as consumer
  if (live) {
    for (int q = g.in_ptr[v]; q < g.in_ptr[v + 1]; ++q) {
      const int u = g.in_idx[q];
      bool cov = false;
      for (int j = 0; j < C; ++j) cov = cov || covers1(packed[u * C + j], (uint32_t)s);
      count += cov ? 0 : 1;
    }
  }
  // Eq. (5), node v as provider
  for (int q = g.out_ptr[v]; q < g.out_ptr[v + 1]; ++q) {
    const int w = g.out_idx[q];
    for (int jw = 0; jw < C; ++jw) {
      const uint32_t pw = packed[w * C + jw];
      if (!live_of(pw)) continue;
      const uint32_t x = pw & 0xFFFFu;
      bool cov = false;
      for (int j = 0; j < C; ++j) cov = cov || covers1(j == i ? mine : packed[v * C + j], x);
      count += cov ? 0 : 1;
    }
  }
  return count;
}

// One move of a copy, from scratch: (violations, peak) of the candidate with that one field
// at `moved`.  The general form; the kernel uses it for copies that are ill-formed before
// the move, where the changed positions are a whole interval.
__device__ __forceinline__ void score_move(const Adj& g, int C, int sz, const NbLds& L, int T, int v, int i,
                                           int field, int s, int e, int moved, int base_viol, int base_peak,
                                           moc_move_score& sc) {
  const int k = v * C + i;
  const int s2 = field == 0 ? moved : s, e2 = field == 0 ? e : moved;
  const bool live_old = live_of(L.packed[k]);
  const bool live_new = (uint32_t)s2 <= (uint32_t)e2 && (uint32_t)e2 < (uint32_t)T;
  int vv = base_viol - (int)L.fold[2 * k] + node_part(g, C, L.packed, v, i, true, live_new, s2, e2);
  if (live_old && bit_at(L.occ2, s)) --vv;
  if (live_new) vv += (live_old && s2 == s) ? (bit_at(L.occ2, s) ? 1 : 0) : (bit_at(L.occ1, s2) ? 1 : 0);
  // peak: positions lost (sign -1) or gained (sign +1)
  int pk = base_peak;
  if (live_old || live_new) {
    int lo = 0, hi = -1, sign = 0;
    if (live_old && live_new) {
      if (field == 0) { lo = min(s, s2); hi = max(s, s2) - 1; sign = s2 < s ? 1 : -1; }
      else { lo = min(e, e2) + 1; hi = max(e, e2); sign = e2 > e ? 1 : -1; }
    } else if (live_old) { lo = s; hi = e; sign = -1; }
    else { lo = s2; hi = e2; sign = 1; }
    int inside = 0;
    for (int t = lo; t <= hi; ++t) inside = max(inside, L.profile[t] + sign * sz);
    pk = max(inside, max(lo > 0 ? L.pmax[lo - 1] : 0, hi + 1 < T ? L.smax[hi + 1] : 0));
  }
  sc.violations = vv;
  sc.peak = pk;
}


// One move of a live copy (v, i): field moved to `moved`, a position in [0, T).
// `mine` is the copy before the move, `fixed` the base violation count without
// f(old copy).  The changed positions of the profile are at most R: the move is
// by at most R, and when it leaves the copy ill formed the copy was shorter than that.
template <int CT>
__device__ __forceinline__ void score_live(const Adj& A, int C, int sz, const NbLds& L, int T, int R, int v, int i,
                                           int field, int moved, uint32_t mine, int fixed, int in_lo, int in_hi,
                                           int out_lo, int out_hi,                                            moc_move_score& sc) {
  const int s = (int)(mine & 0xFFFFu), e = (int)(mine >> 16);
  const int s2 = field == 0 ? moved : s, e2 = field == 0 ? e : moved;
  const bool live_new = s2 <= e2;
  const uint32_t moved_copy = pack_copy(live_new, s2, e2);
  const uint32_t* const row = L.packed + v * C;
  uint32_t cv[CT > 0 ? CT : 1];   // the copies of v after the move
  if constexpr (CT > 0) {
#pragma unroll
    for (int j = 0; j < CT; ++j) cv[j] = j == i ? moved_copy : row[j];
  }
  auto copy_of_v = [&](int j) -> uint32_t {
    if constexpr (CT > 0) return cv[j];
    else return j == i ? moved_copy : row[j];
  };
  int count = live_new ? 0 : 1;   // Eq. (2)/(8)
  // Eq. (3): each live copy of v against the next live one
  int prev_end = -1;
  for (int j = 0; j < C; ++j) {
    const uint32_t p = copy_of_v(j);
    if (!live_of(p)) continue;
    count += prev_end > (int)(p & 0xFFFFu) ? 1 : 0;
    prev_end = (int)(p >> 16);
  }
  // Eq. (6): the old start leaves, the new one arrives
  const int start_twice = bit_at(L.occ2, s) ? 1 : 0;
  count -= start_twice;
  if (live_new) count += s2 == s ? start_twice : (bit_at(L.occ1, s2) ? 1 : 0);
  // Eq. (5), the copy as consumer: in-edges whose provider does not cover the start
  for (int q = in_lo, q1 = live_new ? in_hi : in_lo; q < q1; ++q) {
    const uint32_t* const pu = L.packed + A.in_idx[q] * C;
    bool cov = false;
    for (int j = 0; j < C; ++j) cov = cov || covers1(pu[j], (uint32_t)s2);
    count += cov ? 0 : 1;
  }
  // Eq. (5), node v as provider: every live copy of every consumer
  for (int q = out_lo; q < out_hi; ++q) {
    const uint32_t* const pw = L.packed + A.out_idx[q] * C;
    for (int jw = 0; jw < C; ++jw) {
      const uint32_t pos = pw[jw] & 0xFFFFu;
      if (pos == 0xFFFFu) continue;
      bool cov = false;
      for (int j = 0; j < C; ++j) cov = cov || covers1(copy_of_v(j), pos);
      count += cov ? 0 : 1;
    }
  }
  sc.violations = fixed + count;
  // Eq. (4): positions gained (sign +1) or lost (sign -1)
  int lo, hi;
  bool gain;
  if (!live_new) { lo = s; hi = e; gain = false; }
  else if (field == 0) { lo = min(s, s2); hi = max(s, s2) - 1; gain = s2 < s; }
  else { lo = min(e, e2) + 1; hi = max(e, e2); gain = e2 > e; }
  int top = 0;
  for (int j0 = 0; j0 < R; j0 += 4) {
    int p[4];
#pragma unroll
    for (int x = 0; x < 4; ++x) p[x] = L.profile[min(lo + j0 + x, hi)];
    top = max(max(top, p[0]), max(max(p[1], p[2]), p[3]));
  }
  const int inside = top + (gain ? sz : -sz);
  const int outside = max(lo > 0 ? L.pmax[lo - 1] : 0, hi + 1 < T ? L.smax[hi + 1] : 0);
  sc.peak = max(max(inside, 0), outside);
}

struct Best {
  int viol, peak, move;   // move < 0: none
};

__device__ __forceinline__ bool better(const Best& a, const Best& b, int64_t budget) {
  if (a.move < 0) return false;
  if (b.move < 0) return true;
  if (a.viol != b.viol) return a.viol < b.viol;
  const int64_t ma = max((int64_t)a.peak, budget), mb = max((int64_t)b.peak, budget);
  if (ma != mb) return ma < mb;
  if (a.peak != b.peak) return a.peak < b.peak;
  return a.move < b.move;
}

template <bool ADJ_LDS, int CT>
__global__ __launch_bounds__(kNT) __attribute__((amdgpu_waves_per_eu(8, 8))) void neighbours_kernel(GraphView g, int64_t B, const int32_t* __restrict__ starts,
                                                         const int32_t* __restrict__ ends,
                                                         const uint8_t* __restrict__ active, int R,
                                                         moc_move_score* __restrict__ out_moves,
                                                         moc_best_move* __restrict__ out_best, NbLayout lay) {
  extern __shared__ uint32_t nb_raw[];
  NbLds L;
  L.profile = reinterpret_cast<int32_t*>(nb_raw);
  L.pmax = L.profile + lay.T_pad;
  L.smax = L.pmax + lay.T_pad;
  L.packed = reinterpret_cast<uint32_t*>(L.smax + lay.T_pad);
  L.fold = reinterpret_cast<uint16_t*>(L.packed + lay.T_pad);
  L.list = L.fold + 1;
  L.occ1 = reinterpret_cast<uint32_t*>(L.fold + 2 * lay.T_pad);
  L.occ2 = L.occ1 + lay.bit_words;
  L.scratch = reinterpret_cast<int32_t*>(L.occ2 + lay.bit_words);
  const int tid = threadIdx.x, lane = tid & (kWave - 1);
  const int wave = __builtin_amdgcn_readfirstlane(tid / kWave);
  const int T = g.T, C = CT ? CT : g.C;
  const uint32_t c_magic = 0xFFFFFFFFu / (uint32_t)C + 1u;   // k / C = umulhi(k, c_magic) for C > 1, k < 2^16
  const int two_r = 2 * R, four_r = 4 * R;
  const int moves_per_cand = T * four_r;
  // lane -> move: a wave scores 64 / 4R copies at a time (4R <= 64), or one copy in two pieces
  const int per_wave = four_r <= kWave ? kWave / four_r : 1;
  const int pieces = four_r <= kWave ? 1 : 2;
  const int sub = four_r <= kWave ? lane / four_r : 0;
  const int rem = four_r <= kWave ? lane - sub * four_r : lane;
  int32_t* const counts = L.scratch + 8 * kNW;   // [0] base violations, [1] active copies, [2] inactive copies
  Adj A{g.in_ptr, g.in_idx, g.out_ptr, g.out_idx};
  if constexpr (ADJ_LDS) {   // the adjacency lists are read by every move: keep them in LDS
    int32_t* a = reinterpret_cast<int32_t*>(nb_raw) + lay.adj_off;
    for (int x = tid; x <= g.n; x += kNT) { a[x] = g.in_ptr[x]; a[g.n + 1 + g.m + x] = g.out_ptr[x]; }
    for (int x = tid; x < g.m; x += kNT) { a[g.n + 1 + x] = g.in_idx[x]; a[2 * (g.n + 1) + g.m + x] = g.out_idx[x]; }
    A = Adj{a, a + g.n + 1, a + g.n + 1 + g.m, a + 2 * (g.n + 1) + g.m};
    __syncthreads();
  }

  for (int64_t b = blockIdx.x; b < B; b += gridDim.x) {
    const int64_t row = b * T;
    // ---- base candidate: stage copies, scatter deltas, mark starts
    for (int t = tid; t < T; t += kNT) L.profile[t] = 0;
    for (int w = tid; w < 2 * lay.bit_words; w += kNT) L.occ1[w] = 0;
    if (tid < 4) counts[tid] = 0;
    __syncthreads();
    int viol = 0, nlive = 0;
    for (int k = tid; k < T; k += kNT) {
      const int s = starts[row + k], e = ends[row + k];
      const bool act = active[row + k] != 0;
      const bool live = act && (uint32_t)s <= (uint32_t)e && (uint32_t)e < (uint32_t)T;
      const int v = C == 1 ? k : (int)__umulhi((uint32_t)k, c_magic);
      L.packed[k] = pack_copy(live, s, e);
      if (k == v * C && !act) ++viol;   // Eq. (7)
      if (live) {
        ++nlive;
        const int sz = g.size_dur[v].x;
        atomicAdd(&L.profile[s], sz);
        if (e + 1 < T) atomicSub(&L.profile[e + 1], sz);
        const uint32_t bit = 1u << (s & 31);
        const uint32_t old = atomicOr(&L.occ1[s >> 5], bit);
        if (old & bit) atomicOr(&L.occ2[s >> 5], bit);
      }
    }
    __syncthreads();
    block_scan<AddOp, false>(L.profile, L.profile, T, L.scratch, tid);   // Eq. (4) per position
    block_scan<MaxOp, false>(L.profile, L.pmax, T, L.scratch, tid);
    block_scan<MaxOp, true>(L.profile, L.smax, T, L.scratch, tid);

    // ---- pass 1: f(old copy) per copy; base violation count; the lists of active copies
    // (from the front of `list`) and of inactive ones (from the back)
    for (int k0 = wave * kWave; k0 < T; k0 += kNT) {
      const int k = k0 + lane;
      bool act = false;
      if (k < T) {
        const int v = C == 1 ? k : (int)__umulhi((uint32_t)k, c_magic), i = k - v * C;
        const int s = starts[row + k], e = ends[row + k];
        act = active[row + k] != 0;
        const bool live = live_of(L.packed[k]);
        L.fold[2 * k] = (uint16_t)(act ? node_part(A, C, L.packed, v, i, act, live, s, e) : 0);
        // base count: each instance once -- form, the order pair that copy k opens, its inputs
        viol += (act && !live) ? 1 : 0;
        if (live) {
          for (int j = i + 1; j < C; ++j) {
            const uint32_t p = L.packed[v * C + j];
            if (live_of(p)) {
              viol += e > (int)(p & 0xFFFFu) ? 1 : 0;
              break;
            }
          }
          for (int q = A.in_ptr[v]; q < A.in_ptr[v + 1]; ++q) {
            const int u = A.in_idx[q];
            bool cov = false;
            for (int j = 0; j < C; ++j) cov = cov || covers1(L.packed[u * C + j], (uint32_t)s);
            viol += cov ? 0 : 1;
          }
        }
      }
      const uint64_t am = __ballot(act), im = __ballot(k < T && !act);
      int abase = 0, ibase = 0;
      if (lane == 0) {
        abase = atomicAdd(&counts[1], __popcll(am));
        ibase = atomicAdd(&counts[2], __popcll(im));
      }
      abase = __shfl(abase, 0);
      ibase = __shfl(ibase, 0);
      const uint64_t below = ((uint64_t)1 << lane) - 1;
      if (act) L.list[2 * (abase + __popcll(am & below))] = (uint16_t)k;
      else if (k < T) L.list[2 * (T - 1 - ibase - __popcll(im & below))] = (uint16_t)k;
    }
    int distinct = 0;
    for (int w = tid; w < lay.bit_words; w += kNT) distinct += __popc(L.occ1[w]);
    atomicAdd(&counts[0], viol + nlive - distinct);   // Eq. (6): live copies - distinct starts
    __syncthreads();
    const int base_viol = counts[0], n_active = counts[1];
    const int base_peak = L.pmax[T - 1];

    // ---- pass 2: one lane per move of an active copy
    Best best{0, 0, -1};
    const int groups = (n_active + per_wave - 1) / per_wave;
    for (int it = wave; it < groups * pieces; it += kNW) {
      const int grp = pieces == 1 ? it : it >> 1;
      const int in_copy = pieces == 1 ? rem : rem + (it & 1) * kWave;   // field * 2R + d
      const int entry = grp * per_wave + sub;
      if (sub >= per_wave || entry >= n_active || in_copy >= four_r) continue;
      const int k = L.list[2 * entry];
      const int v = C == 1 ? k : (int)__umulhi((uint32_t)k, c_magic), i = k - v * C;
      const int field = in_copy >= two_r ? 1 : 0, d = in_copy - field * two_r;
      const int delta = d < R ? d - R : d - R + 1;
      const int q = k * four_r + in_copy;
      const uint32_t mine = L.packed[k];
      const int sz = g.size_dur[v].x;
      const int in_lo = A.in_ptr[v], in_hi = A.in_ptr[v + 1], out_lo = A.out_ptr[v], out_hi = A.out_ptr[v + 1];
      moc_move_score sc{-1, -1};
      if (live_of(mine)) {
        const int moved = (int)(field == 0 ? mine & 0xFFFFu : mine >> 16) + delta;
        if (moved >= 0 && moved < T)
          score_live<CT>(A, C, sz, L, T, R, v, i, field, moved, mine, base_viol - (int)L.fold[2 * k], in_lo, in_hi,
                         out_lo, out_hi, sc);
      } else {   // active and ill formed (rare): from scratch
        const int s = starts[row + k], e = ends[row + k];
        const int moved = (field == 0 ? s : e) + delta;
        if (moved >= 0 && moved < T) score_move(A, C, sz, L, T, v, i, field, s, e, moved, base_viol, base_peak, sc);
      }
      if (sc.violations >= 0) {
        const Best cand{sc.violations, sc.peak, q};
        if (better(cand, best, g.budget)) best = cand;
      }
      if (out_moves) out_moves[b * (int64_t)moves_per_cand + q] = sc;
    }
    // ---- the moves of inactive copies are not applicable
    if (out_moves) {
      const int n_inactive = T - n_active;
      const int fill_groups = (n_inactive + per_wave - 1) / per_wave;
      for (int it = wave; it < fill_groups * pieces; it += kNW) {
        const int grp = pieces == 1 ? it : it >> 1;
        const int in_copy = pieces == 1 ? rem : rem + (it & 1) * kWave;
        const int entry = grp * per_wave + sub;
        if (sub >= per_wave || entry >= n_inactive || in_copy >= four_r) continue;
        const int k = L.list[2 * (n_active + entry)];
        out_moves[b * (int64_t)moves_per_cand + k * four_r + in_copy] = moc_move_score{-1, -1};
      }
    }
    // ---- best move of the candidate
    if (out_best) {
#pragma unroll
      for (int off = kWave / 2; off > 0; off >>= 1) {
        Best o;
        o.viol = __shfl_xor(best.viol, off);
        o.peak = __shfl_xor(best.peak, off);
        o.move = __shfl_xor(best.move, off);
        if (better(o, best, g.budget)) best = o;
      }
      if (lane == 0) {
        L.scratch[wave * 4 + 0] = best.viol;
        L.scratch[wave * 4 + 1] = best.peak;
        L.scratch[wave * 4 + 2] = best.move;
      }
      __syncthreads();
      if (tid == 0) {
        Best all{0, 0, -1};
        for (int w = 0; w < kNW; ++w) {
          const Best o{L.scratch[w * 4], L.scratch[w * 4 + 1], L.scratch[w * 4 + 2]};
          if (better(o, all, g.budget)) all = o;
        }
        moc_best_move r;
        r.move = all.move;
        r.violations = all.move < 0 ? 0 : all.viol;
        r.peak = all.move < 0 ? 0 : all.peak;
        out_best[b] = r;
      }
    }
    __syncthreads();
  }
}


using NbKernel = void (*)(GraphView, int64_t, const int32_t*, const int32_t*, const uint8_t*, int, moc_move_score*,
                          moc_best_move*, NbLayout);

template <bool ADJ_LDS>
NbKernel pick_copies(int C) {
  switch (C) {
    case 1: return neighbours_kernel<ADJ_LDS, 1>;
    case 2: return neighbours_kernel<ADJ_LDS, 2>;
    case 3: return neighbours_kernel<ADJ_LDS, 3>;
    case 4: return neighbours_kernel<ADJ_LDS, 4>;
    default: return neighbours_kernel<ADJ_LDS, 0>;   // C read at run time
  }
}

NbKernel pick_kernel(bool adj_lds, int C) { return adj_lds ? pick_copies<true>(C) : pick_copies<false>(C); }

}  // namespace

extern "C" int moc_eval_neighbours(const moc_graph* g, int64_t B, const int32_t* starts, const int32_t* ends,
                                   const uint8_t* active, int32_t R, moc_move_score* out_moves,
                                   moc_best_move* out_best, void* hip_stream) {
  if (!g || B < 0 || R < 1 || R > 32) return MOC_EINVAL;
  if (!out_moves && !out_best) return MOC_EINVAL;
  if (B == 0) return MOC_OK;
  if (!starts || !ends || !active) return MOC_EINVAL;
  if (((uintptr_t)starts | (uintptr_t)ends) & 3) return MOC_EINVAL;
  if (((uintptr_t)out_moves & 7) || ((uintptr_t)out_best & 7)) return MOC_EINVAL;
  int dev = -1;
  MOC_HIP(hipGetDevice(&dev));
  if (dev != g->device) return MOC_EDEVICE;
  if (g->has_self_loop) return MOC_EINVAL;
  const NbLayout lay = nb_layout(g->view.T, g->view.n, g->view.m, g->max_lds);
  if (lay.bytes > g->max_lds) return MOC_EOVERFLOW;
  if ((int64_t)g->view.T * 4 * R > 0x7FFFFFFF) return MOC_EOVERFLOW;
  auto kern = pick_kernel(lay.adj_off != 0, g->view.C);
  MOC_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                              lay.bytes));
  int per_cu = 0;
  MOC_HIP(hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, kern, kNT, lay.bytes));
  if (per_cu < 1) per_cu = 1;
  const int64_t resident = (int64_t)per_cu * g->num_cu;
  const unsigned grid = (unsigned)(B < resident ? B : resident);
  hipLaunchKernelGGL(kern, dim3(grid), dim3(kNT), lay.bytes, static_cast<hipStream_t>(hip_stream), g->view, B,
                     starts, ends, active, R, out_moves, out_best, lay);
  MOC_HIP(hipGetLastError());
  return MOC_OK;
}
