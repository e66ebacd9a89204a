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
// The active copies are listed while the base is staged.  Pass 1 counts the
// violations of the base and marks the copies that take part in one.  Pass 2
// runs one lane per (active copy, field): it builds the 0/1 terms of f as bit
// masks over the displacements, sums them in bit planes and walks outwards from
// the old position (see build_field, walk_own).  Two kernels: for the best move
// alone (fields that cannot win are left out), and with the table of scores (a
// wave writes the rows of consecutive copies, the inactive ones filled in).
// The adjacency lists are kept in LDS when that costs no resident workgroup.
#include "moc_internal.h"

namespace {

constexpr int kNT = 1024;
constexpr int kNW = kNT / kWave;

struct NbLayout {
  int T_pad;      // T rounded up to 4
  int bit_words;  // ceil(T / 32)
  int mask_words; // 2 * ceil(T / 64): the active flags, one bit per copy
  int adj_off;    // word offset of the graph's adjacency lists in LDS, 0 if they stay in global memory
  int bytes;
};

NbLayout nb_layout(int T, int n, int m, int max_lds) {
  NbLayout l;
  l.T_pad = (T + 3) & ~3;
  l.bit_words = (T + 31) / 32;
  l.mask_words = 2 * ((T + 63) / 64);
  // profile, prefix max, suffix max, packed, the list of active copies (16 bits an entry) + bitmaps + scratch
  const int words = 4 * l.T_pad + l.T_pad / 2 + 8 + 2 * l.bit_words + 2 * l.mask_words + 8 * kNW + 16;
  l.adj_off = 0;
  l.bytes = 4 * words;
  // The CSR lists both ways and the sizes, which every move reads, if that costs no resident
  // workgroup (two of 16 waves fit a CU).  (At T = 4000 it would: with them in LDS and one
  // workgroup per CU the table of scores takes 4.2 ms instead of 3.6.)
  const int with_adj = 4 * (words + 2 * (n + 1) + 2 * m + n);
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
  const int32_t* size;   // m_v, one word per node (LDS) or per two words (the graph's {m_v, w_v} pairs)
  int size_stride;
  __device__ __forceinline__ int size_of(int v) const { return size[v * size_stride]; }
};

struct NbLds {
  int32_t* profile;
  int32_t* pmax;
  int32_t* smax;
  uint32_t* packed;
  uint16_t* list;   // the active copies, in order
  uint32_t* occ1;
  uint32_t* occ2;
  uint32_t* involved;   // bit k: copy k takes part in a violation of Eq. (3) or (5)
  uint32_t* amask;      // bit k: copy k is active
  int32_t* scratch;   // 8 * kNW + 16
};

__device__ __forceinline__ bool live_of(uint32_t p) { return (p & 0xFFFFu) != 0xFFFFu; }
__device__ __forceinline__ bool covers1(uint32_t pu, uint32_t x) { return (pu & 0xFFFFu) < x && (pu >> 16) >= x; }
__device__ __forceinline__ uint32_t pack_copy(bool live, int s, int e) {
  return live ? ((uint32_t)s | ((uint32_t)e << 16)) : MOC_DEAD;
}
__device__ __forceinline__ bool bit_at(const uint32_t* bits, int t) { return (bits[t >> 5] >> (t & 31)) & 1u; }

struct AddOp { static __device__ int id() { return 0; } static __device__ int op(int a, int b) { return a + b; } };

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

// dst_up[t] = max(src[0..t]) and dst_down[t] = max(src[t..T-1]) in one pass (src >= 0).
__device__ void block_max_both_ways(const int32_t* src, int32_t* dst_up, int32_t* dst_down, int T, int32_t* scratch,
                                    int tid) {
  const int lane = tid & (kWave - 1), wave = tid / kWave;
  const int L = (T + kNT - 1) / kNT;
  const int lo = tid * L, hi = min(lo + L, T);
  int up = 0, down = 0;
  for (int i = lo; i < hi; ++i) {
    up = max(up, src[i]);
    down = max(down, src[T - 1 - i]);
  }
  int inc_up = up, inc_down = down;
#pragma unroll
  for (int off = 1; off < kWave; off <<= 1) {
    const int a = __shfl_up(inc_up, off), b = __shfl_up(inc_down, off);
    if (lane >= off) {
      inc_up = max(inc_up, a);
      inc_down = max(inc_down, b);
    }
  }
  if (lane == kWave - 1) {
    scratch[wave] = inc_up;
    scratch[kNW + wave] = inc_down;
  }
  __syncthreads();
  int run_up = 0, run_down = 0;
  for (int w = 0; w < wave; ++w) {
    run_up = max(run_up, scratch[w]);
    run_down = max(run_down, scratch[kNW + w]);
  }
  const int prev_up = __shfl_up(inc_up, 1), prev_down = __shfl_up(inc_down, 1);
  if (lane != 0) {
    run_up = max(run_up, prev_up);
    run_down = max(run_down, prev_down);
  }
  for (int i = lo; i < hi; ++i) {
    run_up = max(run_up, src[i]);
    dst_up[i] = run_up;
    run_down = max(run_down, src[T - 1 - i]);
    dst_down[T - 1 - i] = run_down;
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
                                           int field, int s, int e, int moved, int base_rest, int base_peak,
                                           moc_move_score& sc) {   // base_rest: the base count without f(old copy)
  const int k = v * C + i;
  const int s2 = field == 0 ? moved : s, e2 = field == 0 ? e : moved;
  const bool live_old = live_of(L.packed[k]);
  const bool live_new = (uint32_t)s2 <= (uint32_t)e2 && (uint32_t)e2 < (uint32_t)T;
  int vv = base_rest + node_part(g, C, L.packed, v, i, true, live_new, s2, e2);
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

// Sets of moves of one (copy, field) as bit masks.  32 bits serve R <= 15: one bit per
// position first..first+2R around the old one, the old position itself (no move) included.
// 64 bits serve any R this call accepts: one bit per move, d = 0..2R-1 for the displacements
// -R..-1, +1..+R.  below(x, D): the bits under x, clamped to the D bits in use.
template <bool WIDE>
struct Bits;
template <>
struct Bits<false> {
  using M = uint32_t;
  static __device__ __forceinline__ M below(int x, int D) { return (1u << min(max(x, 0), D)) - 1u; }   // D <= 31
  static __device__ __forceinline__ bool any(M m) { return __any(m != 0); }
};
template <>
struct Bits<true> {
  using M = uint64_t;
  static __device__ __forceinline__ M below(int x, int D) {
    const int c = min(x, D);
    return c <= 0 ? 0 : ~(uint64_t)0 >> (64 - c);
  }
  static __device__ __forceinline__ bool any(M m) { return __any(m != 0); }
};

constexpr int kPlanes = 6;           // per-move counters of up to 63 as bit planes; beyond that the slow path
constexpr int kNoCopy = 0x3FFFFFFF;  // start of a copy that does not exist

struct Best {
  int viol, peak, move;   // move < 0: none
};

// Plain stores: a lane writes its row of scores in 16-byte pieces, which the L2 puts together;
// with the non-temporal hint the table takes four times as long.
// `table` is the candidate's table (the same in every lane: a scalar base), `index` the move.
__device__ __forceinline__ void store_score(moc_move_score* table, uint32_t index, const moc_move_score& sc) {
  *reinterpret_cast<moc_move_score*>(reinterpret_cast<char*>(table) + (size_t)(index * 8u)) = sc;
}
__device__ __forceinline__ void store_pair(moc_move_score* table, uint32_t index, const moc_move_score& lo,
                                           const moc_move_score& hi) {   // 16-byte aligned
  *reinterpret_cast<int4*>(reinterpret_cast<char*>(table) + (size_t)(index * 8u)) =
      make_int4(lo.violations, lo.peak, hi.violations, hi.peak);
}

// Order of the best move: (violations, max(peak, budget), peak, move index).  max(peak, budget)
// never decreases with the peak and its ties are broken by the peak, so this is the order
// by (violations, peak, move index).
__device__ __forceinline__ bool better(const Best& a, const Best& b) {
  if (a.move < 0) return false;
  if (b.move < 0) return true;
  if (a.viol != b.viol) return a.viol < b.viol;
  if (a.peak != b.peak) return a.peak < b.peak;
  return a.move < b.move;
}

// What the 2R moves of one field of a live copy add to the violation count, move by move:
// a sum of 0/1 terms, each true on an interval of the moved position.  The terms are built
// as masks over the displacements and summed in bit planes.
template <bool WIDE>
struct FieldState {
  typename Bits<WIDE>::M plane[kPlanes];   // bit d of plane p: bit p of the count of move d
  typename Bits<WIDE>::M live;             // moves that leave the copy well formed
  int fixed, if_live, if_dead;             // violations = fixed + (live ? if_live : if_dead) + count
  int s, e, sz, q0;                        // the copy before the move, its size, index of its first move
  int field;                               // 0: the start moves, 1: the end; -1: nothing to score
};

// The 32-bit masks (R <= 15) have one bit per position first..first+2R, the copy's own
// position (no move) included: the count at that bit is what the copy contributes now, so
// violations of a move = base count - that + count of the move.  The 64-bit masks have one
// bit per move (no room for the extra bit at R = 32); there the copy's present contribution
// is computed edge by edge.  On a counter overflow in any lane the state is marked invalid
// (the caller then scores the moves one by one).
template <int CT, bool WIDE>
__device__ __forceinline__ void build_field(const Adj& A, int C, int sz, const NbLds& L, int T, int R, int v, int i,
                                            int field, uint32_t mine, int base_viol, int q0, FieldState<WIDE>& st) {
  using B = Bits<WIDE>;
  using M = typename B::M;
  const int D = WIDE ? 2 * R : 2 * R + 1;
  const int s = (int)(mine & 0xFFFFu), e = (int)(mine >> 16);
  const int base = field == 0 ? s : e, first = base - R;
  // {bits : moved < x}
  auto lt = [&](int x) -> M {
    if constexpr (WIDE) return B::below(x - first - (x > base ? 1 : 0), D);   // moved: first..base-1, base+1..base+R
    else return B::below(x - first, D);                                        // moved: first..base+R
  };
  const M in_dom = lt(T) & ~lt(0);
  const M live = in_dom & (field == 0 ? lt(e + 1) : ~lt(s));   // start <= end after the move
  // Eq. (3): the live neighbours of copy i among the copies of v
  const uint32_t* const row = L.packed + v * C;
  int prev_end = -1, next_start = kNoCopy;
  for (int j = 0; j < C; ++j) {
    const uint32_t p = row[j];
    if (j == i || !live_of(p)) continue;
    if (j < i) prev_end = (int)(p >> 16);
    else if (next_start == kNoCopy) next_start = (int)(p & 0xFFFFu);
  }
  const int start_twice = bit_at(L.occ2, s) ? 1 : 0;
  const int if_dead = 1 + (prev_end > next_start ? 1 : 0);   // Eq. (2)/(8), Eq. (3) across the gap
  int if_live;   // what a move that keeps the copy well formed adds besides the counted terms
  M plane[kPlanes];
#pragma unroll
  for (int p = 0; p < kPlanes; ++p) plane[p] = 0;
  M overflow = 0;
  auto add = [&](M m) {   // most terms are false for every move of every lane
    M carry = m;
#pragma unroll
    for (int p = 0; p < kPlanes; ++p) {
      if (!B::any(carry)) break;
      const M t = plane[p] & carry;
      plane[p] ^= carry;
      carry = t;
    }
    overflow |= carry;
  };
  const int in_lo = A.in_ptr[v], in_hi = A.in_ptr[v + 1];
  if (field == 0) {
    if_live = e > next_start ? 1 : 0;
    add(live & lt(prev_end));   // Eq. (3): the previous copy ends after the new start
    // Eq. (6): the new start is taken (the copy's own start is not a move)
    {
      auto window = [&](int from, int bits) -> M {   // bits of occ1 from position `from` (>= -R) on; positions below 0 read as 0
        const int f0 = max(from, 0), w = min(f0 >> 5, (T - 1) >> 5), w1 = min(w + 1, (T - 1) >> 5);
        const uint64_t two = (uint64_t)L.occ1[w] | ((uint64_t)(w1 > w ? L.occ1[w1] : 0u) << 32);
        return (M)(((two >> (f0 & 31)) << (f0 - from)) & (((uint64_t)1 << bits) - 1));
      };
      if constexpr (WIDE) add(live & (window(first, R) | (window(base + 1, R) << R)));
      else add(live & window(first, D) & ~((M)1 << R));
    }
    // Eq. (5), the copy as consumer: in-edges whose provider does not cover the new start
    for (int q = in_lo; q < in_hi; ++q) {
      const uint32_t* const pu = L.packed + A.in_idx[q] * C;
      M cov = 0;
      for (int j = 0; j < C; ++j) {
        const uint32_t p = pu[j];
        cov |= lt((int)(p >> 16) + 1) & ~lt((int)(p & 0xFFFFu) + 1);   // start < moved <= end; empty for a dead copy
      }
      add(live & ~cov);
    }
  } else {
    add(live & ~lt(next_start + 1));   // Eq. (3): the new end lies after the next copy's start
    int uncovered = 0;                 // Eq. (5), the copy as consumer: the start stays
    for (int q = in_lo; q < in_hi; ++q) {
      const uint32_t* const pu = L.packed + A.in_idx[q] * C;
      bool cov = false;
      for (int j = 0; j < C; ++j) cov = cov || covers1(pu[j], (uint32_t)s);
      uncovered += cov ? 0 : 1;
    }
    if_live = (prev_end > s ? 1 : 0) + start_twice + uncovered;
  }
  // Eq. (5), node v as provider: every live copy of every consumer that no other copy of v covers
  for (int q = A.out_ptr[v], q1 = A.out_ptr[v + 1]; q < q1; ++q) {
    const uint32_t* const pw = L.packed + A.out_idx[q] * C;
    for (int jw = 0; jw < C; ++jw) {
      const int x = (int)(pw[jw] & 0xFFFFu);
      if (x == 0xFFFF) continue;
      bool cov = false;
      for (int j = 0; j < C; ++j) cov = cov || (j != i && covers1(row[j], (uint32_t)x));
      if (cov) continue;
      // the moved copy covers x: start < x <= end
      const M mine_covers = field == 0 ? (x <= e ? live & lt(x) : (M)0) : (s < x ? live & ~lt(x) : (M)0);
      add(in_dom & ~mine_covers);
    }
  }
  // the copy's contribution now, to be replaced by the move's
  int fixed;
  if constexpr (WIDE) {
    int order_others = 0, pe = -1;   // Eq. (3) between other consecutive live copies, on either side of copy i
    for (int j = 0; j < C; ++j) {
      if (j == i) { pe = -1; continue; }
      const uint32_t p = row[j];
      if (!live_of(p)) continue;
      order_others += pe > (int)(p & 0xFFFFu) ? 1 : 0;
      pe = (int)(p >> 16);
    }
    fixed = base_viol - node_part(A, C, L.packed, v, i, true, true, s, e) + order_others - start_twice;
  } else {
    int now = 0;   // the counted terms at the copy's own position
#pragma unroll
    for (int p = 0; p < kPlanes; ++p) now |= (int)((plane[p] >> R) & 1) << p;
    fixed = base_viol - start_twice - now - (if_live - (field == 0 ? 0 : start_twice));
  }
  st.live = live;
  st.fixed = fixed;
  st.if_live = if_live;
  st.if_dead = if_dead;
  st.s = s;
  st.e = e;
  st.sz = sz;
  st.q0 = q0;
  st.field = B::any(overflow) ? -1 : field;
#pragma unroll
  for (int p = 0; p < kPlanes; ++p) st.plane[p] = plane[p];
}

// The lane walks outwards from the old position of its field, one step per displacement on
// either side.  `top` is the maximum of the profile over the positions gained or lost so far
// on a side; a step adds the position that joins the window.  A start moved down or an end
// moved up gains positions, the other two lose them, no further than the other end of the
// interval (the clamp re-reads that end, which changes no maximum).  The peak of a move is
// max(top +- size, prefix maximum before the window, suffix maximum after it); one of the
// two does not change along a side.  NP: bit planes in use.
// The best move of the field is the minimum of violations << 37 | peak << 6 | index of the move
// in the field (violations < 2^26 for any T this call accepts; a move that is not applicable
// has violations -1, the largest key).
template <int NP, bool WIDE>
__device__ __forceinline__ void walk_own(const FieldState<WIDE>& st, const NbLds& L, int T, int R, bool want_best,
                                         bool pairs, moc_move_score* __restrict__ table, Best& best) {
  const int base = st.field == 0 ? st.s : st.e;
  const bool start_moves = st.field == 0;
  // down: a start gains [moved, s-1], an end loses [max(moved+1, s), e]
  const int from_down = base + (start_moves ? 0 : 1), stop_down = start_moves ? 0 : st.s;
  const int size_down = start_moves ? st.sz : -st.sz;
  const int after_down = L.smax[start_moves ? st.s : st.e + 1];
  // up: a start loses [s, min(moved-1, e)], an end gains [e+1, moved]
  const int from_up = base - (start_moves ? 1 : 0), stop_up = start_moves ? st.e : T - 1;
  const int size_up = -size_down;
  const int before_up = L.pmax[(start_moves ? st.s : st.e + 1) - 1];
  const int if_delta = st.if_live - st.if_dead;
  int top_down = 0, top_up = 0;
  uint64_t key = ~(uint64_t)0;
  const int if_dead = st.fixed + st.if_dead;
  auto bit_of = [](typename Bits<WIDE>::M m, int bit) -> int {
    if constexpr (WIDE) return (int)((m >> bit) & 1);
    else return (int)__builtin_amdgcn_ubfe(m, (uint32_t)bit, 1u);
  };
  auto score = [&](int bit, int top, int size, int outside, bool valid, int index) -> moc_move_score {
    int count = if_dead + bit_of(st.live, bit) * if_delta;
#pragma unroll
    for (int p = 0; p < NP; ++p) count += bit_of(st.plane[p], bit) << p;
    moc_move_score sc;
    sc.violations = valid ? count : -1;
    sc.peak = valid ? max(max(top + size, 0), outside) : -1;
    if (want_best) {
      const uint64_t k = ((uint64_t)(uint32_t)sc.violations << 37) | ((uint64_t)(uint32_t)sc.peak << 6) | (uint32_t)index;
      key = k < key ? k : key;
    }
    return sc;
  };
  auto down = [&](int j) -> moc_move_score {
    const int far = max(from_down - j, stop_down);
    top_down = max(top_down, L.profile[far]);
    return score(R - j, top_down, size_down, max(L.pmax[far - 1], after_down), j <= base, R - j);
  };
  auto up = [&](int j) -> moc_move_score {
    const int far = min(from_up + j, stop_up);
    top_up = max(top_up, L.profile[far]);
    return score(WIDE ? R + j - 1 : R + j, top_up, size_up, max(before_up, L.smax[far + 1]), base + j < T, R + j - 1);
  };
  if (pairs) {   // R even, the table 16-byte aligned: two scores per store
    for (int j = 1; j < R; j += 2) {
      const moc_move_score a0 = down(j), b0 = up(j), a1 = down(j + 1), b1 = up(j + 1);
      if (table) {
        store_pair(table, (uint32_t)(st.q0 + R - j - 1), a1, a0);
        store_pair(table, (uint32_t)(st.q0 + R + j - 1), b0, b1);
      }
    }
  } else {
    for (int j = 1; j <= R; ++j) {
      const moc_move_score a0 = down(j), b0 = up(j);
      if (table) {
        store_score(table, (uint32_t)(st.q0 + R - j), a0);
        store_score(table, (uint32_t)(st.q0 + R + j - 1), b0);
      }
    }
  }
  if (want_best && !(key >> 63)) {
    const Best cand{(int)(key >> 37), (int)((key >> 6) & 0x7FFFFFFFu), st.q0 + (int)(key & 63)};
    if (better(cand, best)) best = cand;
  }
}

template <bool ADJ_LDS, int CT, bool WIDE, bool TABLE>
__global__ __launch_bounds__(kNT) __attribute__((amdgpu_waves_per_eu(8, 8))) void neighbours_kernel(GraphView g, int64_t B, const int32_t* __restrict__ starts,
                                                         const int32_t* __restrict__ ends,
                                                         const uint8_t* __restrict__ active, int R,
                                                         moc_move_score* __restrict__ out_moves,
                                                         moc_best_move* __restrict__ out_best, NbLayout lay) {
  extern __shared__ uint32_t nb_raw[];
  NbLds L;
  L.profile = reinterpret_cast<int32_t*>(nb_raw);
  L.pmax = L.profile + lay.T_pad + 4;   // pmax[-1] = 0
  L.smax = L.pmax + lay.T_pad;          // smax[T] = 0
  L.packed = reinterpret_cast<uint32_t*>(L.smax + lay.T_pad + 4);
  L.list = reinterpret_cast<uint16_t*>(L.packed + lay.T_pad);
  L.occ1 = reinterpret_cast<uint32_t*>(L.list + lay.T_pad);
  L.occ2 = L.occ1 + lay.bit_words;
  L.involved = L.occ2 + lay.bit_words;
  L.amask = L.involved + lay.mask_words;
  L.scratch = reinterpret_cast<int32_t*>(L.amask + lay.mask_words);
  const int tid = threadIdx.x, lane = tid & (kWave - 1);
  const int T = g.T, C = CT ? CT : g.C;
  const uint32_t c_magic = 0xFFFFFFFFu / (uint32_t)C + 1u;   // k / C = umulhi(k, c_magic) for C > 1, k < 2^16
  const int two_r = 2 * R, four_r = 4 * R;
  const int moves_per_cand = T * four_r;
  // lane -> move: a wave scores 64 / 4R copies at a time (4R <= 64), or one copy in two pieces
  const int per_wave = four_r <= kWave ? kWave / four_r : 1;
  const int pieces = four_r <= kWave ? 1 : 2;
  const int sub = four_r <= kWave ? lane / four_r : 0;
  const int rem = four_r <= kWave ? lane - sub * four_r : lane;
  int32_t* const counts = L.scratch + 8 * kNW;   // [0] base violations, [1] active copies, [2] fewest violations of a move so far, [3] work drawn
  const bool pairs = TABLE && (R & 1) == 0 && (reinterpret_cast<uintptr_t>(out_moves) & 15) == 0;   // scores stored two at a time
  Adj A{g.in_ptr, g.in_idx, g.out_ptr, g.out_idx, reinterpret_cast<const int32_t*>(g.size_dur), 2};
  if constexpr (ADJ_LDS) {   // the adjacency lists and sizes are read by every move: keep them in LDS
    int32_t* a = reinterpret_cast<int32_t*>(nb_raw) + lay.adj_off;
    int32_t* const sizes = a + 2 * (g.n + 1) + 2 * g.m;
    for (int x = tid; x <= g.n; x += kNT) { a[x] = g.in_ptr[x]; a[g.n + 1 + g.m + x] = g.out_ptr[x]; }
    for (int x = tid; x < g.m; x += kNT) { a[g.n + 1 + x] = g.in_idx[x]; a[2 * (g.n + 1) + g.m + x] = g.out_idx[x]; }
    for (int x = tid; x < g.n; x += kNT) sizes[x] = g.size_dur[x].x;
    A = Adj{a, a + g.n + 1, a + g.n + 1 + g.m, a + 2 * (g.n + 1) + g.m, sizes, 1};
    __syncthreads();
  }

  for (int64_t b = blockIdx.x; b < B; b += gridDim.x) {
    // what the staging below derives from the thread index is computed again for every base:
    // kept across bases it would sit in registers that the scoring needs, or be spilled
    int t_ = tid;
    asm volatile("" : "+v"(t_));
    const int lane_ = t_ & (kWave - 1);
    const int wave_ = __builtin_amdgcn_readfirstlane(t_ / kWave);

    const int64_t row = b * T;
    moc_move_score* const row0 = TABLE && out_moves ? out_moves + b * (int64_t)moves_per_cand : nullptr;   // this candidate's table
    // ---- base candidate: stage copies, scatter deltas, mark starts
    // The candidate's first kAhead * kNT copies are asked for before the arrays are cleared, all
    // at once and without conditions (lanes past the last copy read it again): they arrive
    // while the workgroup clears and meets at the barrier, instead of one round of loads
    // after the other, each waited for where it is issued.
    constexpr int kAhead = 4;
    int ahead_s[kAhead], ahead_e[kAhead], ahead_sz[kAhead];
    uint32_t ahead_a[kAhead];
    {
      const char* const s_row = reinterpret_cast<const char*>(starts + row);
      const char* const e_row = reinterpret_cast<const char*>(ends + row);
      const char* const a_row = reinterpret_cast<const char*>(active + row);
#pragma unroll
      for (int j = 0; j < kAhead; ++j) {
        const uint32_t k = (uint32_t)min(wave_ * kWave + j * kNT + lane_, T - 1);
        ahead_s[j] = *reinterpret_cast<const int32_t*>(s_row + 4u * k);
        ahead_e[j] = *reinterpret_cast<const int32_t*>(e_row + 4u * k);
        ahead_a[j] = *reinterpret_cast<const uint8_t*>(a_row + k);
        ahead_sz[j] = A.size_of(C == 1 ? (int)k : (int)__umulhi(k, c_magic));
      }
    }
    for (int t = t_; t < T; t += kNT) L.profile[t] = 0;
    for (int w = t_; w < 2 * lay.bit_words + lay.mask_words; w += kNT) L.occ1[w] = 0;   // occ1, occ2, involved
    if (t_ < 4) counts[t_] = t_ == 2 ? 0x7FFFFFFF : 0;
    if (t_ == 0) { L.pmax[-1] = 0; L.smax[T] = 0; }
    __syncthreads();
    // whole waves, 64 consecutive copies each: a ballot gives the active flags of the 64
    int viol = 0, nlive = 0;
    auto stage = [&](int k0, int s, int e, uint32_t flag, int sz) {
      const int k = k0 + lane_;
      bool act = false;
      if (k < T) {
        act = flag != 0;
        const bool live = act && (uint32_t)s <= (uint32_t)e && (uint32_t)e < (uint32_t)T;
        const int v = C == 1 ? k : (int)__umulhi((uint32_t)k, c_magic);
        L.packed[k] = pack_copy(live, s, e);
        if (k == v * C && !act) ++viol;   // Eq. (7)
        if (live) {
          ++nlive;
          atomicAdd(&L.profile[s], sz);
          if (e + 1 < T) atomicSub(&L.profile[e + 1], sz);
          const uint32_t bit = 1u << (s & 31);
          const uint32_t old = atomicOr(&L.occ1[s >> 5], bit);
          if (old & bit) atomicOr(&L.occ2[s >> 5], bit);
        }
      }
      const uint64_t am = __ballot(act);
      if (lane_ == 0) {
        L.amask[k0 >> 5] = (uint32_t)am;
        L.amask[(k0 >> 5) + 1] = (uint32_t)(am >> 32);
        atomicAdd(&counts[1], __popcll(am));
      }
    };
#pragma unroll
    for (int j = 0; j < kAhead; ++j) {
      const int k0 = wave_ * kWave + j * kNT;
      if (k0 < T) stage(k0, ahead_s[j], ahead_e[j], ahead_a[j], ahead_sz[j]);
    }
    for (int k0 = wave_ * kWave + kAhead * kNT; k0 < T; k0 += kNT) {
      const int k = min(k0 + lane_, T - 1);
      stage(k0, starts[row + k], ends[row + k], active[row + k], A.size_of(C == 1 ? k : (int)__umulhi((uint32_t)k, c_magic)));
    }
    __syncthreads();
    // the active copies in order: those of 64 copies go behind those of the copies before
    for (int c = wave_; c < lay.mask_words / 2; c += kNW) {
      int before = 0;
      for (int x = lane_; x < c; x += kWave) before += __popc(L.amask[2 * x]) + __popc(L.amask[2 * x + 1]);
#pragma unroll
      for (int off = kWave / 2; off > 0; off >>= 1) before += __shfl_xor(before, off);
      const uint64_t am = (uint64_t)L.amask[2 * c] | ((uint64_t)L.amask[2 * c + 1] << 32);
      if ((am >> lane_) & 1) L.list[before + __popcll(am & (((uint64_t)1 << lane_) - 1))] = (uint16_t)(c * kWave + lane_);
    }
    block_scan<AddOp, false>(L.profile, L.profile, T, L.scratch, t_);   // Eq. (4) per position
    block_max_both_ways(L.profile, L.pmax, L.smax, T, L.scratch, t_);

    // ---- pass 1: the violations of the base, each instance once: per active copy its form,
    // the order pair it opens and its inputs
    const int n_active = __builtin_amdgcn_readfirstlane(counts[1]);
    for (int j = t_; j < n_active; j += kNT) {
      const int k = L.list[j];
      const uint32_t mine = L.packed[k];
      if (!live_of(mine)) {   // Eq. (2)/(8)
        ++viol;
        continue;
      }
      const int v = C == 1 ? k : (int)__umulhi((uint32_t)k, c_magic), i = k - v * C;
      const int s = (int)(mine & 0xFFFFu), e = (int)(mine >> 16);
      auto mark = [&](int copy) { atomicOr(&L.involved[copy >> 5], 1u << (copy & 31)); };
      if (bit_at(L.occ2, s)) mark(k);   // Eq. (6): the start is shared
      for (int jj = i + 1; jj < C; ++jj) {   // Eq. (3)
        const uint32_t p = L.packed[v * C + jj];
        if (live_of(p)) {
          if (e > (int)(p & 0xFFFFu)) {
            ++viol;
            mark(k);
            mark(v * C + jj);
          }
          break;
        }
      }
      for (int q = A.in_ptr[v]; q < A.in_ptr[v + 1]; ++q) {   // Eq. (5)
        const int u = A.in_idx[q];
        bool cov = false;
        for (int jj = 0; jj < C; ++jj) cov = cov || covers1(L.packed[u * C + jj], (uint32_t)s);
        if (!cov) {   // the consumer and every copy of the provider could mend it
          ++viol;
          mark(k);
          for (int jj = 0; jj < C; ++jj) mark(u * C + jj);
        }
      }
    }
    int distinct = 0;
    for (int w = t_; w < lay.bit_words; w += kNT) distinct += __popc(L.occ1[w]);
    atomicAdd(&counts[0], viol + nlive - distinct);   // Eq. (6): live copies - distinct starts
    __syncthreads();
    const int base_viol = __builtin_amdgcn_readfirstlane(counts[0]);   // the same in every lane_: scalar registers
    const int base_peak = __builtin_amdgcn_readfirstlane(L.pmax[T - 1]);
    // For the best move alone the list is built again, the copies that take part in a violation
    // first: their moves are the ones that can lower the count, and once one has, the others
    // are left out wave_ by wave_ (see below).
    int n_first = n_active;   // entries of the list's first part
    if constexpr (!TABLE) {
      auto chunk = [&](const uint32_t* bits, int c) { return (uint64_t)bits[2 * c] | ((uint64_t)bits[2 * c + 1] << 32); };
      const int chunks = lay.mask_words / 2;
      int all_first = 0;
      for (int x = lane_; x < chunks; x += kWave) all_first += __popcll(chunk(L.amask, x) & chunk(L.involved, x));
#pragma unroll
      for (int off = kWave / 2; off > 0; off >>= 1) all_first += __shfl_xor(all_first, off);
      n_first = __builtin_amdgcn_readfirstlane(all_first);
      for (int c = wave_; c < chunks; c += kNW) {
        int before_first = 0, before_rest = 0;
        for (int x = lane_; x < c; x += kWave) {
          const uint64_t am = chunk(L.amask, x), inv = chunk(L.involved, x);
          before_first += __popcll(am & inv);
          before_rest += __popcll(am & ~inv);
        }
#pragma unroll
        for (int off = kWave / 2; off > 0; off >>= 1) {
          before_first += __shfl_xor(before_first, off);
          before_rest += __shfl_xor(before_rest, off);
        }
        const uint64_t am = chunk(L.amask, c), inv = chunk(L.involved, c), lower = ((uint64_t)1 << lane_) - 1;
        if ((am & inv) >> lane_ & 1) L.list[before_first + __popcll(am & inv & lower)] = (uint16_t)(c * kWave + lane_);
        if ((am & ~inv) >> lane_ & 1) L.list[n_first + before_rest + __popcll(am & ~inv & lower)] = (uint16_t)(c * kWave + lane_);
      }
      __syncthreads();
    }

    // ---- pass 2: one lane per (active copy, field); the waves draw 64 of these at a time.
    // For the best move alone: start moves first, so that all lanes of a wave run the same
    // field's code.  With the table of scores: both fields of 32 consecutive active copies, and
    // the same wave then fills the rows of the inactive copies between them, so that it
    // writes one contiguous stretch of the table (HBM takes long runs much faster than
    // scattered 128-byte rows).
    Best best{0, 0, -1};
    int published = 0x7FFFFFFF;   // the lane's fewest violations as far as the workgroup has been told
    // (TABLE = false compiles the stores away: fewer registers for the best move alone.  With
    // TABLE the pointer is still tested where it was before the kernel was specialised: the
    // build that knows it to be set orders its waits differently and takes 3.5 ms for the table
    // instead of 3.0.)
    const bool table = TABLE && out_moves != nullptr;
    const int draw = table ? kWave / 2 : kWave;
    const int total = table ? max(n_active, 1) : 2 * n_active;
    for (;;) {
      int u0 = 0;
      if (lane == 0) u0 = atomicAdd(&counts[3], draw);
      u0 = __builtin_amdgcn_readfirstlane(u0);
      if (u0 >= total) break;
      int entry, field;
      if (table) {
        entry = u0 + (lane & 31);
        field = lane >> 5;
      } else {   // both fields of the first part of the list, then both of the rest
        const int u = u0 + lane, part = u >= 2 * n_first ? 1 : 0;
        const int in_part = u - part * 2 * n_first, size = part ? n_active - n_first : n_first;
        field = in_part >= size ? 1 : 0;
        entry = part * n_first + in_part - field * size;
      }
      const bool has_unit = entry < n_active;
      const int k = has_unit ? L.list[entry] : 0;
      const int v = C == 1 ? k : (int)__umulhi((uint32_t)k, c_magic), i = k - v * C;
      const int q0 = (2 * k + field) * two_r;
      const int sz = A.size_of(v);
      FieldState<WIDE> st{};
      st.field = -1;
      // For the best move alone, a field none of whose moves can have as few violations as
      // some move already scored (by any wave of the workgroup) is left out.  Before anything
      // is computed for it: a copy that takes part in no violation now (not marked in pass 1,
      // its start not shared) cannot get below the base's count.  After the masks are built:
      // no move has fewer violations than the terms that do not depend on the displacement.
      bool build = has_unit && live_of(L.packed[k]), left_out = false;
      [[maybe_unused]] int least = 0x7FFFFFFF;
      if constexpr (!TABLE) {
        least = *const_cast<volatile int32_t*>(&counts[2]);
        if (build && base_viol > least && !bit_at(L.involved, k) && !bit_at(L.occ2, (int)(L.packed[k] & 0xFFFFu))) {
          build = false;
          left_out = true;
        }
      }
      if (build) build_field<CT, WIDE>(A, C, sz, L, T, R, v, i, field, L.packed[k], base_viol, q0, st);
      bool walk = st.field >= 0;
      if constexpr (!TABLE) walk = walk && st.fixed + min(st.if_live, st.if_dead) <= least;
      if (walk) {
        bool high = false;   // counts above 7 in some lane
#pragma unroll
        for (int p = 3; p < kPlanes; ++p) high = high || Bits<WIDE>::any(st.plane[p]);
        if (high) walk_own<kPlanes, WIDE>(st, L, T, R, out_best != nullptr, pairs, row0, best);
        else walk_own<3, WIDE>(st, L, T, R, out_best != nullptr, pairs, row0, best);
        if constexpr (!TABLE) {
          if (best.move >= 0 && best.viol < published) {
            published = best.viol;
            atomicMin(&counts[2], best.viol);
          }
        }
      }
      if (has_unit && st.field < 0 && !left_out) {   // active and ill formed, or a node with very many edges (rare): move by move, from scratch
        const int s = starts[row + k], e = ends[row + k];
        const int base_rest = base_viol - node_part(A, C, L.packed, v, i, true, live_of(L.packed[k]), s, e);
        for (int d = 0; d < two_r; ++d) {
          const int moved = (field == 0 ? s : e) + (d < R ? d - R : d - R + 1);
          moc_move_score sc{-1, -1};
          if (moved >= 0 && moved < T) {
            score_move(A, C, sz, L, T, v, i, field, s, e, moved, base_rest, base_peak, sc);
            const Best cand{sc.violations, sc.peak, q0 + d};
            if (better(cand, best)) best = cand;
          }
          if (row0) store_score(row0, (uint32_t)(q0 + d), sc);
        }
      }
      if (table) {   // the moves of the inactive copies from this block's first copy to the next block's are not applicable
        const int k_lo = u0 == 0 ? 0 : (int)L.list[u0];
        const int k_hi = u0 + draw < n_active ? (int)L.list[u0 + draw] : T;
        for (int kk0 = k_lo; kk0 < k_hi; kk0 += per_wave) {
          const int kk = kk0 + sub;
          const bool fill = sub < per_wave && kk < k_hi && !((L.amask[kk >> 5] >> (kk & 31)) & 1u);
          for (int piece = 0; piece < pieces; ++piece) {
            const int in_copy = rem + piece * kWave;
            if (fill && in_copy < four_r) store_score(row0, (uint32_t)(kk * four_r + in_copy), moc_move_score{-1, -1});
          }
        }
      }
    }
    // ---- best move of the candidate
    if (out_best) {
      // the lane's index, counted here from a full mask: nothing of it is kept in a register
      // across the scoring, and the thread index need not be fetched back behind the table's stores
      const int own = (int)__builtin_amdgcn_mbcnt_hi(~0u, __builtin_amdgcn_mbcnt_lo(~0u, 0u)) << 2;
#pragma unroll
      for (int off = kWave / 2; off > 0; off >>= 1) {
        Best o;   // of lane ^ off
        const int from = own ^ (off << 2);
        o.viol = __builtin_amdgcn_ds_bpermute(from, best.viol);
        o.peak = __builtin_amdgcn_ds_bpermute(from, best.peak);
        o.move = __builtin_amdgcn_ds_bpermute(from, best.move);
        if (better(o, best)) best = o;
      }
      if (own == 0) {
        L.scratch[wave_ * 4 + 0] = best.viol;
        L.scratch[wave_ * 4 + 1] = best.peak;
        L.scratch[wave_ * 4 + 2] = best.move;
      }
      __syncthreads();
      if (own == 0 && wave_ == 0) {
        Best all{0, 0, -1};
        for (int w = 0; w < kNW; ++w) {
          const Best o{L.scratch[w * 4], L.scratch[w * 4 + 1], L.scratch[w * 4 + 2]};
          if (better(o, all)) all = o;
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



// ---------------------------------------------------------------------------------------------
// moc_eval_toggles: every candidate that differs from the base in one active flag.  The base
// is staged as above (packed intervals, profile with prefix and suffix maxima, start bitmaps);
// the maximum of the profile over a copy's whole interval comes from maxima over blocks of 32
// positions.  One lane per copy: violations' = violations + f(copy with the flag flipped) -
// f(copy as it is) + what Eq. (6) and Eq. (7) see of the flip, with f = node_part (see
// toggle_delta); peak' from the interval the copy gives up or takes; duration' = duration -+ w_v.
// f(copy with its active flag flipped) - f(copy as it is), f = node_part, in one walk over
// the node's edges: the flip makes a well-formed copy leave or join the live copies of v
// (an ill-formed one only starts or stops counting as such).
__device__ __forceinline__ int toggle_delta(const Adj& g, int C, const uint32_t* __restrict__ packed, int v, int i,
                                            bool was, bool well, int s, int e) {
  if (!well) return was ? -1 : 1;   // Eq. (2)/(8)
  const int sign = was ? -1 : 1;    // the copy leaves (-1) or joins (+1)
  // Eq. (3) among the live copies of v, with and without copy i
  int with = 0, without = 0, end_with = -1, end_without = -1;
  for (int j = 0; j < C; ++j) {
    const uint32_t p = j == i ? pack_copy(true, s, e) : packed[v * C + j];
    if (!live_of(p)) continue;
    const int start = (int)(p & 0xFFFFu), end = (int)(p >> 16);
    with += end_with > start ? 1 : 0;
    end_with = end;
    if (j != i) {
      without += end_without > start ? 1 : 0;
      end_without = end;
    }
  }
  int delta = sign * (with - without);
  // Eq. (5), the copy as consumer: its inputs count while it is live
  for (int q = g.in_ptr[v]; q < g.in_ptr[v + 1]; ++q) {
    const int u = g.in_idx[q];
    bool cov = false;
    for (int j = 0; j < C; ++j) cov = cov || covers1(packed[u * C + j], (uint32_t)s);
    delta += cov ? 0 : sign;
  }
  // Eq. (5), node v as provider: the consumer copies that only this copy covers
  for (int q = g.out_ptr[v]; q < g.out_ptr[v + 1]; ++q) {
    const int w = g.out_idx[q];
    for (int jw = 0; jw < C; ++jw) {
      const int x = (int)(packed[w * C + jw] & 0xFFFFu);
      if (x == 0xFFFF || !(s < x && x <= e)) continue;
      bool others = false;
      for (int j = 0; j < C; ++j) others = others || (j != i && covers1(packed[v * C + j], (uint32_t)x));
      delta -= others ? 0 : sign;
    }
  }
  return delta;
}

// max(a[from..to]), from <= to; eight reads in flight at a time (re-reading the last element
// changes no maximum).
__device__ __forceinline__ int range_max8(const int32_t* a, int from, int to) {
  int m = 0;
  for (int t = from; t <= to; t += 8) {
    int x[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) x[j] = a[min(t + j, to)];
    m = max(max(max(m, x[0]), max(x[1], x[2])), max(max(x[3], x[4]), max(max(x[5], x[6]), x[7])));
  }
  return m;
}

// Maxima of the profile over blocks of 32 positions, as a table for range queries:
// level l holds, at i, the maximum over the blocks i .. i + 2^l - 1 (level 0: the blocks).
struct BlockMax {
  const int32_t* level0;
  int blocks;
  __device__ __forceinline__ int over(int first, int last) const {   // blocks [first, last), first < last
    const int l = 31 - __clz(last - first);
    const int32_t* row = level0 + l * blocks;
    return max(row[first], row[last - (1 << l)]);
  }
};

// max(profile[s..e]), s <= e: whole blocks from the table, the rest position by position.
__device__ __forceinline__ int interval_max(const int32_t* profile, const BlockMax& bm, int s, int e) {
  if (e - s < 64) return range_max8(profile, s, e);
  const int first_block = (s + 31) >> 5, last_block = (e + 1) >> 5;   // whole blocks [first, last): at least one
  int top = bm.over(first_block, last_block);
  if (s < 32 * first_block) top = max(top, range_max8(profile, s, 32 * first_block - 1));
  if (32 * last_block <= e) top = max(top, range_max8(profile, 32 * last_block, e));
  return top;
}

// Number of x in [s, e] with profile[x] >= bound.  Whole blocks whose maximum stays below the
// bound are passed over: few blocks come near the peak, and the ranges are long.
__device__ __forceinline__ int count_reaching(const int32_t* profile, const BlockMax& bm, int s, int e, int bound) {
  int cnt = 0;
  const int first_block = (s + 31) >> 5, last_block = (e + 1) >> 5;   // whole blocks [first, last)
  if (first_block >= last_block) {
    for (int x = s; x <= e; ++x) cnt += profile[x] >= bound ? 1 : 0;
    return cnt;
  }
  for (int x = s; x < 32 * first_block; ++x) cnt += profile[x] >= bound ? 1 : 0;
  for (int blk = first_block; blk < last_block; ++blk) {
    if (bm.level0[blk] < bound) continue;
    for (int x = 32 * blk; x < 32 * blk + 32; ++x) cnt += profile[x] >= bound ? 1 : 0;
  }
  for (int x = 32 * last_block; x <= e; ++x) cnt += profile[x] >= bound ? 1 : 0;
  return cnt;
}

// Positions at which the base's profile reaches its peak, countable over any range.
struct PeakCount {
  const uint32_t* bits;
  const int32_t* before;   // per word: such positions in the words below it
  int total;
  __device__ __forceinline__ int up_to(int x) const {   // in [0, x]
    return before[x >> 5] + (int)__popc(bits[x >> 5] & (0xFFFFFFFFu >> (31 - (x & 31))));
  }
  __device__ __forceinline__ int within(int lo, int hi) const {   // in [lo, hi], 1 <= lo <= hi
    return up_to(hi) - up_to(lo - 1);
  }
};

// The cut-and-recompute move for the in-edge (u, v) and copy i of the consumer (see
// moc_eval_cuts in moccasin.h): copy k of u, the last-starting live copy that covers the
// consumer's start t, keeps [s_k, last use before p]; the lowest inactive copy j of u takes
// [p, e_k], p the last position in (s_k, t) where no live copy starts and all inputs of u are
// held.  Only Eq. (3) among the copies of u and Eq. (7) (when j is copy 0) can change: every
// consumer that k covered is covered by one of the two pieces, since no live consumer starts
// in (last use, p], and the new computation finds its inputs by the choice of p.  The profile
// loses m_u on (last use, p).
struct Cut {
  int k, j;        // copy of u that is cut, copy of u that becomes active
  int sk, ek;      // interval of copy k as it stands
  int p;           // start of the recomputation
  int last_use;    // new end of copy k
};

// Which copies and positions the move for producer u and the given consumer copy involves;
// false if it is not applicable.  Reads the packed copies and the start bitmap of L.
// Is node w held at position x (a live copy with s < x <= e)?
__device__ __forceinline__ bool held_at(int C, const uint32_t* __restrict__ packed, int w, int x) {
  bool held = false;
  for (int q = 0; q < C; ++q) held = held || covers1(packed[w * C + q], (uint32_t)x);
  return held;
}

// The live copy of w with the largest end below x, the highest index among equals; -1 if none.
__device__ __forceinline__ int copy_to_keep(int C, const uint32_t* __restrict__ packed, int w, int x, int* end_out) {
  int best = -1, best_end = -1;
  for (int q = 0; q < C; ++q) {
    const uint32_t pw = packed[w * C + q];
    if (live_of(pw) && (int)(pw >> 16) < x && (int)(pw >> 16) >= best_end) {
      best = q;
      best_end = (int)(pw >> 16);
    }
  }
  *end_out = best_end;
  return best;
}

// Calls f(w, q, end) for every predecessor w of u that is not held at p: q is the copy of w that
// the move keeps until p, `end` its end as it stands.  A predecessor listed several times is
// visited once (after the first visit it is held).
template <typename Fn>
__device__ __forceinline__ void for_each_kept_input(const Adj& g, int C, const uint32_t* __restrict__ packed, int u,
                                                    int p, Fn f) {
  const int y0 = g.in_ptr[u], y1 = g.in_ptr[u + 1];
  for (int y = y0; y < y1; ++y) {
    const int w = g.in_idx[y];
    if (held_at(C, packed, w, p)) continue;
    bool seen = false;
    for (int z = y0; z < y; ++z) seen = seen || g.in_idx[z] == w;
    if (seen) continue;
    int end;
    const int q = copy_to_keep(C, packed, w, p, &end);
    f(w, q, end);
  }
}

// mode 0: the recomputation waits where all inputs of u are held.  mode 1: it goes to the last free
// position at which every input is held or has an earlier copy that can be kept until there.
__device__ __forceinline__ bool find_cut(const Adj& g, int C, const NbLds& L, const uint8_t* active_row, int u,
                                         int consumer_copy, int mode, Cut* cut) {
  const uint32_t mine = L.packed[consumer_copy];
  if (!live_of(mine)) return false;
  const uint32_t t = mine & 0xFFFFu;
  int k = -1, j = -1, sk = -1, ek = 0;
  for (int q = 0; q < C; ++q) {
    const uint32_t pu = L.packed[u * C + q];
    if (covers1(pu, t) && (int)(pu & 0xFFFFu) > sk) {
      k = q;
      sk = (int)(pu & 0xFFFFu);
      ek = (int)(pu >> 16);
    }
    if (j < 0 && active_row[u * C + q] == 0) j = q;
  }
  if (k < 0 || j < 0) return false;
  // the last position below t that is free (by words of the start bitmap) and at which every
  // input of u is held; where an input is missing, the search resumes at the end of the
  // nearest earlier copy of that input
  int p = -1;
  for (int hi = (int)t - 1; hi > sk;) {
    int pos = -1;
    for (int x = hi; x > sk;) {
      const uint32_t free_bits = ~L.occ1[x >> 5] & (0xFFFFFFFFu >> (31 - (x & 31)));
      if (free_bits) {
        pos = (x & ~31) + 31 - __clz(free_bits);
        break;
      }
      x = (x & ~31) - 1;
    }
    if (pos <= sk) return false;
    if (mode == 1) {
      bool ok = true;
      for (int y = g.in_ptr[u]; y < g.in_ptr[u + 1] && ok; ++y) {
        const int w = g.in_idx[y];
        int end;
        ok = held_at(C, L.packed, w, pos) || copy_to_keep(C, L.packed, w, pos, &end) >= 0;
      }
      if (ok) {
        p = pos;
        break;
      }
      hi = pos - 1;
      continue;
    }
    int resume = pos;
    for (int y = g.in_ptr[u]; y < g.in_ptr[u + 1]; ++y) {
      const int w = g.in_idx[y];
      bool held = false;
      int below = -1;
      for (int q = 0; q < C; ++q) {
        const uint32_t pw = L.packed[w * C + q];
        held = held || covers1(pw, (uint32_t)pos);
        if (live_of(pw) && (int)(pw >> 16) < pos) below = max(below, (int)(pw >> 16));
      }
      if (!held) resume = min(resume, below);
    }
    if (resume == pos) {
      p = pos;
      break;
    }
    hi = resume;
  }
  if (p <= sk) return false;
  int last_use = sk;
  for (int y = g.out_ptr[u]; y < g.out_ptr[u + 1]; ++y) {
    const int w = g.out_idx[y];
    for (int q = 0; q < C; ++q) {
      const int x = (int)(L.packed[w * C + q] & 0xFFFFu);   // 0xFFFF (not live) is above every p
      if (x > sk && x < p) last_use = max(last_use, x);
    }
  }
  *cut = Cut{k, j, sk, ek, p, last_use};
  return true;
}

__device__ __forceinline__ bool score_cut(const Adj& g, int C, int T, const NbLds& L, const BlockMax& block_max,
                                          const uint8_t* __restrict__ active_row, int u, int consumer_copy,
                                          int base_viol, int base_peak, const PeakCount& at_peak, int mode,
                                          int* viol_out, int* peak_out, int* at_peak_out) {
  Cut cut;
  if (!find_cut(g, C, L, active_row, u, consumer_copy, mode, &cut)) return false;
  const int k = cut.k, j = cut.j, sk = cut.sk, ek = cut.ek, p = cut.p, last_use = cut.last_use;
  int vv = base_viol;
  // Eq. (3) among the live copies of u, before and after
  int before = 0, after = 0, end_before = -1, end_after = -1;
  for (int q = 0; q < C; ++q) {
    const uint32_t pu = L.packed[u * C + q];
    if (live_of(pu)) {
      before += end_before > (int)(pu & 0xFFFFu) ? 1 : 0;
      end_before = (int)(pu >> 16);
    }
    const uint32_t now = q == k ? pack_copy(true, sk, last_use) : q == j ? pack_copy(true, p, ek) : pu;
    if (live_of(now)) {
      after += end_after > (int)(now & 0xFFFFu) ? 1 : 0;
      end_after = (int)(now >> 16);
    }
  }
  vv += after - before;
  // Eq. (5): the inputs of the new computation are held at p by the choice of p
  if (j == 0) --vv;   // Eq. (7)
  int pk = base_peak, at = at_peak.total;
  // mode 1: the inputs that are kept until p.  lo = the lowest position whose memory changes.
  // The first kKept of them are noted (end, size) for the walk below, which looks at each of them
  // once per step: finding them again every time costs a pass over the in-edges of u with
  // several reads per edge.
  constexpr int kKept = 8;
  int kept_end[kKept], kept_size[kKept];
#pragma unroll
  for (int s = 0; s < kKept; ++s) { kept_end[s] = 0; kept_size[s] = 0; }
  int n_kept = 0, lo = last_use + 1;
  if (mode == 1)
    for_each_kept_input(g, C, L.packed, u, p, [&](int w, int q, int end) {
      const int m_w = g.size_of(w);
#pragma unroll
      for (int s = 0; s < kKept; ++s)
        if (s == n_kept) { kept_end[s] = end; kept_size[s] = m_w; }
      ++n_kept;
      lo = min(lo, end + 1);
      // Eq. (3): the kept copy against the next live copy of its node
      for (int c = q + 1; c < C; ++c) {
        const uint32_t nx = L.packed[w * C + c];
        if (live_of(nx)) {
          const int sn = (int)(nx & 0xFFFFu);
          vv += (p > sn ? 1 : 0) - (end > sn ? 1 : 0);
          break;
        }
      }
      // Eq. (5): consumers of w that start in (end, p] are covered now.  None of them was: a copy
      // of w that covered a position in (end, p] would end at or after p and cover p as well
      // (w would be held there), or end in (end, p), and `end` is the largest end below p.
      for (int y = g.out_ptr[w]; y < g.out_ptr[w + 1]; ++y) {
        const int x = g.out_idx[y];
        for (int c = 0; c < C; ++c) {
          const int sx = (int)(L.packed[x * C + c] & 0xFFFFu);   // 0xFFFF if not live: above every p
          if (sx > end && sx <= p) --vv;
        }
      }
    });
  if (n_kept == 0) {
    if (last_use + 1 <= p - 1) {
      const int top = interval_max(L.profile, block_max, last_use + 1, p - 1);
      const int sz = g.size_of(u);
      pk = max(top - sz, max(L.pmax[last_use], L.smax[p]));
      // positions still at the base's peak: those outside the range (all, if nothing is taken away)
      at = pk < base_peak ? 0 : at - (sz > 0 ? at_peak.within(last_use + 1, p - 1) : 0);
    }
  } else {
    // The memory changes on [lo, p]: -m_u on (last_use, p), +m_w on (end_w, p] for every kept
    // input.  All these stretches end at p or just before it, so the change is a step function
    // whose steps are at last_use + 1, at the end_w + 1 and at p: walk it step by step (the next
    // step is found by a pass over the kept inputs; there are few of them).
    const int sz = g.size_of(u);
    int top = max(L.pmax[lo - 1], L.smax[p + 1]);
    int still = at_peak.total - at_peak.within(max(lo, 1), p) - (lo == 0 && bit_at(at_peak.bits, 0) ? 1 : 0);
    for (int from = lo; from <= p;) {
      int next = p + 1, add = 0;   // the step after `from`, and the change on [from, next)
      if (from < last_use + 1) next = min(next, last_use + 1);
      if (from < p) next = min(next, p);
      if (n_kept <= kKept) {
#pragma unroll
        for (int s = 0; s < kKept; ++s) {
          if (s < n_kept) {
            if (kept_end[s] + 1 > from) next = min(next, kept_end[s] + 1);
            else add += kept_size[s];
          }
        }
      } else {
        for_each_kept_input(g, C, L.packed, u, p, [&](int w, int, int end) {
          if (end + 1 > from) next = min(next, end + 1);
          else add += g.size_of(w);
        });
      }
      if (from >= last_use + 1 && from < p) add -= sz;
      const int here = interval_max(L.profile, block_max, from, next - 1);
      top = max(top, here + add);
      // positions of [from, next) that reach the base's peak afterwards
      if (add == 0) {
        still += at_peak.within(max(from, 1), next - 1) + (from == 0 && bit_at(at_peak.bits, 0) ? 1 : 0);
      } else if (add > 0 && here + add >= base_peak) {
        still += count_reaching(L.profile, block_max, from, next - 1, base_peak - add);
      }
      from = next;
    }
    pk = top;
    at = pk < base_peak ? 0 : still;
  }
  *viol_out = vv;
  *peak_out = pk;
  *at_peak_out = at;
  return true;
}

struct TgLayout {
  int T_pad, bit_words, blocks;
  int levels;    // of the table of block maxima: 2^(levels - 1) <= blocks
  int adj_off;   // word offset of the adjacency lists and sizes in LDS, 0 if they stay in global memory
  int bytes;
};

TgLayout tg_layout(int T, int n, int m, int max_lds) {
  TgLayout l;
  l.T_pad = (T + 3) & ~3;
  l.bit_words = (T + 31) / 32;
  l.blocks = (T + 31) / 32;
  l.levels = 1;
  while ((2 << (l.levels - 1)) <= l.blocks) ++l.levels;
  // profile, prefix max, suffix max (with sentinels), packed, block maxima, two start bitmaps, the
  // bitmap of the positions at the peak with its running count per word, scratch, and a queue
  // of 128 moves per wave
  const int words = 4 * l.T_pad + 8 + l.levels * l.blocks + 4 * l.bit_words + 8 * kNW + 16 + 2 * kWave * kNW;
  l.adj_off = 0;
  l.bytes = 4 * words;
  // A lane walks its node's edges one after the other: from LDS whenever the lists fit (the
  // latency of global memory per edge costs more than the second workgroup per CU brings).
  const int with_adj = 4 * (words + 2 * (n + 1) + 2 * m + n);
  if (with_adj <= max_lds) {
    l.adj_off = words;
    l.bytes = with_adj;
  }
  return l;
}

template <bool ADJ_LDS, bool CUTS>
__global__ __launch_bounds__(kNT) void toggles_kernel(GraphView g, int64_t B, const int32_t* __restrict__ starts,
                                                      const int32_t* __restrict__ ends,
                                                      const uint8_t* __restrict__ active,
                                                      moc_toggle_score* __restrict__ out,
                                                      moc_best_move* __restrict__ out_best, int improving,
                                                      int mode, TgLayout lay) {
  extern __shared__ uint32_t nb_raw[];
  NbLds L{};
  L.profile = reinterpret_cast<int32_t*>(nb_raw);
  L.pmax = L.profile + lay.T_pad + 4;   // pmax[-1] = 0
  L.smax = L.pmax + lay.T_pad;          // smax[T] = 0
  L.packed = reinterpret_cast<uint32_t*>(L.smax + lay.T_pad + 4);
  int32_t* const block_max = reinterpret_cast<int32_t*>(L.packed + lay.T_pad);
  L.occ1 = reinterpret_cast<uint32_t*>(block_max + lay.levels * lay.blocks);
  const BlockMax block_table{block_max, lay.blocks};
  L.occ2 = L.occ1 + lay.bit_words;
  uint32_t* const peak_bits = L.occ2 + lay.bit_words;        // bit t: the profile reaches the base's peak at t
  int32_t* const peak_before = reinterpret_cast<int32_t*>(peak_bits + lay.bit_words);   // such positions in earlier words
  L.scratch = reinterpret_cast<int32_t*>(peak_before + lay.bit_words);
  int32_t* const counts = L.scratch + 8 * kNW;   // [0] base violations, [1] base duration
  int32_t* const queue = counts + 16;            // 2 * kWave moves per wave (the descent's sieve)
  const int tid = threadIdx.x;
  const int T = g.T, C = g.C;
  Adj A{g.in_ptr, g.in_idx, g.out_ptr, g.out_idx, reinterpret_cast<const int32_t*>(g.size_dur), 2};
  if constexpr (ADJ_LDS) {
    int32_t* a = reinterpret_cast<int32_t*>(nb_raw) + lay.adj_off;
    int32_t* const sizes = a + 2 * (g.n + 1) + 2 * g.m;
    for (int x = tid; x <= g.n; x += kNT) { a[x] = g.in_ptr[x]; a[g.n + 1 + g.m + x] = g.out_ptr[x]; }
    for (int x = tid; x < g.m; x += kNT) { a[g.n + 1 + x] = g.in_idx[x]; a[2 * (g.n + 1) + g.m + x] = g.out_idx[x]; }
    for (int x = tid; x < g.n; x += kNT) sizes[x] = g.size_dur[x].x;
    A = Adj{a, a + g.n + 1, a + g.n + 1 + g.m, a + 2 * (g.n + 1) + g.m, sizes, 1};
    __syncthreads();
  }

  for (int64_t b = blockIdx.x; b < B; b += gridDim.x) {
    const int64_t row = b * T;
    // ---- the base: copies, deltas, starts.  The first kAhead * kNT copies are asked for before
    // the arrays are cleared, all at once and without conditions (as in the kernel above).
    constexpr int kAhead = 4;
    int ahead_s[kAhead], ahead_e[kAhead];
    uint32_t ahead_a[kAhead];
    int2 ahead_sd[kAhead];
    {
      const char* const s_row = reinterpret_cast<const char*>(starts + row);
      const char* const e_row = reinterpret_cast<const char*>(ends + row);
      const char* const a_row = reinterpret_cast<const char*>(active + row);
      int t = tid;   // offsets formed here for every base, not kept in registers across the bases
      asm volatile("" : "+v"(t));
#pragma unroll
      for (int j = 0; j < kAhead; ++j) {
        const uint32_t k = (uint32_t)min(j * kNT + t, T - 1);
        ahead_s[j] = *reinterpret_cast<const int32_t*>(s_row + 4u * k);
        ahead_e[j] = *reinterpret_cast<const int32_t*>(e_row + 4u * k);
        ahead_a[j] = *reinterpret_cast<const uint8_t*>(a_row + k);
        ahead_sd[j] = g.size_dur[k / (uint32_t)C];
      }
    }
    for (int t = tid; t < T; t += kNT) L.profile[t] = 0;
    for (int w = tid; w < 2 * lay.bit_words; w += kNT) L.occ1[w] = 0;
    if (tid < 2) counts[tid] = 0;
    if (tid == 0) { L.pmax[-1] = 0; L.smax[T] = 0; }
    __syncthreads();
    int viol = 0, nlive = 0, dur = 0;
    auto stage = [&](int k, int s, int e, uint32_t flag, int2 sd) {
      const bool act = flag != 0;
      const bool live = act && (uint32_t)s <= (uint32_t)e && (uint32_t)e < (uint32_t)T;
      const int v = k / C;
      L.packed[k] = pack_copy(live, s, e);
      if (k == v * C && !act) ++viol;   // Eq. (7)
      if (act) dur += sd.y;             // Eq. (1)
      if (live) {
        ++nlive;
        const int sz = sd.x;
        atomicAdd(&L.profile[s], sz);
        if (e + 1 < T) atomicSub(&L.profile[e + 1], sz);
        const uint32_t bit = 1u << (s & 31);
        const uint32_t old = atomicOr(&L.occ1[s >> 5], bit);
        if (old & bit) atomicOr(&L.occ2[s >> 5], bit);
      }
    };
#pragma unroll
    for (int j = 0; j < kAhead; ++j) {
      const int k = j * kNT + tid;
      if (k < T) stage(k, ahead_s[j], ahead_e[j], ahead_a[j], ahead_sd[j]);
    }
    for (int k = kAhead * kNT + tid; k < T; k += kNT)
      stage(k, starts[row + k], ends[row + k], active[row + k], g.size_dur[k / C]);
    __syncthreads();
    block_scan<AddOp, false>(L.profile, L.profile, T, L.scratch, tid);   // Eq. (4) per position
    block_max_both_ways(L.profile, L.pmax, L.smax, T, L.scratch, tid);
    for (int x = tid; x < lay.blocks; x += kNT) {
      int m = 0;
      for (int t = 32 * x; t < min(32 * x + 32, T); ++t) m = max(m, L.profile[t]);
      block_max[x] = m;
    }
    for (int l = 1; l < lay.levels; ++l) {
      __syncthreads();
      const int half = 1 << (l - 1);
      const int32_t* below = block_max + (l - 1) * lay.blocks;
      for (int x = tid; x + 2 * half <= lay.blocks; x += kNT) block_max[l * lay.blocks + x] = max(below[x], below[x + half]);
    }
    // ---- the violations of the base, each instance once (as pass 1 of the kernel above)
    for (int k = tid; k < T; k += kNT) {
      const uint32_t mine = L.packed[k];
      if (!live_of(mine)) {
        viol += active[row + k] != 0 ? 1 : 0;   // Eq. (2)/(8)
        continue;
      }
      const int v = k / C, i = k - v * C;
      const int s = (int)(mine & 0xFFFFu), e = (int)(mine >> 16);
      for (int j = i + 1; j < C; ++j) {   // Eq. (3)
        const uint32_t p = L.packed[v * C + j];
        if (live_of(p)) {
          viol += e > (int)(p & 0xFFFFu) ? 1 : 0;
          break;
        }
      }
      for (int q = A.in_ptr[v]; q < A.in_ptr[v + 1]; ++q) {   // Eq. (5)
        const int u = A.in_idx[q];
        bool cov = false;
        for (int j = 0; j < C; ++j) cov = cov || covers1(L.packed[u * C + j], (uint32_t)s);
        viol += cov ? 0 : 1;
      }
    }
    int distinct = 0;
    for (int w = tid; w < lay.bit_words; w += kNT) distinct += __popc(L.occ1[w]);
    atomicAdd(&counts[0], viol + nlive - distinct);   // Eq. (6): live copies - distinct starts
    atomicAdd(&counts[1], dur);
    __syncthreads();
    const int base_viol = counts[0], base_dur = counts[1], base_peak = L.pmax[T - 1];

    if constexpr (CUTS) {
      // ---- where the base is at its peak: a wave takes 64 positions at a time (two words of
      // the bitmap by one ballot), then one wave turns the words' counts into running counts
      {
        const int lane = tid & (kWave - 1), wave = tid / kWave;
        for (int t0 = wave * kWave; t0 < 32 * lay.bit_words; t0 += kNT) {
          const int t = t0 + lane;
          const uint64_t hit = __ballot(t < T && L.profile[t] == base_peak);
          if (lane == 0) {
            peak_bits[t0 >> 5] = (uint32_t)hit;
            if ((t0 >> 5) + 1 < lay.bit_words) peak_bits[(t0 >> 5) + 1] = (uint32_t)(hit >> 32);
          }
        }
        __syncthreads();
        if (wave == 0) {
          int carry = 0;
          for (int w0 = 0; w0 < lay.bit_words; w0 += kWave) {
            const int w = w0 + lane;
            const int mine = w < lay.bit_words ? (int)__popc(peak_bits[w]) : 0;
            int inc = mine;
#pragma unroll
            for (int off = 1; off < kWave; off <<= 1) {
              const int o = __shfl_up(inc, off);
              if (lane >= off) inc += o;
            }
            if (w < lay.bit_words) peak_before[w] = carry + inc - mine;
            carry += __shfl(inc, kWave - 1);
          }
        }
        __syncthreads();
      }
      const PeakCount at_peak{peak_bits, peak_before,
                              peak_before[lay.bit_words - 1] + (int)__popc(peak_bits[lay.bit_words - 1])};
      // ---- one lane per in-edge and copy of its consumer; the best move is the applicable one
      // that minimises (violations, peak, positions left at the base's peak, index)
      const int64_t out_row = b * ((int64_t)g.m * C);
      uint32_t best_viol = 0xFFFFFFFFu, best_peak = 0xFFFFFFFFu;
      int best_at = 0x7FFFFFFF, best_q = -1;
      auto take = [&](uint32_t ov, uint32_t op, int oa, int oq) {
        if (oq < 0) return;
        if (best_q < 0 || ov < best_viol ||
            (ov == best_viol &&
             (op < best_peak || (op == best_peak && (oa < best_at || (oa == best_at && oq < best_q)))))) {
          best_viol = ov;
          best_peak = op;
          best_at = oa;
          best_q = oq;
        }
      };
      auto score = [&](int q) {
        const int x = q / C, i = q - x * C;
        const int u = A.in_idx[x];
        const int consumer_copy = (int)(g.edge_pair_c[x] >> 16) + i;
        moc_toggle_score sc{-1, -1, 0};
        int vv, pk, at;
        if (score_cut(A, C, T, L, block_table, active + row, u, consumer_copy, base_viol, base_peak, at_peak, mode, &vv,
                      &pk, &at)) {
          sc.violations = vv;
          sc.peak = pk;
          sc.duration = (int64_t)base_dur + g.size_dur[u].y;
          take((uint32_t)vv, (uint32_t)pk, at, q);
        }
        if (out) out[out_row + q] = sc;
      };
      const int n_moves = g.m * C;
      {
        // Most moves are not applicable (the consumer's copy is not live, or no copy of the
        // producer covers it), and scoring is long: each wave sifts its moves by that test, keeps
        // the survivors in a queue of its own and scores them 64 at a time; the others get their
        // "not applicable" score at once.  A descent step from a candidate without violations
        // can, beyond that, only take a move that lowers the peak or the number of positions
        // reaching it: one with such a position inside (s_k, t), which contains the range the
        // move frees; the sieve then lets only those through.
        const bool sift_peak = improving && !out && base_viol == 0;
        const int lane = tid & (kWave - 1), wave = tid / kWave;
        int32_t* const mine_q = queue + wave * (2 * kWave);
        int queued = 0;
        for (int q0 = wave * kWave; q0 < n_moves; q0 += kNT) {
          const int q = q0 + lane;
          bool keep = false;
          if (q < n_moves) {
            const int x = q / C, i = q - x * C;
            const int u = A.in_idx[x];
            const uint32_t consumer = L.packed[(int)(g.edge_pair_c[x] >> 16) + i];
            if (live_of(consumer)) {
              const uint32_t t = consumer & 0xFFFFu;
              int sk = -1;
              for (int c = 0; c < C; ++c) {
                const uint32_t pu = L.packed[u * C + c];
                if (covers1(pu, t)) sk = max(sk, (int)(pu & 0xFFFFu));
              }
              keep = sk >= 0 && (!sift_peak || (sk + 1 <= (int)t - 1 && at_peak.within(sk + 1, (int)t - 1) > 0));
            }
            if (!keep && out) out[out_row + q] = moc_toggle_score{-1, -1, 0};
          }
          const uint64_t kept = __ballot(keep);
          if (keep) mine_q[queued + __popcll(kept & ((1ull << lane) - 1))] = q;
          queued += __popcll(kept);
          __builtin_amdgcn_wave_barrier();
          if (queued >= kWave) {
            queued -= kWave;
            score(mine_q[queued + lane]);
            __builtin_amdgcn_wave_barrier();
          }
        }
        if (lane < queued) score(mine_q[lane]);
      }
      if (out_best) {
#pragma unroll
        for (int off = kWave / 2; off > 0; off >>= 1)
          take(__shfl_xor(best_viol, off), __shfl_xor(best_peak, off), __shfl_xor(best_at, off),
               __shfl_xor(best_q, off));
        __syncthreads();   // the scratch words below were last read by the scans of the staging
        if ((tid & (kWave - 1)) == 0) {
          L.scratch[4 * (tid / kWave)] = (int)best_viol;
          L.scratch[4 * (tid / kWave) + 1] = (int)best_peak;
          L.scratch[4 * (tid / kWave) + 2] = best_at;
          L.scratch[4 * (tid / kWave) + 3] = best_q;
        }
        __syncthreads();
        if (tid == 0) {
          best_q = -1;
          for (int w = 0; w < kNW; ++w)
            take((uint32_t)L.scratch[4 * w], (uint32_t)L.scratch[4 * w + 1], L.scratch[4 * w + 2],
                 L.scratch[4 * w + 3]);
          // a descent step takes the move only if it lowers (violations, max(peak, M)) or, above
          // the budget with both unchanged, leaves fewer positions at the peak
          if (improving && best_q >= 0) {
            const int64_t now = max((int64_t)base_peak, g.budget), then = max((int64_t)best_peak, g.budget);
            const bool better = (int)best_viol < base_viol ||
                                ((int)best_viol == base_viol &&
                                 (then < now || (then == now && base_peak > g.budget && best_at < at_peak.total)));
            if (!better) best_q = -1;
          }
          moc_best_move bm{best_q, best_q < 0 ? 0 : (int)best_viol, best_q < 0 ? 0 : (int64_t)best_peak};
          out_best[b] = bm;
        }
      }
      __syncthreads();
      continue;
    }
    // ---- one lane per copy
    for (int k = tid; k < T; k += kNT) {
      const int v = k / C, i = k - v * C;
      const int s = starts[row + k], e = ends[row + k];
      const bool was = active[row + k] != 0;
      const bool well = (uint32_t)s <= (uint32_t)e && (uint32_t)e < (uint32_t)T;
      const bool live_old = was && well, live_new = !was && well;
      int vv = base_viol + toggle_delta(A, C, L.packed, v, i, was, well, s, e);
      if (live_old && bit_at(L.occ2, s)) --vv;   // Eq. (6): a shared start loses one of its copies
      if (live_new && bit_at(L.occ1, s)) ++vv;   //          or a taken start gains one
      if (i == 0) vv += was ? 1 : -1;            // Eq. (7)
      int pk = base_peak;
      if (well) {   // the copy's interval leaves or joins the profile
        const int top = interval_max(L.profile, block_table, s, e);
        const int sz = A.size_of(v);
        pk = max(max(top + (was ? -sz : sz), 0), max(L.pmax[s - 1], L.smax[e + 1]));
      }
      moc_toggle_score sc;
      sc.violations = vv;
      sc.peak = pk;
      sc.duration = (int64_t)base_dur + (was ? -g.size_dur[v].y : g.size_dur[v].y);
      out[row + k] = sc;
    }
    __syncthreads();
  }
}

using NbKernel = void (*)(GraphView, int64_t, const int32_t*, const int32_t*, const uint8_t*, int, moc_move_score*,
                          moc_best_move*, NbLayout);

template <bool ADJ_LDS, bool WIDE, bool TABLE>
NbKernel pick_copies(int C) {
  switch (C) {
    case 1: return neighbours_kernel<ADJ_LDS, 1, WIDE, TABLE>;
    case 2: return neighbours_kernel<ADJ_LDS, 2, WIDE, TABLE>;
    case 3: return neighbours_kernel<ADJ_LDS, 3, WIDE, TABLE>;
    case 4: return neighbours_kernel<ADJ_LDS, 4, WIDE, TABLE>;
    default: return neighbours_kernel<ADJ_LDS, 0, WIDE, TABLE>;   // C read at run time
  }
}

template <bool ADJ_LDS, bool WIDE>
NbKernel pick_table(int C, bool table) {
  return table ? pick_copies<ADJ_LDS, WIDE, true>(C) : pick_copies<ADJ_LDS, WIDE, false>(C);
}

NbKernel pick_kernel(bool adj_lds, int C, int R, bool table) {
  const bool wide = 2 * R > 31;   // 64-bit displacement masks
  if (adj_lds) return wide ? pick_table<true, true>(C, table) : pick_table<true, false>(C, table);
  return wide ? pick_table<false, true>(C, table) : pick_table<false, false>(C, table);
}

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
  if ((int64_t)g->view.T * 4 * R * 8 > 0xFFFFFFFFll) return MOC_EOVERFLOW;   // byte offsets in a candidate's table are 32 bits
  auto kern = pick_kernel(lay.adj_off != 0, g->view.C, R, out_moves != nullptr);
  int per_cu = 0;
  if (const int rc = moc_kernel_occupancy(g, reinterpret_cast<const void*>(kern), kNT, lay.bytes, false, &per_cu)) return rc;
  const int64_t resident = (int64_t)per_cu * g->num_cu;
  const unsigned grid = (unsigned)(B < resident ? B : resident);
  hipLaunchKernelGGL(kern, dim3(grid), dim3(kNT), lay.bytes, static_cast<hipStream_t>(hip_stream), g->view, B,
                     starts, ends, active, R, out_moves, out_best, lay);
  MOC_HIP(hipGetLastError());
  return MOC_OK;
}

extern "C" int moc_eval_toggles(const moc_graph* g, int64_t B, const int32_t* starts, const int32_t* ends,
                                const uint8_t* active, moc_toggle_score* out, void* hip_stream) {
  if (!g || B < 0) return MOC_EINVAL;
  if (B == 0) return MOC_OK;
  if (!starts || !ends || !active || !out) return MOC_EINVAL;
  if ((((uintptr_t)starts | (uintptr_t)ends) & 3) || ((uintptr_t)out & 7)) return MOC_EINVAL;
  int dev = -1;
  MOC_HIP(hipGetDevice(&dev));
  if (dev != g->device) return MOC_EDEVICE;
  if (g->has_self_loop) return MOC_EINVAL;
  const TgLayout lay = tg_layout(g->view.T, g->view.n, g->view.m, g->max_lds);
  if (lay.bytes > g->max_lds) return MOC_EOVERFLOW;
  auto kern = lay.adj_off ? toggles_kernel<true, false> : toggles_kernel<false, false>;
  int per_cu = 0;
  if (const int rc = moc_kernel_occupancy(g, reinterpret_cast<const void*>(kern), kNT, lay.bytes, false, &per_cu)) return rc;
  const int64_t resident = (int64_t)per_cu * g->num_cu;
  const unsigned grid = (unsigned)(B < resident ? B : resident);
  hipLaunchKernelGGL(kern, dim3(grid), dim3(kNT), lay.bytes, static_cast<hipStream_t>(hip_stream), g->view, B, starts,
                     ends, active, out, static_cast<moc_best_move*>(nullptr), 0, 0, lay);
  MOC_HIP(hipGetLastError());
  return MOC_OK;
}

namespace {

constexpr int kApplyNT = 256;

__global__ void fill_zero_kernel(int32_t* p, int64_t n) {
  const int64_t i = blockIdx.x * (int64_t)blockDim.x + threadIdx.x;
  if (i < n) p[i] = 0;
}

// Applies to each base the move its moc_best_move names (none if move < 0) and counts it.
// One workgroup per base stages what find_cut reads -- packed copies and the start bitmap --
// and one lane edits the three arrays in place.
__global__ __launch_bounds__(kApplyNT) void apply_cuts_kernel(GraphView g, int64_t B, int32_t* starts, int32_t* ends,
                                                              uint8_t* active, const moc_best_move* best,
                                                              int32_t* steps, int mode) {
  extern __shared__ uint32_t ap_raw[];
  const int T = g.T, C = g.C, tid = threadIdx.x;
  const int bit_words = (T + 31) / 32;
  NbLds L{};
  L.packed = ap_raw;
  L.occ1 = ap_raw + T;
  const int64_t b = blockIdx.x;
  if (b >= B) return;
  const int q = best[b].move;
  if (q < 0) return;   // the same for every lane of the workgroup
  const int64_t row = b * T;
  for (int w = tid; w < bit_words; w += kApplyNT) L.occ1[w] = 0;
  __syncthreads();
  for (int k = tid; k < T; k += kApplyNT) {
    const int s = starts[row + k], e = ends[row + k];
    const bool live = active[row + k] != 0 && (uint32_t)s <= (uint32_t)e && (uint32_t)e < (uint32_t)T;
    L.packed[k] = pack_copy(live, s, e);
    if (live) atomicOr(&L.occ1[s >> 5], 1u << (s & 31));
  }
  __syncthreads();
  if (tid == 0) {
    const Adj A{g.in_ptr, g.in_idx, g.out_ptr, g.out_idx, reinterpret_cast<const int32_t*>(g.size_dur), 2};
    const int x = q / C, i = q - x * C;
    const int u = g.in_idx[x];
    Cut cut;
    if (find_cut(A, C, L, active + row, u, (int)(g.edge_pair_c[x] >> 16) + i, mode, &cut)) {
      if (mode == 1)
        for_each_kept_input(A, C, L.packed, u, cut.p, [&](int w, int q, int) { ends[row + w * C + q] = cut.p; });
      ends[row + u * C + cut.k] = cut.last_use;
      starts[row + u * C + cut.j] = cut.p;
      ends[row + u * C + cut.j] = cut.ek;
      active[row + u * C + cut.j] = 1;
      steps[b] += 1;
    }
  }
}

}  // namespace

namespace {

// What the launches of the cuts kernel need, worked out once per call.
struct CutsPlan {
  TgLayout lay;
  void (*kern)(GraphView, int64_t, const int32_t*, const int32_t*, const uint8_t*, moc_toggle_score*, moc_best_move*,
               int, int, TgLayout);
  unsigned grid;
  int apply_bytes;
};

int plan_cuts(const moc_graph* g, int64_t B, bool with_apply, CutsPlan* plan) {
  if (g->has_self_loop) return MOC_EINVAL;
  plan->lay = tg_layout(g->view.T, g->view.n, g->view.m, g->max_lds);
  if (plan->lay.bytes > g->max_lds) return MOC_EOVERFLOW;
  if ((int64_t)g->view.m * g->view.C > 0x7FFFFFFFll) return MOC_EOVERFLOW;
  plan->kern = plan->lay.adj_off ? toggles_kernel<true, true> : toggles_kernel<false, true>;
  int per_cu = 0;
  if (const int rc = moc_kernel_occupancy(g, reinterpret_cast<const void*>(plan->kern), kNT, plan->lay.bytes, false, &per_cu))
    return rc;
  plan->apply_bytes = 4 * (g->view.T + (g->view.T + 31) / 32);
  if (with_apply) {
    int apply_per_cu = 0;   // not used: the call is for the kernel's LDS limit
    if (const int rc = moc_kernel_occupancy(g, reinterpret_cast<const void*>(apply_cuts_kernel), kApplyNT,
                                            plan->apply_bytes, false, &apply_per_cu))
      return rc;
  }
  const int64_t resident = (int64_t)per_cu * g->num_cu;
  plan->grid = (unsigned)(B < resident ? B : resident);
  return MOC_OK;
}

// max_steps times: the best cut of every candidate that improves it, then its application.
void queue_cut_steps(const moc_graph* g, const CutsPlan& plan, int64_t B, int32_t* starts, int32_t* ends,
                     uint8_t* active, int max_steps, int mode, moc_best_move* work_best, int32_t* out_steps,
                     hipStream_t stream) {
  for (int step = 0; step < max_steps; ++step) {
    hipLaunchKernelGGL(plan.kern, dim3(plan.grid), dim3(kNT), plan.lay.bytes, stream, g->view, B, starts, ends, active,
                       static_cast<moc_toggle_score*>(nullptr), work_best, 1, mode, plan.lay);
    hipLaunchKernelGGL(apply_cuts_kernel, dim3((unsigned)B), dim3(kApplyNT), plan.apply_bytes, stream, g->view, B,
                       starts, ends, active, work_best, out_steps, mode);
  }
}

int eval_cuts(const moc_graph* g, int64_t B, const int32_t* starts, const int32_t* ends, const uint8_t* active,
              int mode, moc_cut_score* out_moves, moc_best_move* out_best, void* hip_stream) {
  if (!g || B < 0) return MOC_EINVAL;
  if (!out_moves && !out_best) return MOC_EINVAL;
  if (B == 0) return MOC_OK;
  if (!starts || !ends || !active) return MOC_EINVAL;
  if ((((uintptr_t)starts | (uintptr_t)ends) & 3) || ((uintptr_t)out_moves & 7) || ((uintptr_t)out_best & 7))
    return MOC_EINVAL;
  int dev = -1;
  MOC_HIP(hipGetDevice(&dev));
  if (dev != g->device) return MOC_EDEVICE;
  CutsPlan plan;
  if (const int rc = plan_cuts(g, B, false, &plan)) return rc;
  hipLaunchKernelGGL(plan.kern, dim3(plan.grid), dim3(kNT), plan.lay.bytes, static_cast<hipStream_t>(hip_stream), g->view,
                     B, starts, ends, active, out_moves, out_best, 0, mode, plan.lay);
  MOC_HIP(hipGetLastError());
  return MOC_OK;
}

// ---- merges: the moves of the second phase, scored by the evaluation kernel itself
constexpr int kMergeNT = 256;

__device__ __forceinline__ bool copy_is_live(int s, int e, uint8_t a, int T) {
  return a != 0 && (uint32_t)s <= (uint32_t)e && (uint32_t)e < (uint32_t)T;
}

// The nearest live copy of the same node below copy k (index within the row), -1 if none.
__device__ __forceinline__ int live_copy_below(const int32_t* s, const int32_t* e, const uint8_t* a, int T, int C,
                                               int k) {
  const int first = k - k % C;
  for (int c = k - 1; c >= first; --c)
    if (copy_is_live(s[c], e[c], a[c], T)) return c;
  return -1;
}

// One workgroup per walker: the first K copies, in index order, that are live and have a live
// copy of their node below them, to list[walker][0..K); the rest of the list is -1.
__global__ __launch_bounds__(kMergeNT) void list_merges_kernel(int64_t B, int T, int C, int K,
                                                               const int32_t* __restrict__ starts,
                                                               const int32_t* __restrict__ ends,
                                                               const uint8_t* __restrict__ active,
                                                               int32_t* __restrict__ list) {
  __shared__ int wave_count[kMergeNT / kWave];
  const int64_t b = blockIdx.x;
  const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
  const int32_t* s = starts + b * T;
  const int32_t* e = ends + b * T;
  const uint8_t* a = active + b * T;
  int32_t* out = list + b * K;
  for (int r = tid; r < K; r += kMergeNT) out[r] = -1;
  int found = 0;   // entries written by earlier rounds
  for (int k0 = 0; k0 < T && found < K; k0 += kMergeNT) {
    const int k = k0 + tid;
    const bool mergeable = k < T && copy_is_live(s[k], e[k], a[k], T) && live_copy_below(s, e, a, T, C, k) >= 0;
    const uint64_t hits = __ballot(mergeable);
    __syncthreads();   // the counts of the last round have been read; the -1s above are in place
    if (lane == 0) wave_count[wave] = __popcll(hits);
    __syncthreads();
    int before = found, total = found;
    for (int w = 0; w < kMergeNT / kWave; ++w) {
      if (w < wave) before += wave_count[w];
      total += wave_count[w];
    }
    const int r = before + __popcll(hits & ((1ull << lane) - 1));
    if (mergeable && r < K) out[r] = k;
    found = total;
  }
}

// One workgroup per (walker, entry of its list): the walker's row with that merge applied (the
// copy switched off, the live copy below it kept until the later of the two ends), or the row
// as it is where the list has no entry.
__global__ __launch_bounds__(kMergeNT) void write_merges_kernel(int T, int C, int K, const int32_t* __restrict__ starts,
                                                                const int32_t* __restrict__ ends,
                                                                const uint8_t* __restrict__ active,
                                                                const int32_t* __restrict__ list,
                                                                int32_t* __restrict__ ws, int32_t* __restrict__ we,
                                                                uint8_t* __restrict__ wa) {
  const int64_t idx = blockIdx.x, b = idx / K;
  const int32_t* s = starts + b * T;
  const int32_t* e = ends + b * T;
  const uint8_t* a = active + b * T;
  const int k = list[idx];
  int below = -1, end = 0;
  if (k >= 0) {
    below = live_copy_below(s, e, a, T, C, k);
    end = max(e[below], e[k]);
  }
  for (int x = threadIdx.x; x < T; x += kMergeNT) {
    ws[idx * T + x] = s[x];
    we[idx * T + x] = x == below ? end : e[x];
    wa[idx * T + x] = x == k ? (uint8_t)0 : a[x];
  }
}

// One lane per walker: among the scored merges of its list those whose result is feasible, the
// one with the lowest duration, then the lowest peak, then the lowest copy index, applied in place.
__global__ void select_merges_kernel(int64_t B, int T, int C, int K, int32_t* starts, int32_t* ends, uint8_t* active,
                                     const int32_t* __restrict__ list, const moc_result* __restrict__ results,
                                     int32_t* merges) {
  const int64_t b = blockIdx.x * (int64_t)blockDim.x + threadIdx.x;
  if (b >= B) return;
  int best = -1;
  int64_t best_dur = 0, best_peak = 0;
  for (int r = 0; r < K; ++r) {
    const int k = list[b * K + r];
    if (k < 0) break;
    const moc_result res = results[b * K + r];
    if (!res.feasible) continue;
    if (best < 0 || res.duration < best_dur || (res.duration == best_dur && res.peak < best_peak)) {
      best = k;
      best_dur = res.duration;
      best_peak = res.peak;
    }
  }
  if (best < 0) return;
  int32_t* s = starts + b * T;
  int32_t* e = ends + b * T;
  uint8_t* a = active + b * T;
  const int below = live_copy_below(s, e, a, T, C, best);
  e[below] = max(e[below], e[best]);
  a[best] = 0;
  merges[b] += 1;
}

}  // namespace

extern "C" int moc_search_cuts(const moc_graph* g, int64_t B, int32_t* starts, int32_t* ends, uint8_t* active,
                               int32_t max_steps, moc_best_move* work_best, int32_t* out_steps, void* hip_stream) {
  if (!g || B < 0 || max_steps < 0) return MOC_EINVAL;
  if (B == 0) return MOC_OK;
  if (!starts || !ends || !active || !work_best || !out_steps) return MOC_EINVAL;
  if ((((uintptr_t)starts | (uintptr_t)ends | (uintptr_t)out_steps) & 3) || ((uintptr_t)work_best & 7)) return MOC_EINVAL;
  if (B > 0x7FFFFFFFll) return MOC_EINVAL;
  int dev = -1;
  MOC_HIP(hipGetDevice(&dev));
  if (dev != g->device) return MOC_EDEVICE;
  CutsPlan plan;
  if (const int rc = plan_cuts(g, B, true, &plan)) return rc;
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  hipLaunchKernelGGL(fill_zero_kernel, dim3((unsigned)((B + 255) / 256)), dim3(256), 0, stream, out_steps, B);
  queue_cut_steps(g, plan, B, starts, ends, active, max_steps, 0, work_best, out_steps, stream);
  MOC_HIP(hipGetLastError());
  return MOC_OK;
}

extern "C" int moc_eval_cuts(const moc_graph* g, int64_t B, const int32_t* starts, const int32_t* ends,
                             const uint8_t* active, moc_cut_score* out_moves, moc_best_move* out_best,
                             void* hip_stream) {
  return eval_cuts(g, B, starts, ends, active, 0, out_moves, out_best, hip_stream);
}

extern "C" int moc_eval_cuts_keep(const moc_graph* g, int64_t B, const int32_t* starts, const int32_t* ends,
                                  const uint8_t* active, moc_cut_score* out_moves, moc_best_move* out_best,
                                  void* hip_stream) {
  return eval_cuts(g, B, starts, ends, active, 1, out_moves, out_best, hip_stream);
}

extern "C" int moc_search_two_phase(const moc_graph* g, int64_t B, int32_t* starts, int32_t* ends, uint8_t* active,
                                    int32_t max_cuts, int32_t max_merges, int32_t K, moc_best_move* work_best,
                                    int32_t* work_starts, int32_t* work_ends, uint8_t* work_active,
                                    int32_t* work_list, moc_result* work_results, int32_t* out_cuts,
                                    int32_t* out_merges, void* hip_stream) {
  if (!g || B < 0 || max_cuts < 0 || max_merges < 0 || K < 1) return MOC_EINVAL;
  if (B == 0) return MOC_OK;
  if (!starts || !ends || !active || !work_best || !out_cuts || !out_merges) return MOC_EINVAL;
  if (max_merges > 0 && (!work_starts || !work_ends || !work_active || !work_list || !work_results)) return MOC_EINVAL;
  if ((((uintptr_t)starts | (uintptr_t)ends | (uintptr_t)out_cuts | (uintptr_t)out_merges | (uintptr_t)work_list) & 3) ||
      (((uintptr_t)work_best | (uintptr_t)work_results) & 7))
    return MOC_EINVAL;
  if (((uintptr_t)work_starts | (uintptr_t)work_ends) & 3) return MOC_EINVAL;
  if (B > 0x7FFFFFFFll || (int64_t)B * K > 0x7FFFFFFFll) return MOC_EINVAL;
  int dev = -1;
  MOC_HIP(hipGetDevice(&dev));
  if (dev != g->device) return MOC_EDEVICE;
  CutsPlan plan;
  if (const int rc = plan_cuts(g, B, true, &plan)) return rc;
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  const unsigned blocks = (unsigned)((B + 255) / 256);
  const int T = g->view.T, C = g->view.C;
  hipLaunchKernelGGL(fill_zero_kernel, dim3(blocks), dim3(256), 0, stream, out_cuts, B);
  hipLaunchKernelGGL(fill_zero_kernel, dim3(blocks), dim3(256), 0, stream, out_merges, B);
  // Phase 1: towards the budget by cuts that keep the producer's inputs
  queue_cut_steps(g, plan, B, starts, ends, active, max_cuts, 1, work_best, out_cuts, stream);
  MOC_HIP(hipGetLastError());
  // Phase 2: undo recomputations while the candidate stays within the budget
  for (int step = 0; step < max_merges; ++step) {
    hipLaunchKernelGGL(list_merges_kernel, dim3((unsigned)B), dim3(kMergeNT), 0, stream, B, T, C, (int)K, starts, ends,
                       active, work_list);
    hipLaunchKernelGGL(write_merges_kernel, dim3((unsigned)(B * K)), dim3(kMergeNT), 0, stream, T, C, (int)K, starts,
                       ends, active, work_list, work_starts, work_ends, work_active);
    MOC_HIP(hipGetLastError());
    if (const int rc = moc_eval_batch(g, B * K, work_starts, work_ends, work_active, work_results, hip_stream)) return rc;
    hipLaunchKernelGGL(select_merges_kernel, dim3(blocks), dim3(256), 0, stream, B, T, C, (int)K, starts, ends, active,
                       work_list, work_results, out_merges);
  }
  MOC_HIP(hipGetLastError());
  return MOC_OK;
}

namespace {

// Applies to each base the single-field move its moc_best_move names if that move lowers
// (violations, max(peak, M), peak) against the base's own result, and counts it.
__global__ void apply_moves_kernel(int64_t B, int T, int R, int64_t budget, int32_t* starts, int32_t* ends,
                                   const moc_best_move* best, const moc_result* base, int32_t* steps) {
  const int64_t b = blockIdx.x * (int64_t)blockDim.x + threadIdx.x;
  if (b >= B) return;
  const int q = best[b].move;
  if (q < 0) return;
  const int64_t v1 = best[b].violations, p1 = best[b].peak, v0 = base[b].violations, p0 = base[b].peak;
  const int64_t m1 = max(p1, budget), m0 = max(p0, budget);
  if (!(v1 < v0 || (v1 == v0 && (m1 < m0 || (m1 == m0 && p1 < p0))))) return;
  const int d = q % (2 * R), field = (q / (2 * R)) & 1, k = q / (4 * R);
  const int delta = d < R ? d - R : d - R + 1;
  (field == 0 ? starts : ends)[b * T + k] += delta;
  steps[b] += 1;
}

}  // namespace

extern "C" int moc_search_moves(const moc_graph* g, int64_t B, int32_t* starts, int32_t* ends, const uint8_t* active,
                                int32_t R, int32_t max_steps, moc_result* work_results, moc_best_move* work_best,
                                int32_t* out_steps, void* hip_stream) {
  if (!g || B < 0 || max_steps < 0 || R < 1 || R > 32) return MOC_EINVAL;
  if (B == 0) return MOC_OK;
  if (!starts || !ends || !active || !work_results || !work_best || !out_steps) return MOC_EINVAL;
  if ((((uintptr_t)starts | (uintptr_t)ends | (uintptr_t)out_steps) & 3) ||
      (((uintptr_t)work_best | (uintptr_t)work_results) & 7))
    return MOC_EINVAL;
  if (B > 0x7FFFFFFFll) return MOC_EINVAL;
  int dev = -1;
  MOC_HIP(hipGetDevice(&dev));
  if (dev != g->device) return MOC_EDEVICE;
  if (g->has_self_loop) return MOC_EINVAL;
  const NbLayout lay = nb_layout(g->view.T, g->view.n, g->view.m, g->max_lds);
  if (lay.bytes > g->max_lds) return MOC_EOVERFLOW;
  if ((int64_t)g->view.T * 4 * R * 8 > 0xFFFFFFFFll) return MOC_EOVERFLOW;
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  const unsigned blocks = (unsigned)((B + 255) / 256);
  hipLaunchKernelGGL(fill_zero_kernel, dim3(blocks), dim3(256), 0, stream, out_steps, B);
  for (int step = 0; step < max_steps; ++step) {
    int rc = moc_eval_batch(g, B, starts, ends, active, work_results, hip_stream);
    if (rc != MOC_OK) return rc;
    rc = moc_eval_neighbours(g, B, starts, ends, active, R, nullptr, work_best, hip_stream);
    if (rc != MOC_OK) return rc;
    hipLaunchKernelGGL(apply_moves_kernel, dim3(blocks), dim3(256), 0, stream, B, g->view.T, (int)R, g->view.budget,
                       starts, ends, work_best, work_results, out_steps);
  }
  MOC_HIP(hipGetLastError());
  return MOC_OK;
}

