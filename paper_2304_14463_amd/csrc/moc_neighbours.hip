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
// Pass 1 stores f(old copy) per copy.  Pass 2 runs one lane per (copy, field):
// the lane walks the edges of its node once per 16 displacements and scores
// them side by side (what does not depend on the displacement is computed
// once), then writes its 2R scores, 16R contiguous bytes.  A wave takes 64
// consecutive nodes with the same copy index and field.  The adjacency lists
// are kept in LDS when they fit beside the five T-word arrays.
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
  // the CSR lists both ways, if there is room: every move walks the edges of its node
  const int with_adj = 4 * (words + 2 * (n + 1) + 2 * m);
  if (with_adj <= max_lds) {
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
  int32_t* fold;
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

constexpr int kDisp = 16;   // displacements a lane scores at a time

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
  int vv = base_viol - L.fold[k] + node_part(g, C, L.packed, v, i, true, live_new, s2, e2);
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

template <bool ADJ_LDS>
__global__ __launch_bounds__(kNT) void neighbours_kernel(GraphView g, int64_t B, const int32_t* __restrict__ starts,
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
  L.fold = reinterpret_cast<int32_t*>(L.packed + lay.T_pad);
  L.occ1 = reinterpret_cast<uint32_t*>(L.fold + lay.T_pad);
  L.occ2 = L.occ1 + lay.bit_words;
  L.scratch = reinterpret_cast<int32_t*>(L.occ2 + lay.bit_words);
  const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
  const int T = g.T, C = g.C;
  const int moves_per_cand = T * 4 * R;
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
    if (tid < 4) L.scratch[8 * kNW + tid] = 0;
    __syncthreads();
    int viol = 0, nlive = 0;
    for (int k = tid; k < T; k += kNT) {
      const int s = starts[row + k], e = ends[row + k];
      const bool act = active[row + k] != 0;
      const bool live = act && (uint32_t)s <= (uint32_t)e && (uint32_t)e < (uint32_t)T;
      const int v = k / C;
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

    // ---- pass 1: f(old copy) per copy; base violation count
    for (int k = tid; k < T; k += kNT) {
      const int v = k / C, i = k - v * C;
      const int s = starts[row + k], e = ends[row + k];
      const bool act = active[row + k] != 0;
      const bool live = live_of(L.packed[k]);
      L.fold[k] = act ? node_part(A, C, L.packed, v, i, act, live, s, e) : 0;
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
    int distinct = 0;
    for (int w = tid; w < lay.bit_words; w += kNT) distinct += __popc(L.occ1[w]);
    atomicAdd(&L.scratch[8 * kNW], viol + nlive - distinct);   // Eq. (6): live copies - distinct starts
    __syncthreads();
    const int base_viol = L.scratch[8 * kNW];
    const int base_peak = L.pmax[T - 1];

    // ---- pass 2: one lane per (copy, field); it scores the 2R displacements of that field.
    // A wave takes 64 consecutive nodes, one copy index and one field at a time: the field and
    // the copy index are the same in all its lanes, and a copy index that is rarely active
    // costs the wave next to nothing.
    Best best{0, 0, -1};
    const int two_r = 2 * R;
    const int node_blocks = (g.n + kWave - 1) / kWave;
    for (int blk = wave; blk < node_blocks * C * 2; blk += kNW) {
      const int field = blk & 1, i = (blk >> 1) % C, v = ((blk >> 1) / C) * kWave + lane;
      if (v >= g.n) continue;
      const int k = v * C + i, pf = 2 * k + field;
      const int s = starts[row + k], e = ends[row + k];
      const bool act = active[row + k] != 0;
      const uint32_t mine = L.packed[k];
      const int sz = g.size_dur[v].x;
      moc_move_score* const dst = out_moves ? out_moves + (b * (int64_t)moves_per_cand + (int64_t)pf * two_r) : nullptr;
      if (!act || !live_of(mine)) {
        // not applicable, or a copy that is ill-formed now (rare): move by move
        for (int d = 0; d < two_r; ++d) {
          const int delta = d < R ? d - R : d - R + 1;
          const int moved = (field == 0 ? s : e) + delta;
          moc_move_score sc{-1, -1};
          if (act && moved >= 0 && moved < T) {
            score_move(A, C, sz, L, T, v, i, field, s, e, moved, base_viol, base_peak, sc);
            const Best cand{sc.violations, sc.peak, pf * two_r + d};
            if (better(cand, best, g.budget)) best = cand;
          }
          if (dst) dst[d] = sc;
        }
        continue;
      }
      // ---- copy k is live: what does not depend on the displacement
      // Eq. (3): the live neighbours of copy i among the copies of v, and the violations
      // between other consecutive live copies
      int prev_end = -1, next_start = 0x7FFFFFFF, order_others = 0;
      {
        int pe = -1;
        bool have = false;
        for (int j = 0; j < i; ++j) {
          const uint32_t p = L.packed[v * C + j];
          if (!live_of(p)) continue;
          if (have && pe > (int)(p & 0xFFFFu)) ++order_others;
          pe = (int)(p >> 16);
          have = true;
        }
        if (have) prev_end = pe;
        have = false;
        for (int j = i + 1; j < C; ++j) {
          const uint32_t p = L.packed[v * C + j];
          if (!live_of(p)) continue;
          if (!have) next_start = (int)(p & 0xFFFFu);
          else if (pe > (int)(p & 0xFFFFu)) ++order_others;
          pe = (int)(p >> 16);
          have = true;
        }
      }
      const int order_without = (prev_end >= 0 && next_start != 0x7FFFFFFF && prev_end > next_start) ? 1 : 0;
      const int start_twice = bit_at(L.occ2, s) ? 1 : 0;
      const int fixed = base_viol - L.fold[k] + order_others - start_twice;
      const int in_lo = A.in_ptr[v], in_hi = A.in_ptr[v + 1], out_lo = A.out_ptr[v], out_hi = A.out_ptr[v + 1];
      int lost_all = -1;   // peak inside [s, e] without this copy: computed when first needed
      for (int d0 = 0; d0 < two_r; d0 += kDisp) {
        int vv[kDisp], pk[kDisp];
        // ---- violations
#pragma unroll
        for (int dd = 0; dd < kDisp; ++dd) {
          const int d = d0 + dd, delta = d < R ? d - R : d - R + 1;
          const int s2 = field == 0 ? s + delta : s, e2 = field == 0 ? e : e + delta;
          const bool live_new = s2 >= 0 && s2 <= e2 && e2 < T;
          int c = fixed;
          if (live_new) {
            c += (prev_end > s2 ? 1 : 0) + (e2 > next_start ? 1 : 0);                  // Eq. (3) around the moved copy
            c += s2 == s ? start_twice : (bit_at(L.occ1, s2) ? 1 : 0);               // Eq. (6)
          } else {
            c += 1 + order_without;                                                   // Eq. (2)/(8); Eq. (3) across the gap
          }
          vv[dd] = c;
        }
        // Eq. (5), the copy as consumer: every in-edge whose provider does not cover the start
        if (field == 1) {
          int uncovered = 0;
          for (int q = in_lo; q < in_hi; ++q) {
            const int u = A.in_idx[q];
            bool cov = false;
            for (int j = 0; j < C; ++j) cov = cov || covers1(L.packed[u * C + j], (uint32_t)s);
            uncovered += cov ? 0 : 1;
          }
#pragma unroll
          for (int dd = 0; dd < kDisp; ++dd) {
            const int d = d0 + dd, delta = d < R ? d - R : d - R + 1;
            const int e2 = e + delta;
            vv[dd] += (s <= e2 && e2 < T) ? uncovered : 0;
          }
        } else {
          for (int q = in_lo; q < in_hi; ++q) {
            const int u = A.in_idx[q];
            uint32_t covered = 0;   // bit dd: some copy of u covers the start moved by displacement dd
            for (int j = 0; j < C; ++j) {
              const uint32_t pu = L.packed[u * C + j];
#pragma unroll
              for (int dd = 0; dd < kDisp; ++dd) {
                const int d = d0 + dd, delta = d < R ? d - R : d - R + 1;
                const int s2 = s + delta;
                covered |= (s2 >= 0 && covers1(pu, (uint32_t)s2)) ? 1u << dd : 0u;
              }
            }
#pragma unroll
            for (int dd = 0; dd < kDisp; ++dd) {
              const int d = d0 + dd, delta = d < R ? d - R : d - R + 1;
              const int s2 = s + delta;
              vv[dd] += (s2 >= 0 && s2 <= e && !(covered >> dd & 1u)) ? 1 : 0;
            }
          }
        }
        // Eq. (5), node v as provider: every live copy of every consumer
        for (int q = out_lo; q < out_hi; ++q) {
          const int w = A.out_idx[q];
          for (int jw = 0; jw < C; ++jw) {
            const uint32_t pw = L.packed[w * C + jw];
            if (!live_of(pw)) continue;
            const uint32_t x = pw & 0xFFFFu;
            bool cov_other = false;
            for (int j = 0; j < C; ++j) cov_other = cov_other || (j != i && covers1(L.packed[v * C + j], x));
            if (cov_other) continue;
#pragma unroll
            for (int dd = 0; dd < kDisp; ++dd) {
              const int d = d0 + dd, delta = d < R ? d - R : d - R + 1;
              const int s2 = field == 0 ? s + delta : s, e2 = field == 0 ? e : e + delta;
              const bool live_new = s2 >= 0 && s2 <= e2 && e2 < T;
              vv[dd] += (live_new && s2 < (int)x && (int)x <= e2) ? 0 : 1;
            }
          }
        }
        // ---- peak: the profile changes on the positions between the old and the new value of the field
#pragma unroll
        for (int dd = 0; dd < kDisp; ++dd) {
          const int d = d0 + dd, delta = d < R ? d - R : d - R + 1;
          const int s2 = field == 0 ? s + delta : s, e2 = field == 0 ? e : e + delta;
          const bool in_dom = (field == 0 ? s2 : e2) >= 0 && (field == 0 ? s2 : e2) < T;
          const bool live_new = s2 >= 0 && s2 <= e2 && e2 < T;
          int p = base_peak;
          if (in_dom) {
            if (live_new) {
              int lo, hi, sign;
              if (field == 0) { lo = min(s, s2); hi = max(s, s2) - 1; sign = s2 < s ? 1 : -1; }
              else { lo = min(e, e2) + 1; hi = max(e, e2); sign = e2 > e ? 1 : -1; }
              int inside = 0;
              for (int t = lo; t <= hi; ++t) inside = max(inside, L.profile[t] + sign * sz);
              p = max(inside, max(lo > 0 ? L.pmax[lo - 1] : 0, hi + 1 < T ? L.smax[hi + 1] : 0));
            } else {
              if (lost_all < 0) {
                lost_all = 0;
                for (int t = s; t <= e; ++t) lost_all = max(lost_all, L.profile[t] - sz);
              }
              p = max(lost_all, max(s > 0 ? L.pmax[s - 1] : 0, e + 1 < T ? L.smax[e + 1] : 0));
            }
          }
          pk[dd] = p;
        }
        // ---- results of this group of displacements
#pragma unroll
        for (int dd = 0; dd < kDisp; ++dd) {
          const int d = d0 + dd;
          if (d >= two_r) continue;
          const int delta = d < R ? d - R : d - R + 1;
          const int moved = (field == 0 ? s : e) + delta;
          moc_move_score sc{-1, -1};
          if (moved >= 0 && moved < T) {
            sc.violations = vv[dd];
            sc.peak = pk[dd];
            const Best cand{vv[dd], pk[dd], pf * two_r + d};
            if (better(cand, best, g.budget)) best = cand;
          }
          if (dst) dst[d] = sc;
        }
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
  auto kern = lay.adj_off ? neighbours_kernel<true> : neighbours_kernel<false>;
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
