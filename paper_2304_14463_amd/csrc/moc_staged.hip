// moc_eval_batch_staged: evaluation in the stage-restricted domain of the paper's Section 2.3
// ("Complexity Reduction by Enforcing an Initial Topological Ordering"), gfx950.
//
// The domain has n(n+1)/2 positions in n stages, stage j holding the j + 1 positions
// j(j+1)/2 .. j(j+1)/2 + j.  A node with place k in the topological order may be computed only
// at slot k of a stage, the first time at slot k of stage k.  A start that is not such a value
// is outside the variable's domain: the copy is treated like one with a position outside the
// domain of Eq. (8) (one violation, used by nothing else, still paid for in Eq. (1)).
// Everything else is Eq. (1)-(8) on those positions.
//
// The domain is far too long for a memory profile in LDS (12.5 M positions at n = 5000), but
// memory can only rise where an interval starts (Section 2.2, memory constraints), and every
// other test compares a start with a start or with an end.  So the kernel renumbers: the
// distinct start positions of the usable copies, in increasing order, become 0, 1, 2, ...
// (at most n*C of them); a start takes the rank of its position, an end the rank of the last
// start position not after it.  Eq. (4) and Eq. (5) keep their outcome under that map; Eq. (2),
// (3), (8) are decided on the positions as given, before the map; for Eq. (6) only copies of
// one node can share a position here (a slot belongs to one node), which a lane sees by itself.
// Ranks without sorting: a usable start is (stage j, node k).  Count the distinct ones per
// stage, prefix-sum the counts over the stages, drop the k of each into its stage's bucket; the
// rank of (j, k) is the bucket's offset plus the number of smaller k in the bucket (buckets
// hold the few nodes recomputed in a stage, and the stage's own node).
//
// One workgroup per candidate at a time, one lane per node, all in LDS.
#include "moc_internal.h"

namespace {

constexpr int kNT = 512;
constexpr int kNW = kNT / kWave;

struct StLayout {
  int cur_off, bucket_off, pj_off, pe_off, delta_off, red_off;   // word offsets
  int chunk;      // delta entries per thread (odd: conflict-free strided reads)
  int bytes;
};

StLayout st_layout(int n, int C) {
  const int T = n * C;
  StLayout l;
  l.chunk = ((T + 1 + kNT - 1) / kNT) | 1;
  l.cur_off = 0;                                   // int32 [n]: per stage count, then end of the stage's bucket
  l.bucket_off = l.cur_off + n;                    // uint16 [T]: node places, stage by stage
  l.pj_off = l.bucket_off + (T + 1) / 2;           // int32 [T]: stage of the copy's start, -1 if not usable; then its record
  l.pe_off = l.pj_off + T;                         // int32 [T]: the copy's end as given
  l.delta_off = l.pe_off + T;                      // int32 [kNT * chunk]
  l.red_off = l.delta_off + kNT * l.chunk;
  l.bytes = 4 * (l.red_off + 8 * kNW + 8);
  return l;
}

// First position of stage j, j < 2^16 (24-bit multiply: full rate).
__device__ __forceinline__ uint32_t stage_start(int j) { return __umul24((uint32_t)j, (uint32_t)j + 1u) >> 1; }

// The stage that holds position p (0 <= p < 2^31): the largest j with j(j+1)/2 <= p.  A
// floating-point estimate, then one exact integer step each way, so that the result does not
// depend on how the square root rounds: the estimate's error stays far below one stage (the
// relative error of the root is a few 2^-24 and the root at most 2^17), so its floor is off by
// one at most.
__device__ __forceinline__ int stage_of(uint32_t p) {
  int j = (int)((__fsqrt_rn(8.0f * (float)p + 1.0f) - 1.0f) * 0.5f);
  j = max(j, 0);
  j -= stage_start(j) > p ? 1 : 0;
  j += stage_start(j + 1) <= p ? 1 : 0;
  return j;
}

__device__ __forceinline__ int wave_sum_i(int v) {
#pragma unroll
  for (int off = kWave / 2; off > 0; off >>= 1) v += __shfl_xor(v, off);
  return v;
}

// CT = C when C <= 4 (the copies of a node are then read into registers, for this candidate at
// the top of its turn and for the workgroup's next candidate as soon as they are used), else 0
// (any C, read where needed); U = nodes per lane, ceil(n / kNT), when CT > 0.
template <int CT, int U>
// 64 registers (four workgroups per CU) where the copies of a lane's nodes are few enough to fit
// beside the rest; otherwise as many as they take.
__global__ __launch_bounds__(kNT) __attribute__((amdgpu_waves_per_eu((CT == 0 ? 1 : CT) * U <= 4 && U <= 2 && CT <= 3 ? 8 : 4, 8))) void eval_staged_kernel(GraphView g, const int32_t* __restrict__ place, int64_t B,
                                                          const int32_t* __restrict__ starts,
                                                          const int32_t* __restrict__ ends,
                                                          const uint8_t* __restrict__ active,
                                                          moc_result* __restrict__ out, StLayout lay) {
  extern __shared__ uint32_t st_raw[];
  int32_t* const cur = reinterpret_cast<int32_t*>(st_raw + lay.cur_off);
  uint16_t* const bucket = reinterpret_cast<uint16_t*>(st_raw + lay.bucket_off);
  int32_t* const pj = reinterpret_cast<int32_t*>(st_raw + lay.pj_off);
  int32_t* const pe = reinterpret_cast<int32_t*>(st_raw + lay.pe_off);
  int32_t* const delta = reinterpret_cast<int32_t*>(st_raw + lay.delta_off);
  int32_t* const red = reinterpret_cast<int32_t*>(st_raw + lay.red_off);
  const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
  const int n = g.n, C = g.C, T = g.T;
  const uint32_t D = (uint32_t)n * (uint32_t)(n + 1) / 2u;   // positions of the domain

  for (int i = tid; i < kNT * lay.chunk; i += kNT) delta[i] = 0;

  // registers for the copies of the lane's nodes (CT > 0)
  constexpr int RU = CT > 0 ? U : 1, RC = CT > 0 ? CT : 1;
  [[maybe_unused]] int rs[RU][RC], re[RU][RC];
  // a node's flags as they lie in memory, in one register, taken apart where they are used:
  // bytes put together in a register as they arrive make each load wait where it is issued
  struct Flags { uint8_t a[RC]; };
  static_assert(sizeof(Flags) <= 4, "the flags of a node fit a register");
  [[maybe_unused]] uint32_t ra[RU];
  // The candidate's rows are the same for all lanes (scalar registers); a lane adds a 32-bit
  // offset that is formed here from the thread index each time.  Whole addresses per lane, kept
  // across the loop over the candidates, would be spilled, and fetching them back here makes
  // every load of the request wait for the one before.
  struct alignas(4) Ints { int32_t x[RC]; };
  [[maybe_unused]] auto request = [&](int64_t cand) {
    if constexpr (CT > 0) {
      const char* const s_row = reinterpret_cast<const char*>(starts + cand * T);
      const char* const e_row = reinterpret_cast<const char*>(ends + cand * T);
      const char* const a_row = reinterpret_cast<const char*>(active + cand * T);
      int t = tid;
      asm volatile("" : "+v"(t));
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const uint32_t off = (uint32_t)min(u * kNT + t, n - 1) * CT;   // lanes past the last node re-read it
        const Ints sv = *reinterpret_cast<const Ints*>(s_row + off * 4u);
        const Ints ev = *reinterpret_cast<const Ints*>(e_row + off * 4u);
        const Flags f = *reinterpret_cast<const Flags*>(a_row + off);
#pragma unroll
        for (int i = 0; i < CT; ++i) {
          rs[u][i] = sv.x[i];
          re[u][i] = ev.x[i];
        }
        uint32_t w = 0;
        __builtin_memcpy(&w, &f, sizeof(Flags));
        ra[u] = w;
      }
    }
  };
  if ((int64_t)blockIdx.x < B) request(blockIdx.x);
  // place, m_v, w_v of the lane's nodes: the same for every candidate
  [[maybe_unused]] int rk[RU];
  [[maybe_unused]] int2 rsd[RU];
  if constexpr (CT > 0) {
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int v = min(u * kNT + tid, n - 1);
      rk[u] = place[v];
      rsd[u] = g.size_dur[v];
    }
  }

  for (int64_t b = blockIdx.x; b < B; b += gridDim.x) {
    const int64_t row = b * T;
    for (int j = tid; j < n; j += kNT) cur[j] = 0;
    __syncthreads();

    // ---- per node: Eq. (1), (2), (3), (7), (8) and the domain of the starts; count the distinct
    //      usable starts per stage
    int viol = 0, dur = 0;
    // one copy: i-th of node v (place k, duration w); prev_end = end of the node's latest usable copy so far
    auto copy_step = [&](int v, int k, int w, int i, int s, int e, bool act, int& prev_end) {
      const int c = v * C + i;
      bool live = act && (uint32_t)s <= (uint32_t)e && (uint32_t)e < D;
      int j = -1;
      if (live) {
        j = stage_of((uint32_t)s);
        live = (uint32_t)s - stage_start(j) == (uint32_t)k && (i > 0 || j == k);
      }
      viol += (act && !live) ? 1 : 0;
      if (i == 0) viol += act ? 0 : 1;
      dur += act ? w : 0;
      int code = -1;
      if (live) {
        viol += prev_end > s ? 1 : 0;   // Eq. (3), on the positions as given
        prev_end = e;
        // Eq. (6): a usable start shares its position only with copies of its own node, which
        // sit in the same stage; the first of them stands for the position
        bool first_here = true;
        for (int q = 0; q < i; ++q) first_here = first_here && pj[v * C + q] >> 1 != j;
        if (first_here) atomicAdd(&cur[j], 1);
        else viol += 1;
        code = j << 1 | (first_here ? 1 : 0);
      }
      pj[c] = live ? code : -2;   // -2 >> 1 = -1: no stage
      pe[c] = e;
    };
    if constexpr (CT > 0) {
      // the same per copy, on registers: the start's register takes the copy's code (stage << 1 |
      // first at its position, -2 if not usable), which the next two phases read
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int v = u * kNT + tid;
        if (v < n) {
          const int k = rk[u], w = rsd[u].y;
          int prev_end = -1;
#pragma unroll
          for (int i = 0; i < CT; ++i) {
            const int s = rs[u][i], e = re[u][i];
            const bool act = ((ra[u] >> (8 * i)) & 0xFFu) != 0;
            bool live = act && (uint32_t)s <= (uint32_t)e && (uint32_t)e < D;
            int j = -1;
            if (live) {
              j = stage_of((uint32_t)s);
              live = (uint32_t)s - stage_start(j) == (uint32_t)k && (i > 0 || j == k);
            }
            viol += (act && !live) ? 1 : 0;
            if (i == 0) viol += act ? 0 : 1;
            dur += act ? w : 0;
            int code = -2;
            if (live) {
              viol += prev_end > s ? 1 : 0;   // Eq. (3), on the positions as given
              prev_end = e;
              bool first_here = true;         // Eq. (6), see above
#pragma unroll
              for (int q = 0; q < i; ++q) first_here = first_here && rs[u][q] >> 1 != j;
              if (first_here) atomicAdd(&cur[j], 1);
              else viol += 1;
              code = j << 1 | (first_here ? 1 : 0);
            }
            rs[u][i] = code;
          }
        }
      }
    } else {
      for (int v = tid; v < n; v += kNT) {
        const int k = place[v], w = g.size_dur[v].y;
        int prev_end = -1;
        for (int i = 0; i < C; ++i)
          copy_step(v, k, w, i, starts[row + v * C + i], ends[row + v * C + i], active[row + v * C + i] != 0, prev_end);
      }
    }
    __syncthreads();

    // ---- cur[j] <- number of distinct usable starts in stages 0..j (inclusive running sum)
    {
      const int per = (n + kNT - 1) / kNT;
      const int j0 = min(tid * per, n), j1 = min(j0 + per, n);
      int sum = 0;
      for (int j = j0; j < j1; ++j) sum += cur[j];
      int incl = sum;
#pragma unroll
      for (int off = 1; off < kWave; off <<= 1) {
        const int o = __shfl_up(incl, off);
        if (lane >= off) incl += o;
      }
      if (lane == kWave - 1) red[wave] = incl;
      __syncthreads();
      int before = incl - sum;
      for (int w = 0; w < wave; ++w) before += red[w];
      // leave in cur[j] the offset of the stage's bucket: the fill below advances it to the end
      for (int j = j0; j < j1; ++j) {
        const int c = cur[j];
        cur[j] = before;
        before += c;
      }
    }
    __syncthreads();

    // ---- buckets: the place of every node that has a first-at-its-position start in the stage
    if constexpr (CT > 0) {
#pragma unroll
      for (int u = 0; u < U; ++u) {
        if (u * kNT + tid >= n) continue;
#pragma unroll
        for (int i = 0; i < CT; ++i) {
          const int code = rs[u][i];
          if (code >= 0 && (code & 1)) bucket[atomicAdd(&cur[code >> 1], 1)] = (uint16_t)rk[u];
        }
      }
    } else {
      for (int v = tid; v < n; v += kNT) {
        const int k = place[v];
        for (int i = 0; i < C; ++i) {
          const int code = pj[v * C + i];
          if (code >= 0 && (code & 1)) bucket[atomicAdd(&cur[code >> 1], 1)] = (uint16_t)k;
        }
      }
    }
    __syncthreads();   // now cur[j] = end of stage j's bucket = start of stage j + 1's

    // ---- renumber, stage the records, scatter Eq. (4)
    // Entries of stage j's bucket below `key` (or up to it), on top of the bucket's offset.  A
    // bucket holds the stage's own node and the few nodes recomputed in the stage: the first two
    // entries are read at once, a loop takes the rest.
    [[maybe_unused]] auto rank_in_stage = [&](int j, uint32_t key, bool up_to) -> int {
      const int lo = j ? cur[j - 1] : 0, hi = cur[j];
      const uint32_t b0 = lo < hi ? bucket[lo] : 0xFFFFu, b1 = lo + 1 < hi ? bucket[lo + 1] : 0xFFFFu;   // places stay below 0xFFFF
      const uint32_t bound = key + (up_to ? 1u : 0u);
      int r = lo + (b0 < bound ? 1 : 0) + (b1 < bound ? 1 : 0);
      for (int x = lo + 2; x < hi; ++x) r += bucket[x] < bound ? 1 : 0;
      return r;
    };
    if constexpr (CT > 0) {
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int v = u * kNT + tid;
        if (v >= n) continue;
#pragma unroll
        for (int i = 0; i < CT; ++i) {
          const int code = rs[u][i];
          uint32_t rec = MOC_DEAD;
          if (code >= 0) {
            const int cs = rank_in_stage(code >> 1, (uint32_t)rk[u], false);
            // the last start position not after the end: all starts of earlier stages, and those of
            // the end's stage at slots up to the end's
            const uint32_t e = (uint32_t)re[u][i];
            const int je = stage_of(e);
            const int ce = rank_in_stage(je, e - stage_start(je), true) - 1;
            rec = (uint32_t)cs | (uint32_t)ce << 16;
            atomicAdd(&delta[cs], rsd[u].x);
            atomicSub(&delta[ce + 1], rsd[u].x);
          }
          pj[v * CT + i] = (int32_t)rec;
        }
      }
      if (b + gridDim.x < B) request(b + gridDim.x);   // the rest of this turn works from LDS
    } else
    for (int v = tid; v < n; v += kNT) {
      const int2 sd = g.size_dur[v];
      const int k = place[v];
      for (int i = 0; i < C; ++i) {
        const int c = v * C + i;
        const int code = pj[c];
        uint32_t rec = MOC_DEAD;
        if (code >= 0) {
          const int j = code >> 1;
          int lo = j ? cur[j - 1] : 0, hi = cur[j];
          int cs = lo;
          for (int x = lo; x < hi; ++x) cs += bucket[x] < k ? 1 : 0;
          // the last start position not after the end: all starts of earlier stages, and those of
          // the end's stage at slots up to the end's
          const uint32_t e = (uint32_t)pe[c];
          const int je = stage_of(e);
          const uint32_t slot_e = e - (uint32_t)je * (uint32_t)(je + 1) / 2u;
          lo = je ? cur[je - 1] : 0;
          hi = cur[je];
          int ce = lo - 1;
          for (int x = lo; x < hi; ++x) ce += bucket[x] <= slot_e ? 1 : 0;
          rec = (uint32_t)cs | (uint32_t)ce << 16;
          atomicAdd(&delta[cs], sd.x);
          atomicSub(&delta[ce + 1], sd.x);
        }
        pj[c] = (int32_t)rec;
      }
    }
    __syncthreads();

    // ---- Eq. (4): peak of the running sum over the renumbered positions
    int S = 0, P = 0;
    {
      int own = tid;   // formed here: kept from the top of the kernel it is spilled, and the reload would
      asm volatile("" : "+v"(own));   // wait for the next candidate's loads, which are in flight by now
      int32_t* d = delta + own * lay.chunk;
      for (int x = 0; x < lay.chunk; ++x) {
        const int y = d[x];
        d[x] = 0;
        S += y;
        P = max(P, S);
      }
#pragma unroll
      for (int off = 1; off < kWave; off <<= 1) {   // lane l absorbs lanes l+off .. l+2*off-1
        const int S2 = __shfl_down(S, off), P2 = __shfl_down(P, off);
        if (lane + off < kWave) {
          P = max(P, S + P2);
          S += S2;
        }
      }
    }
    // ---- Eq. (5): one lane per edge, every usable copy of the consumer
    for (int x = tid; x < g.m; x += kNT) {
      const uint32_t pair = g.edge_pair_c[x];
      const int kd = (int)(pair >> 16), ub = (int)(pair & 0xFFFFu);
      for (int i = 0; i < C; ++i) {
        const uint32_t pv = (uint32_t)pj[kd + i];
        const uint32_t at = pv & 0xFFFFu;
        bool cov = false;
        for (int q = 0; q < C; ++q) {
          const uint32_t pu = (uint32_t)pj[ub + q];
          cov = cov || ((pu & 0xFFFFu) < at && (pu >> 16) >= at);   // s_u + 1 <= s_v <= e_u; a dead copy has s = 0xFFFF
        }
        viol += (at != 0xFFFFu && !cov) ? 1 : 0;
      }
    }
    viol = wave_sum_i(viol);
    dur = wave_sum_i(dur);
    if (lane == 0) {
      int32_t* r = red + 8 + wave * 4;
      r[0] = S; r[1] = P; r[2] = viol; r[3] = dur;
    }
    __syncthreads();
    if (tid == 0) {
      int S0 = 0, P0 = 0, V = 0, W = 0;
      for (int w = 0; w < kNW; ++w) {
        const int32_t* r = red + 8 + w * 4;
        P0 = max(P0, S0 + r[1]);
        S0 += r[0];
        V += r[2];
        W += r[3];
      }
      moc_result res;
      res.peak = P0;
      res.duration = W;
      res.violations = V;
      res.feasible = (V == 0 && (int64_t)P0 <= g.budget) ? 1 : 0;
      out[b] = res;
    }
    __syncthreads();
  }
}

}  // namespace

extern "C" int moc_eval_batch_staged(const moc_graph* g, int64_t B, const int32_t* starts, const int32_t* ends,
                                     const uint8_t* active, moc_result* out, void* hip_stream) {
  if (!g || B < 0) return MOC_EINVAL;
  if (!g->place) return MOC_EINVAL;   // moc_graph_set_order has not been called
  if (B == 0) return MOC_OK;
  if (!starts || !ends || !active || !out) return MOC_EINVAL;
  if ((((uintptr_t)starts | (uintptr_t)ends) & 3) || ((uintptr_t)out & 7)) return MOC_EINVAL;
  int dev = -1;
  MOC_HIP(hipGetDevice(&dev));
  if (dev != g->device) return MOC_EDEVICE;
  const StLayout lay = st_layout(g->view.n, g->view.C);
  if (lay.bytes > g->max_lds || g->view.T >= 0xFFFF) return MOC_EOVERFLOW;
  const int per_lane = (g->view.n + kNT - 1) / kNT, C = g->view.C;
  auto kern = eval_staged_kernel<0, 1>;
  if (C <= 4 && per_lane * C <= 16) {   // the copies of a lane's nodes fit its registers
    const int u = per_lane <= 1 ? 1 : per_lane <= 2 ? 2 : per_lane <= 4 ? 4 : 8;
    switch (C * 16 + u) {
      case 1 * 16 + 1: kern = eval_staged_kernel<1, 1>; break;
      case 1 * 16 + 2: kern = eval_staged_kernel<1, 2>; break;
      case 1 * 16 + 4: kern = eval_staged_kernel<1, 4>; break;
      case 1 * 16 + 8: kern = eval_staged_kernel<1, 8>; break;
      case 2 * 16 + 1: kern = eval_staged_kernel<2, 1>; break;
      case 2 * 16 + 2: kern = eval_staged_kernel<2, 2>; break;
      case 2 * 16 + 4: kern = eval_staged_kernel<2, 4>; break;
      case 2 * 16 + 8: kern = eval_staged_kernel<2, 8>; break;
      case 3 * 16 + 1: kern = eval_staged_kernel<3, 1>; break;
      case 3 * 16 + 2: kern = eval_staged_kernel<3, 2>; break;
      case 3 * 16 + 4: kern = eval_staged_kernel<3, 4>; break;
      case 4 * 16 + 1: kern = eval_staged_kernel<4, 1>; break;
      case 4 * 16 + 2: kern = eval_staged_kernel<4, 2>; break;
      case 4 * 16 + 4: kern = eval_staged_kernel<4, 4>; break;
      default: break;
    }
  }
  int per_cu = 0;
  if (const int rc = moc_kernel_occupancy(g, reinterpret_cast<const void*>(kern), kNT, lay.bytes, false, &per_cu)) return rc;
  const int64_t resident = (int64_t)per_cu * g->num_cu;
  const unsigned grid = (unsigned)(B < resident ? B : resident);
  hipLaunchKernelGGL(kern, dim3(grid), dim3(kNT), lay.bytes, static_cast<hipStream_t>(hip_stream), g->view,
                     g->place, B, starts, ends, active, out, lay);
  MOC_HIP(hipGetLastError());
  return MOC_OK;
}
