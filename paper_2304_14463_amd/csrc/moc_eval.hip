// moc_eval_batch: one workgroup evaluates one candidate at a time (Eq. (1)-(8)
// of the paper's Section 2.1) with its whole working set in LDS.
//
// Per candidate:
//   phase 1 (per copy)  the rows of starts/ends/active are streamed with 16-byte
//            loads, four consecutive copies per lane.  Each copy is classified
//            (active / live), counted for Eq. (2),(7),(8) and Eq. (1), staged in
//            LDS as one packed word s | e << 16, and -- if live -- scattered into
//            the memory-delta array (+m_v at s, -m_v at e+1: closed intervals of
//            Eq. (4)) and into a bitmap of occupied start positions (Eq. (6)).
//   phase 2 (a) each thread reduces a contiguous chunk of the delta array to
//            (sum, max prefix); chunks combine associatively in position order,
//            which yields the peak of Eq. (4) without materialising the profile;
//            (b) popcount of the bitmap: distinct start positions, so that
//            sum_t max(0, cnt_t - 1) = live copies - distinct starts;
//            (c) one lane per node (in-degree-sorted slices): Eq. (3) among the
//            node's own copies and Eq. (5) against the staged copies of every
//            predecessor.
// Predicates are counted with wave ballots + scalar popcounts, so violation
// counters live in scalar registers.  All arithmetic is integer: results do not
// depend on the order in which lanes or workgroups run.
#include "moc_internal.h"

namespace {

constexpr int kRedStride = 8;  // ints per wave in the cross-wave exchange area

struct LdsLayout {
  int chunk;       // delta entries per thread (odd: conflict-free strided reads)
  int delta_len;   // NT * chunk >= T + 1
  int packed_len;  // >= T + 6, multiple of 4
  int occ_words;   // ceil(T / 32)
  int bytes;
};

LdsLayout lds_layout(int T, int nt) {
  LdsLayout l;
  l.chunk = ((T + 1 + nt - 1) / nt) | 1;
  l.delta_len = nt * l.chunk;
  l.packed_len = (T + 6 + 3) & ~3;
  l.occ_words = (T + 31) / 32;
  l.bytes = 4 * (l.delta_len + l.packed_len + l.occ_words + (nt / kWave) * kRedStride);
  return l;
}

__device__ __forceinline__ int wave_count(bool pred) { return __popcll(__ballot(pred)); }

// Four consecutive elements starting at flat index idx.  Elements outside
// [lo, hi) are returned as 0 on the guarded path; on the vector path the
// caller masks them.
template <bool VEC>
__device__ __forceinline__ void load4(const int32_t* __restrict__ starts, const int32_t* __restrict__ ends,
                                      const uint8_t* __restrict__ active, int64_t idx, int64_t lo, int64_t hi,
                                      int64_t total, int (&s)[4], int (&e)[4], uint32_t& a4) {
  if (VEC && idx + 3 < total) {
    const int4 sv = *reinterpret_cast<const int4*>(starts + idx);
    const int4 ev = *reinterpret_cast<const int4*>(ends + idx);
    a4 = *reinterpret_cast<const uint32_t*>(active + idx);
    s[0] = sv.x; s[1] = sv.y; s[2] = sv.z; s[3] = sv.w;
    e[0] = ev.x; e[1] = ev.y; e[2] = ev.z; e[3] = ev.w;
  } else {
    a4 = 0;
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      const int64_t i = idx + c;
      const bool in = i >= lo && i < hi;
      s[c] = in ? starts[i] : 0;
      e[c] = in ? ends[i] : 0;
      a4 |= (in ? (uint32_t)active[i] : 0u) << (8 * c);
    }
  }
}

template <int NT, int CT, bool VEC>
__global__ __launch_bounds__(NT) void eval_batch_kernel(GraphView g, int64_t B, const int32_t* __restrict__ starts,
                                                        const int32_t* __restrict__ ends,
                                                        const uint8_t* __restrict__ active,
                                                        moc_result* __restrict__ out, LdsLayout lay) {
  constexpr int NW = NT / kWave;
  extern __shared__ uint32_t lds[];
  int32_t* delta = reinterpret_cast<int32_t*>(lds);
  uint32_t* packed = lds + lay.delta_len;
  uint32_t* occ = packed + lay.packed_len;
  int32_t* red = reinterpret_cast<int32_t*>(occ + lay.occ_words);

  const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
  const int T = g.T;
  const int C = CT ? CT : g.C;
  const int64_t total = B * (int64_t)T;

  for (int i = tid; i < lay.delta_len; i += NT) delta[i] = 0;
  for (int i = tid; i < lay.occ_words; i += NT) occ[i] = 0;
  __syncthreads();

  for (int64_t b = blockIdx.x; b < B; b += gridDim.x) {
    const int64_t row = b * T;
    const int head = VEC ? (int)(row & 3) : 0;   // copies of the previous row sharing the first 16 bytes
    const int64_t base = row - head;
    const int nslots = (head + T + 3) >> 2;
    const int iters = (nslots + NT - 1) / NT;

    int viol = 0, nlive = 0;   // wave-uniform counters
    int dur = 0;               // per lane

    // ---------------- phase 1: per copy
    for (int it = 0; it < iters; ++it) {
      const int slot = it * NT + tid;
      const bool ok = slot < nslots;
      int s[4] = {0, 0, 0, 0}, e[4] = {0, 0, 0, 0};
      uint32_t a4 = 0;
      if (ok) load4<VEC>(starts, ends, active, base + 4 * (int64_t)slot, row, row + T, total, s, e, a4);
      uint32_t pk[4];
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        const int kk = 4 * slot + c - head;                       // copy index within the row
        const bool valid = ok && (unsigned)kk < (unsigned)T;
        const uint32_t a = (a4 >> (8 * c)) & 0xFFu;
        const bool act = valid && a != 0;
        const bool well = (uint32_t)s[c] <= (uint32_t)e[c] && (uint32_t)e[c] < (uint32_t)T;   // Eq. (2), (8)
        const bool live = act && well;
        const int v = (int)((unsigned)kk / (unsigned)C);
        const bool first_off = valid && a == 0 && kk == v * C;   // Eq. (7)
        viol += wave_count((act && !well) || first_off);
        nlive += wave_count(live);
        int2 sd = make_int2(0, 0);
        if (act) sd = g.size_dur[v];
        dur += sd.y;                                              // Eq. (1)
        pk[c] = live ? ((uint32_t)s[c] | ((uint32_t)e[c] << 16)) : MOC_DEAD;
        if (live) {
          atomicAdd(&delta[s[c]], sd.x);                          // Eq. (4): allocated at s ...
          atomicAdd(&delta[e[c] + 1], -sd.x);                     // ... released after e
          atomicOr(&occ[s[c] >> 5], 1u << (s[c] & 31));           // Eq. (6)
        }
      }
      if (ok) *reinterpret_cast<uint4*>(&packed[4 * slot]) = make_uint4(pk[0], pk[1], pk[2], pk[3]);
    }
    __syncthreads();

    // ---------------- phase 2a: (sum, max prefix) of this thread's chunk, then of the wave
    int S = 0, P = 0;
    {
      int32_t* d = delta + tid * lay.chunk;
      for (int j = 0; j < lay.chunk; ++j) {
        const int x = d[j];
        d[j] = 0;
        S += x;
        P = max(P, S);
      }
    }
#pragma unroll
    for (int off = 1; off < kWave; off <<= 1) {
      const int S2 = __shfl_down(S, off), P2 = __shfl_down(P, off);
      if (lane + off < kWave) {
        P = max(P, S + P2);
        S += S2;
      }
    }

    // ---------------- phase 2b: distinct start positions
    int distinct = 0;
    for (int w = tid; w < lay.occ_words; w += NT) {
      distinct += __popc(occ[w]);
      occ[w] = 0;
    }

    // ---------------- phase 2c: per node, Eq. (3) and Eq. (5)
    for (int sl = wave; sl < g.n_slices; sl += NW) {
      const int p = sl * kWave + lane;
      const uint32_t info = g.slot_info[p];
      const bool is_node = p < g.n;
      const int kbase = head + (int)(info & 0xFFFFu);
      const int deg = (int)(info >> 16);
      const int e0 = g.ell_ptr[sl];
      const int width = (g.ell_ptr[sl + 1] - e0) / kWave;
      if constexpr (CT > 0) {
        uint32_t pv[CT], x[CT], xs[CT];
        bool lv[CT];
#pragma unroll
        for (int i = 0; i < CT; ++i) {
          pv[i] = is_node ? packed[kbase + i] : MOC_DEAD;
          lv[i] = pv[i] != MOC_DEAD;
          x[i] = pv[i] & 0xFFFFu;   // start of the consumer copy
          xs[i] = x[i] << 16;
        }
#pragma unroll
        for (int i = 0; i + 1 < CT; ++i) {   // Eq. (3): against the next live copy
          bool seen = false, late = false;
#pragma unroll
          for (int j = i + 1; j < CT; ++j) {
            late = late || (!seen && lv[j] && (pv[i] >> 16) > x[j]);
            seen = seen || lv[j];
          }
          viol += wave_count(lv[i] && late);
        }
        for (int j = 0; j < width; ++j) {
          const int ub = head + (int)g.ell_pred[e0 + j * kWave + lane];
          const bool has = j < deg;
          uint32_t pu[CT];
#pragma unroll
          for (int q = 0; q < CT; ++q) pu[q] = packed[ub + q];
#pragma unroll
          for (int i = 0; i < CT; ++i) {
            bool cov = false;   // Eq. (5): s_u + 1 <= s_v  and  s_v <= e_u
#pragma unroll
            for (int q = 0; q < CT; ++q) cov = cov || ((pu[q] & 0xFFFFu) < x[i] && pu[q] >= xs[i]);
            viol += wave_count(has && lv[i] && !cov);
          }
        }
      } else {
        for (int i = 0; i < C; ++i) {
          const uint32_t pvi = is_node ? packed[kbase + i] : MOC_DEAD;
          const bool lvi = pvi != MOC_DEAD;
          const uint32_t xi = pvi & 0xFFFFu, xsi = xi << 16;
          bool seen = false, late = false;
          for (int j = i + 1; j < C; ++j) {
            const uint32_t pvj = is_node ? packed[kbase + j] : MOC_DEAD;
            const bool lvj = pvj != MOC_DEAD;
            late = late || (!seen && lvj && (pvi >> 16) > (pvj & 0xFFFFu));
            seen = seen || lvj;
          }
          viol += wave_count(lvi && late);
          for (int j = 0; j < width; ++j) {
            const int ub = head + (int)g.ell_pred[e0 + j * kWave + lane];
            bool cov = false;
            for (int q = 0; q < C; ++q) {
              const uint32_t pu = packed[ub + q];
              cov = cov || ((pu & 0xFFFFu) < xi && pu >= xsi);
            }
            viol += wave_count(j < deg && lvi && !cov);
          }
        }
      }
    }

    // ---------------- combine
#pragma unroll
    for (int off = kWave / 2; off > 0; off >>= 1) {
      dur += __shfl_xor(dur, off);
      distinct += __shfl_xor(distinct, off);
    }
    if (lane == 0) {
      int32_t* r = red + wave * kRedStride;
      r[0] = S; r[1] = P; r[2] = viol; r[3] = nlive; r[4] = distinct; r[5] = dur;
    }
    __syncthreads();
    if (tid == 0) {
      int Sa = 0, Pa = 0, va = 0, la = 0, da = 0, ua = 0;
      for (int w = 0; w < NW; ++w) {
        const int32_t* r = red + w * kRedStride;
        Pa = max(Pa, Sa + r[1]);
        Sa += r[0];
        va += r[2]; la += r[3]; da += r[4]; ua += r[5];
      }
      va += la - da;   // Eq. (6): live copies minus distinct start positions
      moc_result res;
      res.peak = Pa;
      res.duration = ua;
      res.violations = va;
      res.feasible = (va == 0 && (int64_t)Pa <= g.budget) ? 1 : 0;
      out[b] = res;
    }
  }
}

template <int NT, int CT, bool VEC>
int launch(const moc_graph* g, int64_t B, const int32_t* starts, const int32_t* ends, const uint8_t* active,
           moc_result* out, hipStream_t stream) {
  const LdsLayout lay = lds_layout(g->view.T, NT);
  if (lay.bytes > g->max_lds) return MOC_EOVERFLOW;
  auto kern = eval_batch_kernel<NT, CT, VEC>;
  MOC_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                              lay.bytes));
  int per_cu = 0;
  MOC_HIP(hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, kern, NT, lay.bytes));
  if (per_cu < 1) per_cu = 1;
  const int64_t resident = (int64_t)per_cu * g->num_cu;
  const unsigned grid = (unsigned)(B < resident ? B : resident);
  hipLaunchKernelGGL(kern, dim3(grid), dim3(NT), lay.bytes, stream, g->view, B, starts, ends, active, out, lay);
  MOC_HIP(hipGetLastError());
  return MOC_OK;
}

template <int NT, bool VEC>
int launch_c(const moc_graph* g, int64_t B, const int32_t* s, const int32_t* e, const uint8_t* a, moc_result* out,
             hipStream_t st) {
  switch (g->view.C) {
    case 1: return launch<NT, 1, VEC>(g, B, s, e, a, out, st);
    case 2: return launch<NT, 2, VEC>(g, B, s, e, a, out, st);
    case 3: return launch<NT, 3, VEC>(g, B, s, e, a, out, st);
    case 4: return launch<NT, 4, VEC>(g, B, s, e, a, out, st);
    default: return launch<NT, 0, VEC>(g, B, s, e, a, out, st);
  }
}

template <bool VEC>
int launch_nt(const moc_graph* g, int64_t B, const int32_t* s, const int32_t* e, const uint8_t* a, moc_result* out,
              hipStream_t st) {
  // Workgroup size by row length: one wave per candidate while a row is a few
  // vector loads per lane, a full 1024-thread workgroup for the longest rows.
  const int T = g->view.T;
  if (T <= 1024) return launch_c<64, VEC>(g, B, s, e, a, out, st);
  if (T <= 6144) return launch_c<256, VEC>(g, B, s, e, a, out, st);
  return launch_c<1024, VEC>(g, B, s, e, a, out, st);
}

}  // namespace

extern "C" int moc_eval_batch(const moc_graph* g, int64_t B, const int32_t* starts, const int32_t* ends,
                              const uint8_t* active, moc_result* out, void* hip_stream) {
  if (!g || B < 0) return MOC_EINVAL;
  if (B == 0) return MOC_OK;
  if (!starts || !ends || !active || !out) return MOC_EINVAL;
  if (((uintptr_t)starts | (uintptr_t)ends) & 3 || ((uintptr_t)out & 7)) return MOC_EINVAL;
  int dev = -1;
  MOC_HIP(hipGetDevice(&dev));
  if (dev != g->device) return MOC_EDEVICE;
  const bool vec = ((((uintptr_t)starts | (uintptr_t)ends) & 15) == 0) && (((uintptr_t)active & 3) == 0);
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  return vec ? launch_nt<true>(g, B, starts, ends, active, out, st)
             : launch_nt<false>(g, B, starts, ends, active, out, st);
}
