// moc_decode_batch: from candidate assignments back to the rematerialisation sequences they
// stand for, with each sequence's own cost (gfx950).
//
// Section 2 of the paper (arXiv 2304.14463): the start of an active interval is the event at
// which its node is computed, so the active copies read in order of their starts are the
// sequence.  Section 1 (problem statement): a sequence is valid when every node occurs and the
// outputs of all predecessors of a node are in memory when it is computed; it costs the summed
// duration and the peak footprint.  The footprint taken here is the sequence's own: a use is
// served by the most recent earlier computation of the producer, an output is held from its
// step through the last step it serves.
//
// One workgroup per candidate, everything in LDS.  Starts are distinct (otherwise the
// candidate is not decodable), so sorting is a scatter by start followed by a prefix count of
// the occupied positions; the footprint is computed over positions rather than steps -- an
// empty position holds a subset of what the next step holds -- by the same difference array
// and running sum as Eq. (4).
#include "moc_internal.h"

namespace {

constexpr int kNT = 512;
constexpr int kNW = kNT / kWave;
constexpr uint32_t kNoStart = 0xFFFFu;

struct DcLayout {
  int T_pad;      // words in each of the two position arrays (>= T + 1, a multiple of 4)
  int st_words;   // words of the array of starts (16-bit entries; C = 3: 4 per node, so that a node's starts are two words)
  int bytes;
};

DcLayout dc_layout(int n, int C) {
  const int T = n * C;
  DcLayout l;
  l.T_pad = (T + 4) & ~3;   // > T, a multiple of 4
  l.st_words = C == 3 ? 2 * n + 2 : l.T_pad / 2;
  const int words = 2 * l.T_pad + l.st_words + 2 * kNW + 16;
  l.bytes = words * 4;
  return l;
}

// The value of the lane CTRL names (a lane shift of the vector ALU), 0 where that lane does not
// exist or the row is not in ROWS.
template <int CTRL, int ROWS>
__device__ __forceinline__ int from_lane(int x) { return __builtin_amdgcn_update_dpp(0, x, CTRL, ROWS, 0xF, true); }

// Inclusive wave scan of one value per lane: inside rows of 16 lanes by shifts of 1, 2, 4, 8,
// then lane 15 of rows 0 and 2 is added to rows 1 and 3, then lane 31 to rows 2 and 3.
__device__ __forceinline__ int wave_scan_add(int x, int /*lane*/) {
  x += from_lane<0x111, 0xF>(x);   // row_shr:1
  x += from_lane<0x112, 0xF>(x);   // row_shr:2
  x += from_lane<0x114, 0xF>(x);   // row_shr:4
  x += from_lane<0x118, 0xF>(x);   // row_shr:8
  x += from_lane<0x142, 0xA>(x);   // row_bcast:15
  x += from_lane<0x143, 0xC>(x);   // row_bcast:31
  return x;
}

// (sum, max prefix >= 0) of consecutive segments, one per lane, combined in lane order: the
// last lane ends with the whole wave.
template <int CTRL, int ROWS>
__device__ __forceinline__ void absorb_earlier(int& S, int& P) {
  const int Se = from_lane<CTRL, ROWS>(S), Pe = from_lane<CTRL, ROWS>(P);
  P = max(Pe, Se + P);
  S = Se + S;
}
__device__ __forceinline__ void wave_combine_ordered(int& S, int& P) {
  absorb_earlier<0x111, 0xF>(S, P);
  absorb_earlier<0x112, 0xF>(S, P);
  absorb_earlier<0x114, 0xF>(S, P);
  absorb_earlier<0x118, 0xF>(S, P);
  absorb_earlier<0x142, 0xA>(S, P);
  absorb_earlier<0x143, 0xC>(S, P);
}

// Both scans below walk the array in rows of 64 consecutive positions, one lane per position
// (no bank conflicts); wave w owns the rows [w * rows_per_wave, (w + 1) * rows_per_wave).

// a[x] in {0, 1}: a[x] <- number of ones before x, for x in [0, T); returns the number of ones.
// Every thread of the workgroup calls it; ends with a barrier.
__device__ int block_rank_of_ones(int32_t* a, int T, int32_t* scratch, int tid) {
  const int lane = tid & (kWave - 1), wave = tid / kWave;
  const int rows = (T + kWave - 1) / kWave, rows_per_wave = (rows + kNW - 1) / kNW;
  const int r0 = min(wave * rows_per_wave, rows), r1 = min(r0 + rows_per_wave, rows);
  int carry = 0;
  for (int r = r0; r < r1; ++r) {
    const int x = r * kWave + lane;
    const bool one = x < T && a[x] != 0;
    const uint64_t ones = __ballot(one);
    if (x < T) a[x] = carry + __popcll(ones & ((1ull << lane) - 1));
    carry += __popcll(ones);
  }
  if (lane == 0) scratch[wave] = carry;
  __syncthreads();
  int before = 0, total = 0;
  for (int w = 0; w < kNW; ++w) {
    const int t = scratch[w];
    if (w < wave) before += t;
    total += t;
  }
  if (before)
    for (int r = r0; r < r1; ++r) {
      const int x = r * kWave + lane;
      if (x < T) a[x] += before;
    }
  __syncthreads();
  return total;
}

// max over x in [0, T) of a[0] + ... + a[x] (at least 0).  Ends with a barrier.
__device__ int block_peak_of_running_sum(const int32_t* a, int T, int32_t* scratch, int tid) {
  const int lane = tid & (kWave - 1), wave = tid / kWave;
  const int rows = (T + kWave - 1) / kWave, rows_per_wave = (rows + kNW - 1) / kNW;
  const int r0 = min(wave * rows_per_wave, rows), r1 = min(r0 + rows_per_wave, rows);
  int carry = 0, top = INT32_MIN;   // sum and highest running sum of this wave's rows, from the wave's first position
  for (int r = r0; r < r1; ++r) {
    const int x = r * kWave + lane;
    const int inc = wave_scan_add(x < T ? a[x] : 0, lane);
    top = max(top, carry + inc);
    carry += __builtin_amdgcn_readlane(inc, kWave - 1);
  }
#pragma unroll
  for (int off = kWave / 2; off > 0; off >>= 1) top = max(top, __shfl_xor(top, off));
  if (lane == 0) {
    scratch[wave] = carry;
    scratch[kNW + wave] = top;
  }
  __syncthreads();
  int best = 0, before = 0;
  for (int w = 0; w < kNW; ++w) {
    const int t = scratch[kNW + w];
    if (t != INT32_MIN) best = max(best, before + t);
    before += scratch[w];
  }
  __syncthreads();
  return best;
}

// Loops over copies, nodes and edges run the same number of rounds in every lane, kUnroll
// items per lane and round, and read what they need from global memory at the top of a round:
// the loads of a round are in flight together instead of one behind the other.
constexpr int kUnroll = 4;

__global__ __launch_bounds__(kNT) __attribute__((amdgpu_waves_per_eu(8, 8)))
void decode_kernel(GraphView G, int64_t B, const int32_t* __restrict__ starts, const uint8_t* __restrict__ active,
                   moc_decode_result* __restrict__ out, int32_t* __restrict__ out_seq, DcLayout lay) {
  extern __shared__ int32_t lds[];
  int32_t* a = lds;                 // occupancy, then step number, then memory differences, per position
  int32_t* b = a + lay.T_pad;       // the sequence, then the last position each computation serves
  uint16_t* st = reinterpret_cast<uint16_t*>(b + lay.T_pad);   // start of each copy, kNoStart if inactive
  int32_t* scratch = reinterpret_cast<int32_t*>(st + lay.T_pad);
  int32_t* flags = scratch + 2 * kNW;   // [0] not decodable, [1] not a valid sequence, [2] duration
  const int tid = threadIdx.x, T = G.T, n = G.n, C = G.C, m = G.m;

  for (int64_t cand = blockIdx.x; cand < B; cand += gridDim.x) {
    const int32_t* s_row = starts + cand * T;
    const uint8_t* a_row = active + cand * T;
    int32_t* seq_row = out_seq ? out_seq + cand * T : nullptr;

    for (int x = tid; x <= T; x += kNT) a[x] = 0;
    if (tid < 4) flags[tid] = 0;
    __syncthreads();

    // scatter by start: a[x] = 1 where a computation happens
    for (int round = 0; round < T; round += kUnroll * kNT) {
      const int base = round + tid;
      // loads without conditions (lanes past the last copy read it again), a register per flag:
      // under a condition, or packed into one register, each load waits for the one before
      uint32_t on[kUnroll];
      int32_t s[kUnroll];
#pragma unroll
      for (int u = 0; u < kUnroll; ++u) {
        const int k = min(base + u * kNT, T - 1);
        on[u] = a_row[k];
        s[u] = s_row[k];
      }
#pragma unroll
      for (int u = 0; u < kUnroll; ++u) {
        const int k = base + u * kNT;
        if (k >= T) continue;
        uint32_t sk = kNoStart;
        if (on[u]) {
          if (s[u] < 0 || s[u] >= T) {
            flags[0] = 1;                       // Eq. (8)
          } else {
            sk = (uint32_t)s[u];
            if (atomicAdd(&a[s[u]], 1) != 0) flags[0] = 1;   // Eq. (6)
          }
        }
        st[k] = (uint16_t)sk;
      }
    }
    __syncthreads();
    if (flags[0]) {
      if (seq_row)
        for (int x = tid; x < T; x += kNT) seq_row[x] = -1;
      if (tid == 0) out[cand] = moc_decode_result{-1, 0, 0, 0};
      __syncthreads();
      continue;
    }

    // step number of each occupied position
    const int length = block_rank_of_ones(a, T, scratch, tid);

    if (seq_row) {
      for (int v = tid; v < n; v += kNT)
        for (int i = 0; i < C; ++i) {
          const uint32_t p = st[v * C + i];
          if (p != kNoStart) b[a[p]] = v;
        }
      for (int x = length + tid; x < T; x += kNT) b[x] = -1;
      __syncthreads();
      for (int x = tid; x < T; x += kNT) seq_row[x] = b[x];
      __syncthreads();
    }

    // every computation serves at least its own step; the difference array starts at zero
    for (int x = tid; x <= T; x += kNT) a[x] = 0;
    for (int k = tid; k < T; k += kNT) {
      const uint32_t p = st[k];
      if (p != kNoStart) b[p] = (int)p;
    }
    __syncthreads();

    // one lane per edge (u, v): each computation of v is served by the latest computation of u before it
    for (int round = 0; round < m; round += kUnroll * kNT) {
      const int base = round + tid;
      uint32_t pair[kUnroll];
#pragma unroll
      for (int u = 0; u < kUnroll; ++u) pair[u] = base + u * kNT < m ? G.edge_pair_c[base + u * kNT] : 0u;
#pragma unroll
      for (int u = 0; u < kUnroll; ++u) {
        if (base + u * kNT >= m) continue;
        const int uC = (int)(pair[u] & 0xFFFFu), vC = (int)(pair[u] >> 16);
        for (int i = 0; i < C; ++i) {
          const uint32_t p = st[vC + i];
          if (p == kNoStart) continue;
          int q = -1;
          for (int j = 0; j < C; ++j) {
            const uint32_t sj = st[uC + j];
            if (sj < p) q = max(q, (int)sj);    // kNoStart is above every position
          }
          if (q < 0) flags[1] = 1;
          else atomicMax(&b[q], (int)p);
        }
      }
    }
    __syncthreads();

    // per node: does it occur, what does it add to the duration; its outputs are held from p through b[p]
    int my_dur = 0;
    for (int round = 0; round < n; round += kUnroll * kNT) {
      const int base = round + tid;
      int2 sd[kUnroll];
#pragma unroll
      for (int u = 0; u < kUnroll; ++u) sd[u] = base + u * kNT < n ? G.size_dur[base + u * kNT] : make_int2(0, 0);
#pragma unroll
      for (int u = 0; u < kUnroll; ++u) {
        const int v = base + u * kNT;
        if (v >= n) continue;
        int times = 0;
        for (int i = 0; i < C; ++i) {
          const uint32_t p = st[v * C + i];
          if (p == kNoStart) continue;
          ++times;
          atomicAdd(&a[p], sd[u].x);
          atomicAdd(&a[b[p] + 1], -sd[u].x);
        }
        if (times == 0) flags[1] = 1;
        my_dur += times * sd[u].y;
      }
    }
    if (my_dur) atomicAdd(&flags[2], my_dur);
    __syncthreads();
    const int peak = block_peak_of_running_sum(a, T, scratch, tid);

    if (tid == 0) {
      const bool valid = flags[1] == 0;
      out[cand] = moc_decode_result{valid ? 1 : 0, length, valid ? (int64_t)peak : 0, valid ? (int64_t)flags[2] : 0};
    }
    __syncthreads();
  }
}


// ---- the same for C <= 4, with fewer passes (five barriers per candidate instead of twelve).
// The copies of a node are adjacent, so a node's starts are one or two LDS words; the position
// array holds the node computed at each position (v + 1) instead of a flag, so that the pass
// that ranks the occupied positions can write the sequence out itself, in order, and clear the
// array on its way; the running-sum scan at the end clears the difference array as it reads it.

// The copies of a node as they lie in a candidate's row: aligned as their elements are, no more
// (the global loads of this chip take several words at any word boundary).
template <int CT>
struct alignas(4) CopyStarts {
  int32_t s[CT];
};
template <int CT>
struct CopyFlags {
  uint8_t a[CT];
};

template <int CT>
struct NodeStarts {
  uint32_t s[CT];   // kNoStart if the copy is not computed
};

constexpr int starts_stride(int C) { return C == 3 ? 4 : C; }   // 16-bit entries per node

template <int CT>
__device__ __forceinline__ NodeStarts<CT> read_starts(const uint16_t* st, int v) {
  NodeStarts<CT> r;
  if constexpr (CT == 1) {
    r.s[0] = st[v];
  } else if constexpr (CT == 2) {
    const uint32_t w = *reinterpret_cast<const uint32_t*>(st + 2 * v);
    r.s[0] = w & 0xFFFFu; r.s[1] = w >> 16;
  } else {
    const uint2 w = *reinterpret_cast<const uint2*>(st + 4 * v);
    r.s[0] = w.x & 0xFFFFu; r.s[1] = w.x >> 16; r.s[2] = w.y & 0xFFFFu;
    if constexpr (CT == 4) r.s[3] = w.y >> 16;
  }
  return r;
}

// max over x in [0, T] of a[0] + ... + a[x] (at least 0); every a[x] is left at zero.  The entry
// at T only ever holds releases (values <= 0), so it cannot raise the maximum.  A wave takes
// rows of 256 positions, four per lane in one 16-byte read; `words` (a multiple of 4, > T) is
// the length of the array.
__device__ int block_peak_and_clear(int32_t* a, int words, int32_t* scratch, int tid) {
  const int lane = tid & (kWave - 1), wave = tid / kWave;
  const int rows = (words + 4 * kWave - 1) / (4 * kWave), rows_per_wave = (rows + kNW - 1) / kNW;
  const int r0 = min(wave * rows_per_wave, rows), r1 = min(r0 + rows_per_wave, rows);
  int carry = 0, top = 0;   // last lane: sum and highest running sum of this wave's rows, from the wave's first position
  for (int r = r0; r < r1; ++r) {
    const int x = (r * kWave + lane) * 4;
    int4 v = make_int4(0, 0, 0, 0);
    if (x < words) {
      v = *reinterpret_cast<int4*>(a + x);
      *reinterpret_cast<int4*>(a + x) = make_int4(0, 0, 0, 0);
    }
    int S = v.x, P = max(S, 0);
    S += v.y; P = max(P, S);
    S += v.z; P = max(P, S);
    S += v.w; P = max(P, S);
    wave_combine_ordered(S, P);
    top = max(top, carry + P);
    carry += S;
  }
  if (lane == kWave - 1) {   // the lane that holds the rows' combined values
    scratch[wave] = carry;
    scratch[kNW + wave] = top;
  }
  __syncthreads();
  int best = 0, before = 0;
  for (int w = 0; w < kNW; ++w) {
    best = max(best, before + scratch[kNW + w]);
    before += scratch[w];
  }
  // No barrier here: the caller's next write to `scratch` lies behind its next barrier, and the
  // array is clear for every wave since the barrier above.
  return best;
}

// SMALL: the graph has at most kUnroll * kNT nodes, a lane's nodes are the same for every
// candidate: their sizes and durations stay in registers, and the starts and flags of the
// workgroup's next candidate are asked for while this one is still being worked on (after the
// edge pass, whose own loads would otherwise queue behind them), so that its first phase does
// not begin with a wait for HBM.
template <int CT, bool SMALL>
__global__ __launch_bounds__(kNT) __attribute__((amdgpu_waves_per_eu(8, 8)))
void decode_fixed_kernel(GraphView G, int64_t B, const int32_t* __restrict__ starts, const uint8_t* __restrict__ active,
                         moc_decode_result* __restrict__ out, int32_t* __restrict__ out_seq, DcLayout lay) {
  extern __shared__ int32_t lds[];
  constexpr int SS = starts_stride(CT);
  int32_t* a = lds;                 // node computed at each position (v + 1), then memory differences
  int32_t* b = a + lay.T_pad;       // the last position each computation serves
  uint16_t* st = reinterpret_cast<uint16_t*>(b + lay.T_pad);   // [n][SS] start of each copy, kNoStart if not computed
  int32_t* scratch = reinterpret_cast<int32_t*>(st) + lay.st_words;
  int32_t* flag_words = scratch + 2 * kNW;   // two sets of [0] not decodable, [1] not a valid sequence, [2] duration
  const int tid = threadIdx.x;
  const int T = G.T, n = G.n, m = G.m;

  for (int x = tid; x < lay.T_pad; x += kNT) a[x] = 0;
  if (tid < 8) flag_words[tid] = 0;
  if (tid < SS) st[n * SS + tid] = (uint16_t)kNoStart;   // node n: behind the last node, never computed; padding edges lead there
  // The loads of a round of nodes are issued without conditions (lanes past the last node read
  // it again and drop what they get) and all of them before the first is looked at; the flags
  // take a register each.  Loads under a condition, or flags packed into the bytes of one
  // register, end up one behind the other, each waiting for the one before.
  struct Round {
    int32_t s[kUnroll][CT];
    uint32_t on[kUnroll][CT];
  };
  // (the candidate's rows are scalar base addresses, a lane adds a 32-bit offset)
  auto request = [&](int64_t c, int round, int t, Round& r) {
    const char* const s_row = reinterpret_cast<const char*>(starts + c * T);
    const char* const a_row = reinterpret_cast<const char*>(active + c * T);
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
      const uint32_t off = (uint32_t)min(round + u * kNT + t, n - 1) * CT;
      const CopyStarts<CT> sv = *reinterpret_cast<const CopyStarts<CT>*>(s_row + off * 4u);
      const CopyFlags<CT> av = *reinterpret_cast<const CopyFlags<CT>*>(a_row + off);
#pragma unroll
      for (int i = 0; i < CT; ++i) {
        r.s[u][i] = sv.s[i];
        r.on[u][i] = av.a[i];
      }
    }
  };
  [[maybe_unused]] Round ahead;            // SMALL: the workgroup's next candidate
  [[maybe_unused]] int2 my_sd[kUnroll];    // SMALL: m_v, w_v of the lane's nodes
  if constexpr (SMALL) {
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) my_sd[u] = G.size_dur[min(u * kNT + tid, n - 1)];
    request(blockIdx.x, 0, tid, ahead);   // the grid is not larger than the batch
  }
  __syncthreads();

  int turn = 0;
  for (int64_t cand = blockIdx.x; cand < B; cand += gridDim.x, turn ^= 1) {
    // What derives from the thread index (row bounds, LDS addresses) is formed again for every
    // candidate: kept across candidates it takes registers that the next candidate's copies need.
    int t_ = tid;
    asm volatile("" : "+v"(t_));
    const int lane_ = t_ & (kWave - 1);
    const int wave_ = __builtin_amdgcn_readfirstlane(t_ / kWave);
    int32_t* seq_row = out_seq ? out_seq + cand * T : nullptr;
    int32_t* flags = flag_words + 4 * turn;
    const int64_t after = cand + gridDim.x < B ? cand + gridDim.x : cand;   // SMALL: whose loads go out next (the last candidate asks for itself again)

    // ---- who is computed where; every computation serves at least its own step
    // What makes the candidate undecodable is collected and reported once per round: the
    // compare-and-swaps of a round are all under way before the first answer is looked at.
    auto place = [&](int round, const Round& r) {
      uint32_t taken = 0;    // != 0: a position was taken already, Eq. (6)
      bool outside = false;  // a start outside [0, T), Eq. (8)
#pragma unroll
      for (int u = 0; u < kUnroll; ++u) {
        const int v = round + u * kNT + t_;
        if (v >= n) continue;
        uint32_t where[SS];   // the node's entry of `st`, written in one piece
#pragma unroll
        for (int i = 0; i < SS; ++i) where[i] = kNoStart;
#pragma unroll
        for (int i = 0; i < CT; ++i) {
          if (r.on[u][i]) {
            if (r.s[u][i] < 0 || r.s[u][i] >= T) {
              outside = true;
            } else {
              const uint32_t sk = (uint32_t)r.s[u][i];
              where[i] = sk;
              taken |= (uint32_t)atomicCAS(&a[sk], 0, v + 1);   // the node there before, + 1
              b[sk] = (int)sk;
            }
          }
        }
        if constexpr (SS == 1) st[v] = (uint16_t)where[0];
        else if constexpr (SS == 2) *reinterpret_cast<uint32_t*>(st + 2 * v) = where[0] | where[1] << 16;
        else *reinterpret_cast<uint2*>(st + 4 * v) = make_uint2(where[0] | where[1] << 16, where[2] | where[3] << 16);
      }
      if (outside || taken != 0) flags[0] = 1;
    };
    if constexpr (SMALL) {
      place(0, ahead);
    } else {
      for (int round = 0; round < n; round += kUnroll * kNT) {
        Round now;
        request(cand, round, t_, now);
        __builtin_amdgcn_sched_barrier(0);
        place(round, now);
      }
    }
    __syncthreads();
    if (flags[0]) {
      if constexpr (SMALL) request(after, 0, t_, ahead);
      if (seq_row)
        for (int x = t_; x < T; x += kNT) seq_row[x] = -1;
      for (int x = t_; x <= T; x += kNT) a[x] = 0;
      __syncthreads();
      if (t_ == 0) {
        out[cand] = moc_decode_result{-1, 0, 0, 0};
        flags[0] = 0;
      }
      __syncthreads();
      turn ^= 1;   // the same set of flags serves the next candidate (it is clear again)
      continue;
    }
    if (t_ == 0) {   // the other set, for the workgroup's next candidate
      int32_t* other = flag_words + 4 * (turn ^ 1);
      other[0] = 0; other[1] = 0; other[2] = 0;
    }

    // ---- the sequence: occupied positions in order.  A wave_ owns rows of 256 positions, four per lane_.
    const int rows = (lay.T_pad + 4 * kWave - 1) / (4 * kWave), rows_per_wave = (rows + kNW - 1) / kNW;
    const int r0 = min(wave_ * rows_per_wave, rows), r1 = min(r0 + rows_per_wave, rows);
    int mine = 0;
    for (int r = r0; r < r1; ++r) {
      const int x = (r * kWave + lane_) * 4;
      if (x < lay.T_pad) {
        const int4 who = *reinterpret_cast<const int4*>(a + x);
        mine += (who.x != 0) + (who.y != 0) + (who.z != 0) + (who.w != 0);
      }
    }
    mine = __builtin_amdgcn_readlane(wave_scan_add(mine, lane_), kWave - 1);
    if (lane_ == 0) scratch[wave_] = mine;
    __syncthreads();
    int before = 0, length = 0;
    for (int w = 0; w < kNW; ++w) {
      const int t = scratch[w];
      if (w < wave_) before += t;
      length += t;
    }
    for (int r = r0; r < r1; ++r) {
      const int x = (r * kWave + lane_) * 4;
      int4 who = make_int4(0, 0, 0, 0);
      if (x < lay.T_pad) who = *reinterpret_cast<const int4*>(a + x);
      const int cnt = (who.x != 0) + (who.y != 0) + (who.z != 0) + (who.w != 0);
      const int incl = wave_scan_add(cnt, lane_);
      if (cnt) {
        int at = before + incl - cnt;
        if (seq_row) {
          if (who.x) seq_row[at++] = who.x - 1;
          if (who.y) seq_row[at++] = who.y - 1;
          if (who.z) seq_row[at++] = who.z - 1;
          if (who.w) seq_row[at++] = who.w - 1;
        }
        *reinterpret_cast<int4*>(a + x) = make_int4(0, 0, 0, 0);
      }
      before += __builtin_amdgcn_readlane(incl, kWave - 1);
    }
    if (seq_row)
      for (int x = length + t_; x < T; x += kNT) seq_row[x] = -1;

    // ---- one lane_ per edge (u, v): each computation of v is served by the latest computation of u before it
    bool unserved = false;
    auto serve = [&](const NodeStarts<CT>& su, const NodeStarts<CT>& sv) {
#pragma unroll
      for (int i = 0; i < CT; ++i) {
        const uint32_t p = sv.s[i];
        int q = -1;
#pragma unroll
        for (int j = 0; j < CT; ++j)
          if (su.s[j] < p) q = max(q, (int)su.s[j]);    // kNoStart is above every position
        const bool computed = p != kNoStart;
        if (computed && q >= 0) atomicMax(&b[q], (int)p);
        unserved = unserved || (computed && q < 0);
      }
    };
    // The same for two copies per node on the entries of `st` as they are, both copies of the
    // consumer at once in 16-bit halves of a register.  As signed 16-bit numbers kNoStart is -1
    // and every position is far below 2^15 (LDS bounds T), so "the latest start of the producer
    // before p, or -1" is max over the producer's copies of (s < p ? s : -1) = s | ((p - 1 - s) >> 15),
    // and a consumer copy that is not computed (p = -1) gets -1 by itself.
    [[maybe_unused]] uint32_t unserved2 = 0;   // sign bits of the halves: computed and not served
    [[maybe_unused]] auto serve2 = [&](uint32_t su, uint32_t sv) {
      typedef short Halves __attribute__((ext_vector_type(2)));
      const auto halves = [](uint32_t x) { return __builtin_bit_cast(Halves, x); };
      const auto word = [](Halves x) { return __builtin_bit_cast(uint32_t, x); };
      const Halves before = halves(sv) - Halves{1, 1};                 // p - 1, per copy of the consumer
      const uint32_t s0 = __builtin_amdgcn_perm(su, su, 0x01000100u);   // the producer's first start in both halves
      const uint32_t s1 = __builtin_amdgcn_perm(su, su, 0x03020302u);   // its second
      const uint32_t c0 = s0 | word((before - halves(s0)) >> 15);
      const uint32_t c1 = s1 | word((before - halves(s1)) >> 15);
      const Halves q = __builtin_elementwise_max(halves(c0), halves(c1));
      unserved2 |= word(q) & ~sv;
      const int q0 = q.x, q1 = q.y;
      if (q0 >= 0) atomicMax(&b[q0], (int)(sv & 0xFFFFu));
      if (q1 >= 0) atomicMax(&b[q1], (int)(sv >> 16));
    };
    for (int round = 0; round < m; round += kUnroll * kNT) {
      const int base = round + t_;
      uint32_t pair[kUnroll];
#pragma unroll
      for (int u = 0; u < kUnroll; ++u) {
        const uint32_t got = G.edge_pair_c[min(base + u * kNT, m - 1)];
        pair[u] = base + u * kNT < m ? got : (uint32_t)T << 16;   // beyond the list: an edge into node n
      }
#pragma unroll
      for (int u = 0; u < kUnroll; ++u) {
        if constexpr (CT == 2) serve2(*reinterpret_cast<const uint32_t*>(st + (pair[u] & 0xFFFFu)), *reinterpret_cast<const uint32_t*>(st + (pair[u] >> 16)));
        else serve(read_starts<CT>(st, (int)(pair[u] & 0xFFFFu) / CT), read_starts<CT>(st, (int)(pair[u] >> 16) / CT));
      }
    }
    if (unserved || (unserved2 & 0x80008000u)) flags[1] = 1;
    if constexpr (SMALL) request(after, 0, t_, ahead);
    __syncthreads();

    // ---- per node: does it occur, what does it add to the duration; its outputs are held from p through b[p]
    int my_dur = 0;
    for (int round = 0; round < n; round += kUnroll * kNT) {
      const int base = round + t_;
      int2 sd[kUnroll];
#pragma unroll
      for (int u = 0; u < kUnroll; ++u) {
        if constexpr (SMALL) sd[u] = my_sd[u];
        else sd[u] = G.size_dur[min(base + u * kNT, n - 1)];
      }
#pragma unroll
      for (int u = 0; u < kUnroll; ++u) {
        const int v = base + u * kNT;
        if (v >= n) continue;
        const NodeStarts<CT> sv = read_starts<CT>(st, v);
        int times = 0;
#pragma unroll
        for (int i = 0; i < CT; ++i) {
          const uint32_t p = sv.s[i];
          if (p == kNoStart) continue;
          ++times;
          atomicAdd(&a[p], sd[u].x);
          atomicAdd(&a[b[p] + 1], -sd[u].x);
        }
        if (times == 0) flags[1] = 1;
        my_dur += times * sd[u].y;
      }
    }
    if (my_dur) atomicAdd(&flags[2], my_dur);
    __syncthreads();
    const int peak = block_peak_and_clear(a, lay.T_pad, scratch, t_);

    if (t_ == 0) {
      const bool valid = flags[1] == 0;
      out[cand] = moc_decode_result{valid ? 1 : 0, length, valid ? (int64_t)peak : 0, valid ? (int64_t)flags[2] : 0};
    }
  }
}

template <int CT>
auto fixed_kernel_for(int n) {
  return n <= kUnroll * kNT ? decode_fixed_kernel<CT, true> : decode_fixed_kernel<CT, false>;
}

}  // namespace

extern "C" int moc_decode_batch(const moc_graph* g, int64_t B, const int32_t* starts, const uint8_t* active,
                                moc_decode_result* out, int32_t* out_seq, void* hip_stream) {
  if (!g || B < 0) return MOC_EINVAL;
  if (B == 0) return MOC_OK;
  if (!starts || !active || !out) return MOC_EINVAL;
  if (((uintptr_t)starts & 3) || ((uintptr_t)out & 7) || ((uintptr_t)out_seq & 3)) return MOC_EINVAL;
  int dev = -1;
  MOC_HIP(hipGetDevice(&dev));
  if (dev != g->device) return MOC_EDEVICE;
  const DcLayout lay = dc_layout(g->view.n, g->view.C);
  if (lay.bytes > g->max_lds) return MOC_EOVERFLOW;
  auto kern = decode_kernel;
  switch (g->view.C) {
    case 1: kern = fixed_kernel_for<1>(g->view.n); break;
    case 2: kern = fixed_kernel_for<2>(g->view.n); break;
    case 3: kern = fixed_kernel_for<3>(g->view.n); break;
    case 4: kern = fixed_kernel_for<4>(g->view.n); break;
    default: break;
  }
  int per_cu = 0;
  if (const int rc = moc_kernel_occupancy(g, reinterpret_cast<const void*>(kern), kNT, lay.bytes, false, &per_cu)) return rc;
  const int64_t resident = (int64_t)per_cu * g->num_cu;
  const unsigned grid = (unsigned)(B < resident ? B : resident);
  hipLaunchKernelGGL(kern, dim3(grid), dim3(kNT), lay.bytes, static_cast<hipStream_t>(hip_stream), g->view, B,
                     starts, active, out, out_seq, lay);
  MOC_HIP(hipGetLastError());
  return MOC_OK;
}
