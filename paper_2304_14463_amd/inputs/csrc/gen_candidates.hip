// Device twin of the seeded candidate generator (inputs/candidates.py): the
// same draws, bit for bit, written straight into HBM so that large batches
// never cross PCIe.  One thread per (candidate b, node v) writes the C copies
// of that node.  Holds no arithmetic of the evaluated method.
//
// Hash: the 64-bit finaliser of SplitMix64 (Steele, Lea, Flood 2014) chained
// over (seed, b, v, j), j = fixed counter of the decision.
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace {

constexpr uint64_t kGolden = 0x9E3779B97F4A7C15ull;
constexpr uint64_t kSeedXor = 0xC0FFEE5EEDull;

__device__ __forceinline__ uint64_t mix64(uint64_t z) {
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
  return z ^ (z >> 31);
}

__global__ void gen_candidates_kernel(uint64_t seed, int n, int C, int64_t B_total, const int32_t* __restrict__ pos,
                                      const int32_t* __restrict__ out_ptr, const int32_t* __restrict__ cons_pos,
                                      const int32_t* __restrict__ win_hi, const int32_t* __restrict__ ncut,
                                      int64_t b0, int64_t count, int dense, int32_t* __restrict__ starts,
                                      int32_t* __restrict__ ends, uint8_t* __restrict__ active) {
  const int64_t gid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (gid >= count * n) return;
  const int64_t r = gid / n;
  const int v = (int)(gid - r * n);
  const int64_t b = b0 + r;
  const int T = n * C;
  const uint64_t kb = mix64((seed ^ kSeedXor) + kGolden * (uint64_t)(b + 1));
  const uint64_t kv = mix64(kb + kGolden * (uint64_t)(v + 1));
  auto draw = [&](int j) { return mix64(kv + kGolden * (uint64_t)(j + 1)); };

  const int o0 = out_ptr[v], d = out_ptr[v + 1] - o0;
  const int pv = pos[v];
  const int end_default = d ? max(pv, cons_pos[o0 + d - 1]) : pv;
  const bool type_b = b >= B_total / 2;
  int32_t* s = starts + r * T + (int64_t)v * C;
  int32_t* e = ends + r * T + (int64_t)v * C;
  uint8_t* a = active + r * T + (int64_t)v * C;

  for (int i = 0; i < C; ++i) { s[i] = 0; e[i] = 0; a[i] = 0; }
  s[0] = pv; e[0] = end_default; a[0] = 1;

  const int nc = ncut[v], wh = win_hi[v];
  if (dense) {   // every node computed C times in a row, each copy kept until the next one starts
    int nxt = min(end_default + C - 1, T - 1);
    for (int i = C - 1; i >= 1; --i) {
      if ((draw(8 + i) & 7) == 0) continue;
      a[i] = 1; s[i] = pv + i; e[i] = nxt;
      nxt = pv + i;
    }
    e[0] = nxt;
  }
  int lo = 0;
  for (int i = 1; i < C && nc >= 1 && !dense; ++i) {
    const int avail = nc - lo;
    const uint64_t gate = draw(2 * i), pick = draw(2 * i + 1);
    if (avail < 1 || (gate & 3) != 0) break;
    const int c = lo + (int)((pick & 0xFFFFFFFFull) % (uint64_t)avail);
    const int cut = cons_pos[o0 + c];
    const int span = min(cons_pos[o0 + c + 1] - 1, wh) - cut;
    const int nfree = max(span - span / C, 1);
    const int q = (int)((pick >> 32) % (uint64_t)nfree);
    e[i - 1] = cut;
    s[i] = cut + 1 + q + q / (C - 1);
    e[i] = end_default;
    a[i] = 1;
    lo = c + 1;
  }
  if (type_b) {
    for (int i = 0; i < C; ++i) {
      if (!a[i]) continue;
      const uint64_t rs = draw(16 + 2 * i), re = draw(16 + 2 * i + 1);
      if ((rs & 3) == 0) s[i] = min(max(s[i] + (int)((rs >> 8) % 9) - 4, 0), T - 1);
      if ((re & 3) == 0) e[i] = min(max(e[i] + (int)((re >> 8) % 9) - 4, 0), T - 1);
    }
  }
}

}  // namespace

// Fill starts/ends/active [count][n*C] (device) with candidates b0 .. b0+count-1 of a batch of
// B_total (dense != 0: the dense batch).  Tables are device arrays as produced by inputs.candidates.candidate_tables.
// Returns the hipError_t of the launch (0 = success).
extern "C" int mocgen_candidates(uint64_t seed, int32_t n, int32_t C, int64_t B_total, const int32_t* pos,
                                 const int32_t* out_ptr, const int32_t* cons_pos, const int32_t* win_hi,
                                 const int32_t* ncut, int64_t b0, int64_t count, int32_t dense, int32_t* starts,
                                 int32_t* ends, uint8_t* active, void* hip_stream) {
  if (count <= 0 || n <= 0) return 0;
  const int64_t threads = count * n;
  const int block = 256;
  const int64_t grid = (threads + block - 1) / block;
  if (grid > 0x7FFFFFFF) return (int)hipErrorInvalidValue;
  hipLaunchKernelGGL(gen_candidates_kernel, dim3((unsigned)grid), dim3(block), 0, static_cast<hipStream_t>(hip_stream),
                     seed, n, C, B_total, pos, out_ptr, cons_pos, win_hi, ncut, b0, count, dense, starts, ends, active);
  return (int)hipGetLastError();
}
