// moc_eval_batch: one workgroup evaluates one candidate at a time (Eq. (1)-(8)
// of the paper's Section 2.1) with its whole working set in LDS.
//
// Per candidate (register-resident kernel, C <= 4):
//   phase 1  one lane per node, nodes in id order.  The lane holds the C copies
//            of its node in registers (requested from HBM while the previous
//            candidate was being worked on), classifies them (active / live),
//            counts Eq. (2),(7),(8) and Eq. (3), adds the node's share of
//            Eq. (1), stages the node in LDS as packed words s | e << 16, and
//            scatters every live copy into the memory-delta array (+m_v at s,
//            -m_v at e+1: the closed intervals of Eq. (4)) and into a bitmap of
//            occupied start positions (Eq. (6)).
//   phase 2  (a) the delta array is cut into chunks of 32 positions; a thread reads
//            its chunk with 16-byte LDS loads, zeroes it, and reduces it to
//            (sum, max prefix); chunks combine associatively in position order,
//            which yields the peak of Eq. (4) without materialising the profile;
//            (b) popcount of the start bitmap: distinct start positions, so that
//            sum_t max(0, cnt_t - 1) = live copies - distinct starts;
//            (c) one lane per edge (u,v), Eq. (5).  The edges of a lane never
//            change, so they stay in registers.  C <= 2: the records of u and v
//            are fetched whole and every live copy of v is tested against the
//            copies of u.  C >= 3: copies beyond the first are rarely live, so
//            the first copies are kept in an array of their own (one word per
//            node), the start of each node's first copy once more in an array
//            of 16-bit entries that the node's in-edges read, and an edge is
//            settled on those two reads when the first copy of u covers the
//            first copy of v; a consumer with other live copies carries a mark
//            in its 16-bit entry that makes this test fail.  The edges that are
//            not settled go to a queue per wave and take the full test
//            afterwards, 64 per instruction.
//            Phase 2 touches no global memory; the loads of the workgroup's next
//            candidate are issued in slices between its steps, so that HBM
//            streams while the LDS work runs.
// Predicates are lane masks: a vector compare writes a 64-bit scalar, the scalar
// unit combines the masks, counts come from popcounts or an add-with-carry per
// lane.  Which candidate a workgroup takes next is drawn from a counter, an
// iteration ahead (see the kernel).
// What shaped this, measured on gfx950.  A SIMD needs 4 clocks for a 64-lane
// vector instruction, and with one 1024-thread workgroup per compute unit (the
// LDS working set of a large graph allows no more) only 4 waves share a SIMD and
// meet at two barriers per candidate: the vector unit is the busiest part (60 %
// at n = 5000), scalar instructions run beside it.  Hence the scalar masks.
// LDS, per compute unit: a 64-lane 4-byte access to random addresses takes 2.6
// times as long as one whose 32 lanes served together fall into distinct banks,
// read, write or atomic alike; 8-byte accesses (16 lanes at a time) 1.7 times.
// Hence records and chunks are sized for wide accesses, nothing is read twice,
// and the edge list is laid out for distinct banks at upload.
// All arithmetic is integer: results do not depend on the order in which
// lanes or workgroups run.
#include <type_traits>

#include "moc_internal.h"

namespace {

constexpr int kRedStride = 8;      // ints per wave in the cross-wave exchange area (4 in use)
constexpr int kRedPass = 4;        // word of that area through which thread 0 passes a value to all
constexpr int kMaxIters = 6;       // nodes per lane the register-resident kernel is built for
constexpr int kEdgesPerNode = 3;   // edges per lane = kEdgesPerNode * nodes per lane
// The delta array is kept in chunks of 32 positions, one per scanning lane, stored 36 words
// apart (16 lanes x 16 bytes then hit 64 distinct banks); workgroups of one or two waves take
// chunks of 16 positions, 20 words apart, so that more of their lanes share the scan.
constexpr int chunk_positions(int nt) { return nt <= 128 ? 16 : 32; }
constexpr int chunk_stride(int nt) { return chunk_positions(nt) + 4; }
constexpr int64_t kMaxLaunch = (int64_t)1 << 31;   // candidates per launch
static_assert(MOC_MAX_T < 0x8000, "bit 15 of a consumer's 16-bit start marks nodes with other live copies (C >= 3)");
constexpr int kQueueCap = 320;     // C >= 3: edges a wave sets aside before it has to work them off

// ------------------------------------------------------------------ LDS layouts
// Word offsets of the arrays inside the dynamic LDS segment, and their sizes in words.
struct LdsLayout {
  int packed_off, cons_off, rest_off, delta_off, occ_off, red_off, queue_off;
  int chunk;       // general kernel: delta entries per thread (odd: conflict-free strided reads)
  int n_chunks;    // register-resident kernel: chunks of chunk_positions(nt) positions
  int delta_len;
  int packed_len;  // node records (register-resident kernel, C >= 3: first copies, then the rest)
  int occ_words;   // ceil(T / 32)
  int qcap;        // register-resident kernel, C >= 3: entries per wave in the queue of edges set aside
  int edge_slices; // register-resident kernel: slices of kEdgesPerNode edges per lane that hold edges
  int edge_slots;  // ... and edges per lane that do (the last slice may hold fewer than kEdgesPerNode)
  int bytes;
};

constexpr int round4(int x) { return (x + 3) & ~3; }

// Register-resident kernel.  Node records first, at LDS address 0: with C <= 2 one record of
// C words per node; with C >= 3 the first copy of every node (1 word), then 16 bits per node
// for its role as a consumer (the start of its first copy, bit 15 set if it has other live
// copies), then the other copies of every node (2 words for C = 3, 4 for C = 4; the three
// arrays lie within the first 128 KB, so that a 16-bit index reaches an entry of the second).
// Dummy nodes end the arrays: C <= 2 one
// node n that is never live; C >= 3 a consumer n and a provider n + 1 that form a satisfied
// edge, and a node n + 2 that is never live.  Then the delta array in padded chunks, the start bitmap, the cross-wave
// exchange area and (C >= 3) a queue per wave, shrunk to fit when LDS is short.
LdsLayout fast_layout(int n, int m, int C, int nt, int max_lds) {
  const int T = n * C, nw = nt / kWave;
  LdsLayout l;
  l.chunk = 0;
  l.n_chunks = (T + 1 + chunk_positions(nt) - 1) / chunk_positions(nt);
  l.delta_len = l.n_chunks * chunk_stride(nt);
  const int first_len = round4((n + (C >= 3 ? 3 : 1)) * moc_node_stride(C));
  const int rest_len = C >= 3 ? round4((n + 3) * (C == 3 ? 2 : 4)) : 0;
  const int cons_len = C >= 3 ? round4((n + 3 + 1) / 2) : 0;   // 16 bits per node
  l.packed_len = first_len + cons_len + rest_len;
  l.occ_words = (T + 31) / 32;
  l.packed_off = 0;
  l.cons_off = first_len;
  l.rest_off = first_len + cons_len;
  l.delta_off = l.packed_len;
  l.occ_off = l.delta_off + l.delta_len;
  l.red_off = l.occ_off + l.occ_words;
  l.queue_off = l.red_off + nw * kRedStride;
  l.edge_slices = (m + kEdgesPerNode * nt - 1) / (kEdgesPerNode * nt);
  l.edge_slots = (m + nt - 1) / nt;
  l.qcap = C >= 3 ? kQueueCap : 0;
  l.bytes = 4 * (l.queue_off + nw * l.qcap);
  while (l.bytes > max_lds && l.qcap > kEdgesPerNode * kWave) {   // a slice of edges must fit
    l.qcap -= kWave;
    l.bytes = 4 * (l.queue_off + nw * l.qcap);
  }
  return l;
}

LdsLayout general_layout(int n, int C, int nt) {
  const int T = n * C;
  LdsLayout l;
  l.chunk = ((T + 1 + nt - 1) / nt) | 1;
  l.n_chunks = 0;
  l.delta_len = nt * l.chunk;
  l.packed_len = round4(T);
  l.occ_words = (T + 31) / 32;
  l.delta_off = 0;
  l.packed_off = l.delta_len;
  l.rest_off = l.packed_off;
  l.occ_off = l.packed_off + l.packed_len;
  l.red_off = l.occ_off + l.occ_words;
  l.queue_off = l.red_off + (nt / kWave) * kRedStride;
  l.qcap = 0;
  l.edge_slices = 0;
  l.edge_slots = 0;
  l.bytes = 4 * l.queue_off;
  return l;
}

struct Lds {
  int32_t* delta;
  uint32_t* packed;
  uint32_t* rest;
  uint16_t* cons;
  uint32_t* occ;
  int32_t* red;
  uint32_t* queue;
};

__device__ __forceinline__ Lds carve(uint32_t* base, const LdsLayout& lay) {
  Lds l;
  l.delta = reinterpret_cast<int32_t*>(base + lay.delta_off);
  l.packed = base + lay.packed_off;
  l.rest = base + lay.rest_off;
  l.cons = reinterpret_cast<uint16_t*>(base + lay.cons_off);
  l.occ = base + lay.occ_off;
  l.red = reinterpret_cast<int32_t*>(base + lay.red_off);
  l.queue = base + lay.queue_off;
  return l;
}

// ------------------------------------------------------------------ wave helpers
template <int CTRL>
__device__ __forceinline__ int dpp_move(int v) {
  return __builtin_amdgcn_update_dpp(0, v, CTRL, 0xF, 0xF, true);
}

// Sum over the 64 lanes, returned in every lane (wave-uniform).
__device__ __forceinline__ int wave_sum(int v) {
  v += dpp_move<0xB1>(v);    // quad_perm [1,0,3,2]
  v += dpp_move<0x4E>(v);    // quad_perm [2,3,0,1]
  v += dpp_move<0x141>(v);   // row_half_mirror
  v += dpp_move<0x140>(v);   // row_mirror: every lane of a row of 16 holds the row's sum
  return __builtin_amdgcn_readlane(v, 0) + __builtin_amdgcn_readlane(v, 16) + __builtin_amdgcn_readlane(v, 32) +
         __builtin_amdgcn_readlane(v, 48);
}

// (sum, max prefix) of consecutive segments, one per lane (max prefix >= 0 and >= sum, as a
// running maximum that starts at 0 gives it), combined in lane order; the last lane ends with
// the whole wave (the result stays in a vector register: scalar registers are scarce where this
// is called).  Each lane takes in the lanes before it: inside rows of 16 by shifts of 1, 2, 4,
// 8 (a lane with no source gets (0, 0), which changes nothing), then lane 15 of rows 0 and 2
// goes to rows 1 and 3, then lane 31 to rows 2 and 3; lane 63 ends with the whole wave.
template <int CTRL, int ROWS>
__device__ __forceinline__ void absorb_earlier(int& S, int& P) {
  const int Se = __builtin_amdgcn_update_dpp(0, S, CTRL, ROWS, 0xF, true);
  const int Pe = __builtin_amdgcn_update_dpp(0, P, CTRL, ROWS, 0xF, true);
  P = max(Pe, Se + P);
  S = Se + S;
}
// IN_ALU: with the lane shifts of the vector ALU itself, else through the LDS crossbar, which
// takes longer but leaves the vector ALU to the other waves.  Measured: the first is faster with
// workgroups of up to 512 threads (n = 442: 43.9 -> 45.4 % of HBM peak, n = 1000: 57.4 -> 60.0 %),
// the second with 1024 (n = 5000: 63.9 against 63.1 %), where the vector ALU is the busiest unit
// and eight waves of a workgroup combine at the same time.
template <bool IN_ALU>
__device__ __forceinline__ void wave_combine_ordered(int lane, int& S, int& P) {
  if constexpr (IN_ALU) {
    absorb_earlier<0x111, 0xF>(S, P);   // row_shr:1
    absorb_earlier<0x112, 0xF>(S, P);   // row_shr:2
    absorb_earlier<0x114, 0xF>(S, P);   // row_shr:4
    absorb_earlier<0x118, 0xF>(S, P);   // row_shr:8
    absorb_earlier<0x142, 0xA>(S, P);   // row_bcast:15 into rows 1 and 3
    absorb_earlier<0x143, 0xC>(S, P);   // row_bcast:31 into rows 2 and 3
  } else {
#pragma unroll
    for (int off = 1; off < kWave; off <<= 1) {   // lane l takes in lanes l-2*off+1 .. l-off
      const int Se = __shfl_up(S, off), Pe = __shfl_up(P, off);
      if (lane >= off) {
        P = max(Pe, Se + P);
        S = Se + S;
      }
    }
  }
}

__device__ __forceinline__ bool is_live(uint32_t packed) { return (packed & 0xFFFFu) != 0xFFFFu; }

// Eq. (5) for one consumer start x (xs = x << 16) against one staged provider copy:
// s_u + 1 <= x  and  x <= e_u.  A copy that is not live has s = 0xFFFF and fails.
__device__ __forceinline__ bool covers(uint32_t pu, uint32_t x, uint32_t xs) { return ((pu & 0xFFFFu) < x) & (pu >= xs); }

template <int NT>
__device__ __forceinline__ int count_distinct_starts(const Lds& L, const LdsLayout& lay, int tid) {
  int distinct = 0;
  for (int w = tid; w < lay.occ_words; w += NT) {
    distinct += __popc(L.occ[w]);
    L.occ[w] = 0;
  }
  return distinct;
}

// Cross-wave combine.  Every wave leaves its partial results in LDS; after the
// barrier the lanes of wave 0 pick up one wave each and reduce in registers.
// WAVE_TOTALS: viol and nlive are already sums over the wave (counted with ballots).
// `pass` (thread 0's value) travels through the same barrier: every thread gets it back in
// `passed`.  The kernel hands the workgroup's next candidate index around this way.
template <int NT, bool WAVE_TOTALS = false>
__device__ __forceinline__ void finish(const Lds& L, const GraphView& g, int tid, int lane, int wave, int S, int P,
                                       int viol, int nlive, int distinct, int dur, moc_result* __restrict__ out,
                                       int64_t b, uint32_t pass = 0, uint32_t* passed = nullptr) {
  constexpr int NW = NT / kWave;
  if (passed && tid == 0) L.red[kRedPass] = (int32_t)pass;
  if constexpr (!WAVE_TOTALS) {
    viol = wave_sum(viol);
    nlive = wave_sum(nlive);
  }
  distinct = wave_sum(distinct);
  dur = wave_sum(dur);
  if constexpr (NW > 1) {
    if (lane == kWave - 1) {   // the lane that holds the wave's (S, P); the sums are in every lane
      int32_t* r = L.red + wave * kRedStride;
      r[0] = S; r[1] = P; r[2] = viol + nlive - distinct; r[3] = dur;
    }
    __syncthreads();
    if (passed) *passed = (uint32_t)L.red[kRedPass];
    if (wave != 0) return;
    if constexpr (NW <= 4) {   // few waves: every lane adds them up by itself (the reads are broadcasts)
      S = 0; P = 0; viol = 0; dur = 0;
#pragma unroll
      for (int w = 0; w < NW; ++w) {
        const int32_t* r = L.red + w * kRedStride;
        P = max(P, S + r[1]);
        S += r[0];
        viol += r[2];
        dur += r[3];
      }
    } else {
      const bool has = lane < NW;
      const int32_t* r = L.red + (has ? lane : 0) * kRedStride;
      S = has ? r[0] : 0;
      P = has ? r[1] : 0;
      viol = wave_sum(has ? r[2] : 0);
      dur = wave_sum(has ? r[3] : 0);
      wave_combine_ordered<(NT < 1024)>(lane, S, P);   // lanes >= NW hold (0, 0), which changes nothing
    }
  } else {
    viol += nlive - distinct;   // Eq. (6): live copies minus distinct start positions
    __syncthreads();
    if (passed) *passed = (uint32_t)L.red[kRedPass];
  }
  if (tid == kWave - 1) {
    moc_result res;
    res.peak = P;
    res.duration = dur;
    res.violations = viol;
    res.feasible = (viol == 0 && (int64_t)P <= g.budget) ? 1 : 0;
    out[b] = res;
  }
}

// ------------------------------------------------------------------ register-resident kernel
template <int CT>
struct NodeIn {
  int s[CT], e[CT];
  // The flag bytes, byte i = a of copy i.  C <= 2: one 16-bit value; C = 3: a 16-bit value and
  // the third byte in a2; C = 4: one 32-bit value.  The 16-bit values are never widened: they
  // go into the byte compares as they are, so that no conversion instruction sits between
  // the load and its first use (the compiler places such a conversion, and with it the wait
  // for the load, at the end of the iteration that issued the load).
  typename std::conditional<CT <= 3, uint16_t, uint32_t>::type a;
  uint16_t a2;
};

struct __attribute__((packed, aligned(4))) Int3 { int x, y, z; };

// Loads the C copies of one node.  s_row/e_row/a_row point at the candidate's row (uniform
// over the workgroup, so they live in scalar registers) and `off` = v*C is the lane's
// element offset, turned into 32-bit byte offsets so that the loads take the scalar base +
// 32-bit lane offset form.
template <typename V>
__device__ __forceinline__ V load_at(const void* base, uint32_t byte_off) {
  return *reinterpret_cast<const V*>(static_cast<const char*>(base) + byte_off);
}

template <int CT>
__device__ __forceinline__ void load_node(const int32_t* __restrict__ s_row, const int32_t* __restrict__ e_row,
                                          const uint8_t* __restrict__ a_row, uint32_t off, NodeIn<CT>& r) {
  const uint32_t boff = off * 4u;   // T <= 19455: no overflow
  if constexpr (CT == 1) {
    r.s[0] = load_at<int>(s_row, boff); r.e[0] = load_at<int>(e_row, boff); r.a = load_at<uint8_t>(a_row, off);   // widened to 16 bits by the load itself
  } else if constexpr (CT == 2) {
    const int2 sv = load_at<int2>(s_row, boff);
    const int2 ev = load_at<int2>(e_row, boff);
    r.s[0] = sv.x; r.s[1] = sv.y; r.e[0] = ev.x; r.e[1] = ev.y;
    r.a = load_at<uint16_t>(a_row, off);
  } else if constexpr (CT == 3) {
    const Int3 sv = load_at<Int3>(s_row, boff);
    const Int3 ev = load_at<Int3>(e_row, boff);
    r.s[0] = sv.x; r.s[1] = sv.y; r.s[2] = sv.z; r.e[0] = ev.x; r.e[1] = ev.y; r.e[2] = ev.z;
    r.a = load_at<uint16_t>(a_row, off);            // flags of copies 0 and 1 (any alignment)
    r.a2 = load_at<uint8_t>(a_row, off + 2);        // flag of copy 2, widened to 16 bits by the load itself
  } else {
    const int4 sv = load_at<int4>(s_row, boff);
    const int4 ev = load_at<int4>(e_row, boff);
    r.s[0] = sv.x; r.s[1] = sv.y; r.s[2] = sv.z; r.s[3] = sv.w;
    r.e[0] = ev.x; r.e[1] = ev.y; r.e[2] = ev.z; r.e[3] = ev.w;
    r.a = load_at<uint32_t>(a_row, off);
  }
}

// ------------------------------------------------------------------ LDS by byte address
// The dynamic LDS segment starts at address 0 (the kernels declare no static LDS, which the
// host verifies before the first launch) and the node records are its first array: the LDS
// address of a record is its word index times 4 and needs no base register.
typedef __attribute__((address_space(3))) uint32_t lds_u32;
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef __attribute__((address_space(3))) u32x2 lds_u32x2;
__device__ __forceinline__ uint32_t lds_read(uint32_t addr) { return *(const lds_u32*)(uintptr_t)addr; }
__device__ __forceinline__ uint2 lds_read2(uint32_t addr) {
  const u32x2 v = *(const lds_u32x2*)(uintptr_t)addr;
  return make_uint2(v.x, v.y);
}

// 4 * (low / high half of p): the LDS address of the record whose word index is packed in p.
// Written out so that the half is picked by the shift itself, and kept where it is used: the
// operand never changes, and the optimiser would otherwise hold every such address in a
// register of its own for the whole kernel.
__device__ __forceinline__ uint32_t addr_lo16(uint32_t p) {
  uint32_t r;
  asm volatile("v_lshlrev_b32_sdwa %0, %1, %2 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:WORD_0"
               : "=v"(r) : "s"(2u), "v"(p));
  return r;
}
__device__ __forceinline__ uint32_t addr_hi16(uint32_t p) {
  uint32_t r;
  asm volatile("v_lshlrev_b32_sdwa %0, %1, %2 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:WORD_1"
               : "=v"(r) : "s"(2u), "v"(p));
  return r;
}

typedef __attribute__((address_space(3))) uint16_t lds_u16;
__device__ __forceinline__ uint32_t lds_read_u16(uint32_t addr) { return *(const lds_u16*)(uintptr_t)addr; }
// 2 * (high half of p): the LDS address of a 16-bit entry
__device__ __forceinline__ uint32_t addr_hi16_half(uint32_t p) {
  uint32_t r;
  asm volatile("v_lshlrev_b32_sdwa %0, %1, %2 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:WORD_1"
               : "=v"(r) : "s"(1u), "v"(p));
  return r;
}

// The copies of a node as packed words s | e << 16 (MOC_DEAD if not live).
template <int CT>
struct Record {
  uint32_t w[CT];
};

// position t of the delta array -> word index t + 4 * (t / CH) (chunks of CH words, CH + 4
// apart), in the two instructions it takes
template <int CH>
__device__ __forceinline__ int delta_at(int t) {
  static_assert(CH == 16 || CH == 32, "chunks of 16 or 32 positions");
  int idx;
  if constexpr (CH == 32) asm("v_lshrrev_b32 %0, 5, %1\n\tv_lshl_add_u32 %0, %0, 2, %1" : "=&v"(idx) : "v"(t));
  else asm("v_lshrrev_b32 %0, 4, %1\n\tv_lshl_add_u32 %0, %0, 2, %1" : "=&v"(idx) : "v"(t));
  return idx;
}

// Lane masks.  A predicate over the wave is one 64-bit scalar: a vector compare writes it
// directly, the scalar unit combines and counts them, and nothing per lane is spent on
// booleans.  The compares that pick a 16-bit half or a byte of their operand are written out
// (sub-dword operand selects) since the compiler would first extract the field into a register.
// Lanes that are switched off read as 0.  Use in wave-uniform control flow only.
using lanemask = uint64_t;
#define MOC_MASK_CMP(name, text, breg)                                             \
  __device__ __forceinline__ lanemask name(uint32_t a, uint32_t b) {               \
    lanemask m;                                                                    \
    asm(text : "=s"(m) : "v"(a), breg(b));                                         \
    return m;                                                                      \
  }
MOC_MASK_CMP(u_le, "v_cmp_le_u32_e64 %0, %1, %2", "v")
MOC_MASK_CMP(i_gt, "v_cmp_gt_i32_e64 %0, %1, %2", "v")
// b the same in every lane (a scalar register)
MOC_MASK_CMP(u_lt_k, "v_cmp_lt_u32_e64 %0, %1, %2", "s")
#undef MOC_MASK_CMP
#define MOC_BYTE_CMP(name, sel)                                                                   \
  template <typename F>                                                                           \
  __device__ __forceinline__ lanemask name(F a, uint32_t b) {                                     \
    lanemask m;                                                                                   \
    asm("v_cmp_ne_u32_sdwa %0, %1, %2 src0_sel:" sel " src1_sel:DWORD" : "=s"(m) : "v"(a), "s"(b)); \
    return m;                                                                                     \
  }
MOC_BYTE_CMP(byte0_ne_k, "BYTE_0")
MOC_BYTE_CMP(byte1_ne_k, "BYTE_1")
MOC_BYTE_CMP(byte2_ne_k, "BYTE_2")
MOC_BYTE_CMP(byte3_ne_k, "BYTE_3")
#undef MOC_BYTE_CMP
template <typename F>
__device__ __forceinline__ lanemask byte_ne_k(F a, int i, uint32_t b) {
  return i == 0 ? byte0_ne_k(a, b) : i == 1 ? byte1_ne_k(a, b) : i == 2 ? byte2_ne_k(a, b) : byte3_ne_k(a, b);
}
// per lane: m ? yes : no
__device__ __forceinline__ uint32_t pick(lanemask m, uint32_t yes, uint32_t no) {
  uint32_t r;
  asm("v_cndmask_b32_e64 %0, %1, %2, %3" : "=v"(r) : "v"(no), "v"(yes), "s"(m));
  return r;
}
// per lane: m ? yes : 0
__device__ __forceinline__ uint32_t pick(lanemask m, uint32_t yes) {
  uint32_t r;
  asm("v_cndmask_b32_e64 %0, 0, %1, %2" : "=v"(r) : "v"(yes), "s"(m));
  return r;
}
__device__ __forceinline__ int count(lanemask m) { return __builtin_popcountll(m); }
// true in exactly the lanes of m: `if (lanes(m))` runs its body with those lanes switched on
__device__ __forceinline__ bool lanes(lanemask m) { return __builtin_amdgcn_inverse_ballot_w64(m); }
// number of lanes of m below the calling lane, plus base
__device__ __forceinline__ uint32_t rank_in(lanemask m, uint32_t base) {
  return __builtin_amdgcn_mbcnt_hi((uint32_t)(m >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)m, base));
}
// LDS[addr] = val in the lanes of m, without a branch: a branch would end the basic block, and
// 16-bit values that live across blocks are widened again where they are used.  LDS
// operations of a wave complete in order, so later reads see the write; the wave's count of
// outstanding LDS operations is only ever higher than the compiler assumes, never lower.
__device__ __forceinline__ void lds_write_lanes(lanemask m, uint32_t addr, uint32_t val) {
  lanemask saved;
  asm volatile("s_and_saveexec_b64 %0, %1\n\tds_write_b32 %2, %3\n\ts_mov_b64 exec, %0"
               : "=&s"(saved) : "s"(m), "v"(addr), "v"(val) : "memory", "scc");
}

// Eq. (5) for one copy of the consumer, packed as s | e << 16 in pv, against the CT copies of
// the provider in pu: adds to viol the number of lanes in which the copy is live and no copy of
// the provider has s_u + 1 <= s_v <= e_u (a dead copy has s = 0xFFFF and covers nothing).
// One block of instructions that ends in the count, so that three masks exist at a time
// however the surrounding code is scheduled: the masks of many edges in flight at once do not
// fit the scalar registers.
#define MOC_COVER_FIRST(U)                                                        \
  "v_cmp_lt_u32_sdwa %1, " U ", %5 src0_sel:WORD_0 src1_sel:WORD_0\n\t"           \
  "v_cmp_ge_u32_sdwa %2, " U ", %5 src0_sel:WORD_1 src1_sel:WORD_0\n\t"           \
  "s_and_b64 %1, %1, %2\n\t"
#define MOC_COVER_NEXT(U)                                                         \
  "v_cmp_lt_u32_sdwa %2, " U ", %5 src0_sel:WORD_0 src1_sel:WORD_0\n\t"           \
  "v_cmp_ge_u32_sdwa %3, " U ", %5 src0_sel:WORD_1 src1_sel:WORD_0\n\t"           \
  "s_and_b64 %2, %2, %3\n\t"                                                      \
  "s_or_b64 %1, %1, %2\n\t"
#define MOC_COVER_LAST                                                            \
  "v_cmp_ne_u32_sdwa %2, %5, %6 src0_sel:WORD_0 src1_sel:DWORD\n\t"               \
  "s_andn2_b64 %1, %2, %1\n\t"                                                    \
  "v_addc_co_u32 %0, vcc, 0, %0, %1"
// the same with "live" read off the word itself: a staged copy is live iff s <= e
#define MOC_COVER_LAST_SE                                                         \
  "v_cmp_le_u32_sdwa %2, %5, %5 src0_sel:WORD_0 src1_sel:WORD_1\n\t"              \
  "s_andn2_b64 %1, %2, %1\n\t"                                                    \
  "v_addc_co_u32 %0, vcc, 0, %0, %1"
#define MOC_COVER_REGS "+v"(viol), "=&s"(t1), "=&s"(t2), "=&s"(t3), "=&s"(c) : "v"(pv), "s"(dead)
template <int CT>
__device__ __forceinline__ void count_live_uncovered(int& viol, const Record<CT>& pu, uint32_t pv) {
  lanemask t1, t2, t3;
  int c;
  const uint32_t dead = MOC_DEAD;
  if constexpr (CT == 1)
    asm(MOC_COVER_FIRST("%7") MOC_COVER_LAST : MOC_COVER_REGS, "v"(pu.w[0]) : "scc", "vcc");
  else if constexpr (CT == 2)
    asm(MOC_COVER_FIRST("%7") MOC_COVER_NEXT("%8") MOC_COVER_LAST : MOC_COVER_REGS, "v"(pu.w[0]), "v"(pu.w[1]) : "scc", "vcc");
  else if constexpr (CT == 3)
    asm(MOC_COVER_FIRST("%7") MOC_COVER_NEXT("%8") MOC_COVER_NEXT("%9") MOC_COVER_LAST_SE
        : MOC_COVER_REGS, "v"(pu.w[0]), "v"(pu.w[1]), "v"(pu.w[2]) : "scc", "vcc");
  else
    asm(MOC_COVER_FIRST("%7") MOC_COVER_NEXT("%8") MOC_COVER_NEXT("%9") MOC_COVER_NEXT("%10") MOC_COVER_LAST_SE
        : MOC_COVER_REGS, "v"(pu.w[0]), "v"(pu.w[1]), "v"(pu.w[2]), "v"(pu.w[3]) : "scc", "vcc");
}
#undef MOC_COVER_FIRST
#undef MOC_COVER_NEXT
#undef MOC_COVER_LAST
#undef MOC_COVER_LAST_SE
#undef MOC_COVER_REGS

// C <= 2: the records of the two nodes of an edge held in a register as pair = u*C | v*C << 16
// (word indices of the records)
template <int CT>
__device__ __forceinline__ void fetch_edge(uint32_t pair, Record<CT>& pv, Record<CT>& pu) {
  if constexpr (CT == 1) {
    pv.w[0] = lds_read(addr_hi16(pair));
    pu.w[0] = lds_read(addr_lo16(pair));
  } else {
    const uint2 rv = lds_read2(addr_hi16(pair)), ru = lds_read2(addr_lo16(pair));
    pv.w[0] = rv.x; pv.w[1] = rv.y; pu.w[0] = ru.x; pu.w[1] = ru.y;
  }
}

// Eq. (5), C >= 3, first pass over an edge (u, v): the first copy of u (pu, a record word) and
// the 16-bit entry of v as a consumer (pv) are fetched.  The instance is settled, with no
// violation, where the first copy of u covers the start of the first copy of v and v has no
// other live copy.  All other edges are returned and go to the wave's queue for the full test:
// the first copy of v not covered by the first copy of u (another copy of u may cover it, or
// it is a violation, or v's first copy is not live at all), or a consumer with other live
// copies, each of which needs an input.  Such a consumer carries bit 15 on top of the start in
// its entry (positions stay below 2^15): the start then lies above every end, so the test
// fails by itself and costs nothing extra.  Whether u has other copies does not matter where
// its first copy covers.
__device__ __forceinline__ lanemask check_first_copies(int& viol, uint32_t pu, uint32_t pv) {
  lanemask t1, t2, more;
  asm("v_cmp_lt_u32_sdwa %0, %3, %4 src0_sel:WORD_0 src1_sel:WORD_0\n\t"
      "v_cmp_ge_u32_sdwa %1, %3, %4 src0_sel:WORD_1 src1_sel:WORD_0\n\t"
      "s_and_b64 %0, %0, %1\n\t"   // covered by the first copy of u
      "s_andn2_b64 %2, exec, %0"
      : "=&s"(t1), "=&s"(t2), "=&s"(more)
      : "v"(pu), "v"(pv)
      : "scc");
  return more;
}

// Eq. (5), C >= 3, second pass: the full test (every live copy of v against every copy of u)
// for the `count` edges in the wave's queue, 64 at a time.
template <int CT>
__device__ __forceinline__ void drain_queue(int& viol, const Lds& L, const uint32_t* queue, int count, int lane,
                                            uint32_t dummy_pair, uint32_t cons_base) {
  constexpr int RS = CT == 3 ? 2 : 4;
  for (int base = 0; base < count; base += kWave) {
    const int idx = base + lane;   // inside the queue: its capacity is a multiple of 64
    const uint32_t pair = pick(u_lt_k((uint32_t)idx, (uint32_t)count), queue[idx], dummy_pair);
    const uint32_t v = (pair >> 16) - cons_base, u = pair & 0xFFFFu;
    Record<CT> pv, pu;
    pv.w[0] = L.packed[v];
    pu.w[0] = L.packed[u];
    if constexpr (CT == 3) {
      const uint2 rv = *reinterpret_cast<const uint2*>(L.rest + v * RS);
      const uint2 ru = *reinterpret_cast<const uint2*>(L.rest + u * RS);
      pv.w[1] = rv.x; pv.w[2] = rv.y; pu.w[1] = ru.x; pu.w[2] = ru.y;
    } else {
      const uint4 rv = *reinterpret_cast<const uint4*>(L.rest + v * RS);
      const uint4 ru = *reinterpret_cast<const uint4*>(L.rest + u * RS);
      pv.w[1] = rv.x; pv.w[2] = rv.y; pv.w[3] = rv.z; pu.w[1] = ru.x; pu.w[2] = ru.y; pu.w[3] = ru.z;
    }
#pragma unroll
    for (int i = 0; i < CT; ++i) count_live_uncovered<CT>(viol, pu, pv.w[i]);
  }
}

template <int NT, int CT, int ITERS>
__global__ __launch_bounds__(NT) void eval_batch_kernel(GraphView g, int64_t B, const int32_t* __restrict__ starts,
                                                        const int32_t* __restrict__ ends,
                                                        const uint8_t* __restrict__ active,
                                                        moc_result* __restrict__ out, LdsLayout lay,
                                                        uint32_t* __restrict__ ticket, int groups) {
  constexpr int EPT = kEdgesPerNode * ITERS;
  constexpr bool kSplit = CT >= 3;          // first copies and other copies in separate arrays
  constexpr int NS = kSplit ? 1 : CT;       // words per node in the first array
  constexpr int RS = CT == 3 ? 2 : 4;       // kSplit: words per node in the second
  constexpr int kEarly = ITERS * 3 / 5;     // node slots re-requested during phase 1
  constexpr int CH = chunk_positions(NT);   // delta positions per chunk
  extern __shared__ uint32_t lds_raw[];
  const Lds L = carve(lds_raw, lay);
  const int tid = threadIdx.x;
  const int wave = __builtin_amdgcn_readfirstlane(tid / kWave);   // the same in every lane: say so
  const int T = g.T, n = g.n;
  const uint32_t group = groups ? blockIdx.x % (uint32_t)groups : 0u;
  uint32_t* const counter = ticket + (size_t)group * kTicketStride;
  uint32_t first_draw = 0;   // thread 0: the first two candidates of this workgroup, asked for before anything else
  if (tid == 0 && groups != 0) first_draw = atomicAdd(counter, 2u);
  uint32_t* const queue = L.queue + wave * lay.qcap;   // kSplit: this wave's edges set aside
  const uint32_t queue_addr = 4u * (uint32_t)(lay.queue_off + wave * lay.qcap);   // its LDS address
  // kSplit: the high half of an edge register is the index of the consumer's 16-bit entry, counted
  // in 16-bit units from LDS address 0 (n + 2 * cons_off stays far below 2^16 for any T accepted)
  const uint32_t cons_base = kSplit ? 2u * (uint32_t)lay.cons_off : 0u;
  // the pair of a node that is never live with itself: what idle lanes of the second pass look at
  const uint32_t dummy_pair = kSplit ? (uint32_t)(n + 2) * 0x10001u + (cons_base << 16) : (uint32_t)(n * NS) * 0x10001u;

  for (int i = tid; i < lay.delta_len; i += NT) L.delta[i] = 0;
  for (int i = tid; i < lay.occ_words; i += NT) L.occ[i] = 0;
  for (int i = tid; i < lay.packed_len; i += NT) L.packed[i] = MOC_DEAD;   // the record arrays and the consumers' entries, incl. the dummy nodes
  if constexpr (kSplit) {
    __syncthreads();
    if (tid == 0) {   // the padding of the edge list is the edge (n + 1, n): start 1 inside [0, 0x7FFF]
      L.packed[n] = 1u;
      L.cons[n] = 1;
      L.packed[n + 1] = 0x7FFF0000u;
    }
  }

  // what a lane owns never changes: its edges stay in registers
  uint32_t edge[EPT];
#pragma unroll
  for (int j = 0; j < EPT; ++j) {
    const int e = j * NT + tid;
    edge[j] = g.edge_pair[e] + (cons_base << 16);   // the list is padded with dummy edges to EPT * NT entries
  }
  NodeIn<CT> in[ITERS];
  // m_v, w_v of the lane's nodes: the same for every candidate, read once
  int2 sd[ITERS];
  auto request_size_dur = [&]() {
#pragma unroll
    for (int it = 0; it < ITERS; ++it) {
      int v = min(it * NT + tid, n - 1);       // lanes past the last node re-read it; their results are masked
      asm volatile("" : "+v"(v));
      sd[it] = load_at<int2>(g.size_dur, (uint32_t)v * 8u);
    }
  };
  // Loads of node slot `it` of the candidate at `row`.  Issued unconditionally (lanes past the
  // last node re-read it) so that the count of loads in flight is the same on every path.
  auto request = [&](int it, int64_t row) {
    int v = min(it * NT + tid, n - 1);
    asm volatile("" : "+v"(v));                // keep the per-slot offsets out of registers
    load_node<CT>(starts + row, ends + row, active + row, (uint32_t)v * CT, in[it]);
  };
  // Eq. (4), (6): one live copy [s, e] of a node of size m_v into the delta array (+m_v at s,
  // -m_v after e) and the bitmap of start positions
  auto scatter = [&](int s, int e, int size) {
    atomicAdd(&L.delta[delta_at<CH>(s)], size);
    atomicSub(&L.delta[delta_at<CH>(e + 1)], size);
    atomicOr(&L.occ[s >> 5], 1u << (s & 31));
  };
  request_size_dur();
  // Candidates are handed out dynamically, so that compute units that hold fewer or faster
  // workgroups take more of the batch, and a workgroup that starts late finds nothing left
  // and goes.  They are dealt into `groups` interleaved sequences, group r = {r + groups * t};
  // a workgroup belongs to group blockIdx.x % groups and draws t from the group's counter
  // (many counters: one would be drawn from faster than a single address serves).  It starts
  // with two draws; then the draw for the candidate after next is made at the top of an
  // iteration and collected at its end: its latency never shows, and the next candidate is
  // known early enough to prefetch it.  A workgroup thus holds two candidates beyond the one
  // it works on, which is too many when the batch has only a few per workgroup: then
  // (groups == 0) the split is fixed, workgroup w takes w, w + grid, ...  32 bits are enough
  // for t: the host launches at most 2^31 candidates at a time.
  const auto dealt = [&](uint32_t t) {
    return groups ? (int64_t)group + (int64_t)groups * t : (int64_t)blockIdx.x + (int64_t)gridDim.x * t;
  };
  if (groups == 0) {
#pragma unroll
    for (int it = 0; it < ITERS; ++it) request(it, (int64_t)blockIdx.x * T);   // the grid is not larger than the batch
  }
  if (tid == 0) L.red[kRedPass] = (int32_t)first_draw;
  __syncthreads();
  uint32_t next = (uint32_t)__builtin_amdgcn_readfirstlane(L.red[kRedPass]);
  int64_t b = dealt(next);
  ++next;
  if (groups != 0 && b < B) {
#pragma unroll
    for (int it = 0; it < ITERS; ++it) request(it, b * T);
  }
  uint32_t drawn = 0;   // thread 0

  // Workgroups that share a compute unit do not run equally fast: the issue logic prefers the
  // oldest waves, and with four waves or fewer per workgroup many workgroups share a unit.  Each
  // then takes the four issue priorities in turn, one candidate at a time, out of step with its
  // neighbours, so that over a few candidates all get the same share and a batch that is split
  // statically (a short one) does not wait for the workgroups that were dispatched last.
  [[maybe_unused]] int turn = (int)(blockIdx.x / 256u);
  while (b < B) {
    // Large workgroups (C >= 3 graphs): lane predicates and addresses derived from the thread
    // index are formed where they are used.  Kept across candidates they take scalar registers
    // that the masks of phase 1 need, and are spilled to vector lanes (two instructions to fetch
    // one back, against one to form it again): n = 5000 63.6 -> 64.3 % of HBM peak.  The small
    // kernels lose by it (n = 442: 50 -> 42 %) and keep them.
    int t_ = tid;
    if constexpr (NT >= 1024) asm volatile("" : "+v"(t_));
    const int lane_ = t_ & (kWave - 1);
    if constexpr (NT <= 256) {
      switch (turn++ & 3) {
        case 0: __builtin_amdgcn_s_setprio(0); break;
        case 1: __builtin_amdgcn_s_setprio(1); break;
        case 2: __builtin_amdgcn_s_setprio(2); break;
        default: __builtin_amdgcn_s_setprio(3); break;
      }
    }
    int viol = wave == 0 ? n : 0;   // per wave (the same in every lane_, counted on lane_ masks); see phase 1
    int dur = 0;               // per lane_
    if (t_ == 0) drawn = groups ? atomicAdd(counter, 1u) : next + 1;
    // The workgroup's next candidate; the last one re-reads itself so that the loads below
    // need no condition.  Slot `it` is requested as soon as phase 1 has consumed the
    // registers of slot `it` (the first kEarly slots) or between the steps of phase 2 (the
    // rest): HBM streams through both phases and no wave queues all its loads at once.
    const int64_t b_next = dealt(next);
    const int64_t next_row = (b_next < B ? b_next : b) * T;

    // ---------------- phase 1: per node, copies in registers
#pragma unroll
    for (int it = 0; it < ITERS; ++it) {
      int v = it * NT + t_;
      asm volatile("" : "+v"(v));               // as for the edges: keep derived addresses out of registers
      if (it * NT + wave * kWave < n) {   // else: whole wave past the last node
        const NodeIn<CT>& r = in[it];
        // Eq. (2), (7), (8), (3) on lane_ masks; Eq. (1) per lane_
        const lanemask isn = u_lt_k((uint32_t)v, (uint32_t)n);
        lanemask act[CT], live[CT];
        Record<CT> rec;
#pragma unroll
        for (int i = 0; i < CT; ++i) {
          if constexpr (CT == 3) act[i] = (i < 2 ? byte_ne_k(r.a, i, 0u) : byte_ne_k(r.a2, 0, 0u)) & isn;
          else act[i] = byte_ne_k(r.a, i, 0u) & isn;
          const lanemask well = u_le((uint32_t)r.s[i], (uint32_t)r.e[i]) & u_lt_k((uint32_t)r.e[i], (uint32_t)T);
          live[i] = act[i] & well;
          // an active copy is either ill-formed, one violation of Eq. (2)/(8), or live, one
          // more start for Eq. (6) (the distinct start positions are taken off at the end):
          // both end up in the same sum.  The first copy adds one in every case, for when
          // it is not active Eq. (7) is violated: that makes n, which the sum starts from.
          if (i > 0) viol += count(act[i]);
          dur += (int)pick(act[i], (uint32_t)sd[it].y);
          rec.w[i] = pick(live[i], (uint32_t)r.s[i] | ((uint32_t)r.e[i] << 16), MOC_DEAD);
        }
#pragma unroll
        for (int i = 0; i + 1 < CT; ++i) {   // Eq. (3): against the next live copy
          lanemask seen = 0, late = 0;
#pragma unroll
          for (int j = i + 1; j < CT; ++j) {
            late |= ~seen & live[j] & i_gt((uint32_t)r.e[i], (uint32_t)r.s[j]);
            seen |= live[j];
          }
          viol += count(live[i] & late);
        }
        lanemask others = 0;   // lanes whose node has a live copy besides the first
#pragma unroll
        for (int i = 1; i < CT; ++i) others |= live[i];
        if (lanes(isn)) {
          if constexpr (CT == 1) {
            L.packed[v] = rec.w[0];
          } else if constexpr (CT == 2) {
            *reinterpret_cast<uint2*>(L.packed + v * 2) = make_uint2(rec.w[0], rec.w[1]);
          } else {
            // bit 15: the node has other live copies, its in-edges take the full test (see check_first_copies)
            L.packed[v] = rec.w[0];
            L.cons[v] = (uint16_t)(rec.w[0] | pick(others, 0x00008000u));
            if constexpr (CT == 3) *reinterpret_cast<uint2*>(L.rest + v * RS) = make_uint2(rec.w[1], rec.w[2]);
            else *reinterpret_cast<uint4*>(L.rest + v * RS) = make_uint4(rec.w[1], rec.w[2], rec.w[3], MOC_DEAD);
          }
        }
        if (lanes(live[0])) scatter(r.s[0], r.e[0], sd[it].x);
        // The other copies are rarely live: in round k every lane_ brings the k-th of its
        // live ones, so that a wave runs as many rounds as its busiest node has such copies
        // rather than one per copy.
        lanemask left[CT];
#pragma unroll
        for (int i = 1; i < CT; ++i) left[i] = live[i];
#pragma unroll
        for (int round = 1; round < CT; ++round) {
          if (others == 0) break;
          int sx = r.s[CT - 1], ex = r.e[CT - 1];
#pragma unroll
          for (int i = CT - 2; i >= round; --i) {   // the first of the lane_'s copies that are left
            sx = (int)pick(left[i], (uint32_t)r.s[i], (uint32_t)sx);
            ex = (int)pick(left[i], (uint32_t)r.e[i], (uint32_t)ex);
          }
          if (lanes(others)) scatter(sx, ex, sd[it].x);
          lanemask before = 0;
          others = 0;
#pragma unroll
          for (int i = round; i < CT; ++i) {
            const lanemask taken = left[i] & ~before;
            before |= left[i];
            left[i] &= ~taken;
            others |= left[i];
          }
        }
      }
      if (it < kEarly) request(it, next_row);
    }
    __syncthreads();

    // ---------------- phase 2 (LDS only), with the next candidate's loads issued in slices
    if (kEarly < ITERS) request(kEarly, next_row);
    __builtin_amdgcn_sched_barrier(0);
    // (a) one chunk of CH delta positions per thread
    int S = 0, P = 0;
    if (wave * kWave < lay.n_chunks) {
      if (t_ < lay.n_chunks) {
        int4* d = reinterpret_cast<int4*>(L.delta + t_ * (CH + 4));
#pragma unroll
        for (int h = 0; h < CH / 8; ++h) {   // 8 positions at a time keeps the register count down
          const int4 x0 = d[2 * h], x1 = d[2 * h + 1];
          d[2 * h] = make_int4(0, 0, 0, 0);
          d[2 * h + 1] = make_int4(0, 0, 0, 0);
          S += x0.x; P = max(P, S);
          S += x0.y; P = max(P, S);
          S += x0.z; P = max(P, S);
          S += x0.w; P = max(P, S);
          S += x1.x; P = max(P, S);
          S += x1.y; P = max(P, S);
          S += x1.z; P = max(P, S);
          S += x1.w; P = max(P, S);
          __builtin_amdgcn_sched_barrier(0);
        }
      }
      wave_combine_ordered<(NT < 1024)>(lane_, S, P);
    }
    const int distinct = count_distinct_starts<NT>(L, lay, t_);
    // (c) edges, three per slice of the prefetch; their violations are counted per lane_
    int queued = 0, eviol = 0;
#pragma unroll
    for (int it = 0; it < ITERS; ++it) {
      __builtin_amdgcn_sched_barrier(0);
      if (it > 0 && kEarly + it < ITERS) request(kEarly + it, next_row);
      __builtin_amdgcn_sched_barrier(0);
      if (it >= lay.edge_slices) continue;   // the edge list fills the first slices; the others hold padding only
      // the records of the slice's edges are asked for together and looked at afterwards: one
      // LDS latency per slice, not one per edge
      if constexpr (!kSplit) {
        auto edges_of_slice = [&](auto count) {
          constexpr int N = decltype(count)::value;
          Record<CT> pv[N], pu[N];
#pragma unroll
          for (int j = 0; j < N; ++j) fetch_edge<CT>(edge[it * kEdgesPerNode + j], pv[j], pu[j]);
          __builtin_amdgcn_sched_barrier(0);   // all reads of the slice before its first test
#pragma unroll
          for (int j = 0; j < N; ++j) {
#pragma unroll
            for (int i = 0; i < CT; ++i) count_live_uncovered<CT>(eviol, pu[j], pv[j].w[i]);
          }
        };
        // The lane_'s last slice may hold edges in its first one or two entries only (padding in
        // every lane_ beyond): blocks of their own, each one straight run of reads, then tests.
        const int here = lay.edge_slots - it * kEdgesPerNode;   // > 0
        if (it == ITERS - 1 && here == 1) edges_of_slice(std::integral_constant<int, 1>{});
        else if (it == ITERS - 1 && here == 2) edges_of_slice(std::integral_constant<int, 2>{});
        else edges_of_slice(std::integral_constant<int, kEdgesPerNode>{});
      } else {
        if (queued > lay.qcap - kEdgesPerNode * kWave) {   // the slice might not fit: work the queue off first
          drain_queue<CT>(eviol, L, queue, queued, lane_, dummy_pair, cons_base);
          queued = 0;
        }
        uint32_t pv[kEdgesPerNode], pu[kEdgesPerNode];
#pragma unroll
        for (int j = 0; j < kEdgesPerNode; ++j) {
          pv[j] = lds_read_u16(addr_hi16_half(edge[it * kEdgesPerNode + j]));
          pu[j] = lds_read(addr_lo16(edge[it * kEdgesPerNode + j]));
        }
#pragma unroll
        for (int j = 0; j < kEdgesPerNode; ++j) {
          const lanemask more = check_first_copies(eviol, pu[j], pv[j]);
          const uint32_t tail = queue_addr + 4u * (uint32_t)queued;   // the same in every lane_: scalar arithmetic
          lds_write_lanes(more, tail + 4u * rank_in(more, 0u), edge[it * kEdgesPerNode + j]);
          queued += count(more);
        }
      }
    }
    if constexpr (kSplit) drain_queue<CT>(eviol, L, queue, queued, lane_, dummy_pair, cons_base);
    uint32_t after_next;
    finish<NT, true>(L, g, t_, lane_, wave, S, P, viol, 0, distinct - eviol, dur, out, b, drawn, &after_next);
    b = b_next;
    next = (uint32_t)__builtin_amdgcn_readfirstlane(after_next);
  }
  // The last workgroup to leave puts the counters back to zero for the next launch.  No fence
  // is needed: a workgroup has received the results of all its draws before it signs off, and
  // all accesses to the counters are atomic operations, which meet in one place.
  if (tid == 0 && groups != 0) {
    uint32_t* const left = ticket + (size_t)groups * kTicketStride;
    if (atomicAdd(left, 1u) == gridDim.x - 1) {
      for (int r = 0; r <= groups; ++r) atomicExch(&ticket[(size_t)r * kTicketStride], 0u);
    }
  }
}

// ------------------------------------------------------------------ general kernel: any C, any n, any alignment
template <int NT>
__global__ __launch_bounds__(NT) void eval_batch_general_kernel(GraphView g, int64_t B,
                                                                const int32_t* __restrict__ starts,
                                                                const int32_t* __restrict__ ends,
                                                                const uint8_t* __restrict__ active,
                                                                moc_result* __restrict__ out, LdsLayout lay,
                                                                uint32_t* __restrict__ /*ticket*/, int /*groups*/) {
  extern __shared__ uint32_t lds_raw[];
  const Lds L = carve(lds_raw, lay);
  const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
  const int T = g.T, n = g.n, C = g.C;

  for (int i = tid; i < lay.delta_len; i += NT) L.delta[i] = 0;
  for (int i = tid; i < lay.occ_words; i += NT) L.occ[i] = 0;
  __syncthreads();

  for (int64_t b = blockIdx.x; b < B; b += gridDim.x) {
    const int64_t row = b * T;
    int viol = 0, nlive = 0, dur = 0;
    // phase 1: per node, copies read one by one
    for (int v = tid; v < n; v += NT) {
      const int2 sd = g.size_dur[v];
      int prev_end = -1;   // end of the latest live copy seen so far (Eq. (3))
      for (int i = 0; i < C; ++i) {
        const int64_t at = row + (int64_t)v * C + i;
        const int s = starts[at], e = ends[at];
        const bool act = active[at] != 0;
        const bool well = (uint32_t)s <= (uint32_t)e && (uint32_t)e < (uint32_t)T;
        const bool live = act && well;
        viol += (act && !well) ? 1 : 0;
        if (i == 0) viol += act ? 0 : 1;
        dur += act ? sd.y : 0;
        L.packed[v * C + i] = live ? ((uint32_t)s | ((uint32_t)e << 16)) : MOC_DEAD;
        if (live) {
          nlive += 1;
          viol += prev_end > s ? 1 : 0;
          prev_end = e;
          atomicAdd(&L.delta[s], sd.x);
          atomicAdd(&L.delta[e + 1], -sd.x);
          atomicOr(&L.occ[s >> 5], 1u << (s & 31));
        }
      }
    }
    __syncthreads();

    // phase 2a: contiguous odd-length chunk per thread
    int S = 0, P = 0;
    {
      int32_t* d = L.delta + tid * lay.chunk;
#pragma unroll 5
      for (int j = 0; j < lay.chunk; ++j) {
        const int x = d[j];
        d[j] = 0;
        S += x;
        P = max(P, S);
      }
    }
    wave_combine_ordered<(NT < 1024)>(lane, S, P);
    const int distinct = count_distinct_starts<NT>(L, lay, tid);
    // Eq. (5): one lane per edge, every live copy of the consumer; edge_pair_c = u*C | v*C << 16
    for (int e = tid; e < g.m; e += NT) {
      const uint32_t pair = g.edge_pair_c[e];
      const int kd = (int)(pair >> 16), ub = (int)(pair & 0xFFFFu);
      for (int i = 0; i < C; ++i) {
        const uint32_t pv = L.packed[kd + i];
        const uint32_t x = pv & 0xFFFFu, xs = x << 16;
        bool cov = false;
        for (int q = 0; q < C; ++q) cov = cov || covers(L.packed[ub + q], x, xs);
        viol += (is_live(pv) && !cov) ? 1 : 0;
      }
    }
    finish<NT>(L, g, tid, lane, wave, S, P, viol, nlive, distinct, dur, out, b);
  }
}

// ------------------------------------------------------------------ host side
// fixed: the set of work counters to use instead of the graph handle's set for the stream.
// prepare_only: do everything a launch does on the host except the launch itself (first-use
// set-up of the kernel and its occupancy, which the handle then remembers).
struct LaunchOpts {
  uint32_t* fixed;
  bool prepare_only;
};

template <typename K>
int launch_kernel(K kern, int nt, const moc_graph* g, const LdsLayout& lay, int64_t B, const int32_t* starts,
                  const int32_t* ends, const uint8_t* active, moc_result* out, hipStream_t stream,
                  const LaunchOpts& src) {
  if (lay.bytes > g->max_lds) return MOC_EOVERFLOW;
  // Nothing may be placed before the dynamic LDS segment: the kernels address the node
  // records from LDS address 0.
  int per_cu = 0;
  const int rc = moc_kernel_occupancy(g, reinterpret_cast<const void*>(kern), nt, lay.bytes, true, &per_cu);
  if (rc != MOC_OK) return rc;
  if (src.prepare_only) return MOC_OK;
  const int64_t resident = (int64_t)per_cu * g->num_cu;
  const unsigned grid = (unsigned)(B < resident ? B : resident);
  // About 16 workgroups share a counter.  A batch of fewer than 8 candidates per workgroup is
  // split statically (groups = 0), and so is a launch for which no set of counters is free.
  int groups = grid / 16 < 1 ? 1 : grid / 16 > kTicketGroups ? kTicketGroups : (int)(grid / 16);
  if (B < (int64_t)8 * grid) groups = 0;
  uint32_t* ticket = nullptr;
  if (groups != 0) {
    ticket = src.fixed ? src.fixed : moc_ticket_set(g, stream);
    if (!ticket) groups = 0;
  }
  hipLaunchKernelGGL(kern, dim3(grid), dim3(nt), lay.bytes, stream, g->view, B, starts, ends, active, out, lay,
                     ticket, groups);
  MOC_HIP(hipGetLastError());
  return MOC_OK;
}

template <int NT, int CT, int IT = kMaxIters>
int launch_iters(int iters, const moc_graph* g, const LdsLayout& lay, int64_t B, const int32_t* s, const int32_t* e,
                 const uint8_t* a, moc_result* out, hipStream_t st, const LaunchOpts& src) {
  if constexpr (IT == 0) {
    return MOC_EINVAL;
  } else {
    if (iters == IT) return launch_kernel(eval_batch_kernel<NT, CT, IT>, NT, g, lay, B, s, e, a, out, st, src);
    return launch_iters<NT, CT, IT - 1>(iters, g, lay, B, s, e, a, out, st, src);
  }
}

// Node slots per lane the register-resident kernel needs with nt threads: enough for the
// nodes (one per slot) and for the edges (kEdgesPerNode per slot).
int slots_per_lane(int n, int m, int nt) {
  const int by_nodes = (n + nt - 1) / nt, by_edges = (m + kEdgesPerNode * nt - 1) / (kEdgesPerNode * nt);
  return by_nodes > by_edges ? by_nodes : by_edges;
}

// Workgroup size: the smallest that leaves at most 5 node slots per lane and at most one delta
// chunk per thread (one wave per
// candidate for small graphs, up to a full 1024-thread workgroup per compute unit).
int block_threads(int n, int m, int C) {
  for (int nt = 64; nt < 1024; nt *= 2)
    if (slots_per_lane(n, m, nt) <= 5 && (n * C + chunk_positions(nt)) / chunk_positions(nt) <= nt) return nt;
  return 1024;
}

// The register-resident kernel applies when C <= 4, a lane's nodes and edges fit its
// registers, and every thread has at most one delta chunk.
bool fast_shape(int n, int m, int C, int nt) {
  return C <= 4 && n * C >= 4 && slots_per_lane(n, m, nt) <= kMaxIters && (n * C + chunk_positions(nt)) / chunk_positions(nt) <= nt &&
         (n + 3) * moc_node_stride(C) <= 0xFFFF;
}

template <int NT>
int launch_nt(const moc_graph* g, int64_t B, const int32_t* s, const int32_t* e, const uint8_t* a, moc_result* out,
              hipStream_t st, bool aligned, const LaunchOpts& src) {
  const int n = g->view.n, m = g->view.m, C = g->view.C;
  if (aligned && fast_shape(n, m, C, NT)) {
    const LdsLayout lay = fast_layout(n, m, C, NT, g->max_lds);
    const int iters = slots_per_lane(n, m, NT);
    switch (C) {
      case 1: return launch_iters<NT, 1>(iters, g, lay, B, s, e, a, out, st, src);
      case 2: return launch_iters<NT, 2>(iters, g, lay, B, s, e, a, out, st, src);
      case 3: return launch_iters<NT, 3>(iters, g, lay, B, s, e, a, out, st, src);
      default: return launch_iters<NT, 4>(iters, g, lay, B, s, e, a, out, st, src);
    }
  }
  return launch_kernel(eval_batch_general_kernel<NT>, NT, g, general_layout(n, C, NT), B, s, e, a, out, st, src);
}

}  // namespace

int moc_node_stride(int C) { return C == 2 ? 2 : 1; }

bool moc_eval_shape(int n, int m, int C, int* nt, int* edges_per_lane, int* edges_per_lane_used) {
  *nt = block_threads(n, m, C);
  *edges_per_lane = kEdgesPerNode * slots_per_lane(n, m, *nt);
  *edges_per_lane_used = (m + *nt - 1) / *nt;   // = LdsLayout::edge_slots
  return fast_shape(n, m, C, *nt);
}

int moc_eval_lds_bytes(int n, int m, int C, int max_lds) {
  const int nt = block_threads(n, m, C);
  const int general = general_layout(n, C, nt).bytes;
  if (!fast_shape(n, m, C, nt)) return general;
  const int fast = fast_layout(n, m, C, nt, max_lds).bytes;   // misaligned candidate arrays fall back to the general kernel
  return fast > general ? fast : general;
}

namespace {

// One launch per 2^31 candidates of the kernel this graph and these arrays take.
int dispatch(const moc_graph* g, int64_t B, const int32_t* starts, const int32_t* ends, const uint8_t* active,
             moc_result* out, hipStream_t st, bool aligned, const LaunchOpts& src) {
  const int nt = block_threads(g->view.n, g->view.m, g->view.C);
  // The kernels count candidates handed out in 32 bits: longer batches go in several launches.
  const int64_t T = g->view.T;
  for (int64_t at = 0; at < B; at += kMaxLaunch) {
    const int64_t count = B - at < kMaxLaunch ? B - at : kMaxLaunch;
    const int32_t* s = starts + at * T;
    const int32_t* e = ends + at * T;
    const uint8_t* a = active + at * T;
    int rc;
    switch (nt) {
      case 64: rc = launch_nt<64>(g, count, s, e, a, out + at, st, aligned, src); break;
      case 128: rc = launch_nt<128>(g, count, s, e, a, out + at, st, aligned, src); break;
      case 256: rc = launch_nt<256>(g, count, s, e, a, out + at, st, aligned, src); break;
      case 512: rc = launch_nt<512>(g, count, s, e, a, out + at, st, aligned, src); break;
      default: rc = launch_nt<1024>(g, count, s, e, a, out + at, st, aligned, src); break;
    }
    if (rc != MOC_OK) return rc;
  }
  return MOC_OK;
}

int check_arguments(const moc_graph* g, int64_t B, const int32_t* starts, const int32_t* ends,
                    const uint8_t* active, moc_result* out) {
  if (!g || B < 0) return MOC_EINVAL;
  if (B == 0) return MOC_OK;
  if (!starts || !ends || !active || !out) return MOC_EINVAL;
  if (((uintptr_t)starts | (uintptr_t)ends) & 3 || ((uintptr_t)out & 7)) return MOC_EINVAL;
  int dev = -1;
  MOC_HIP(hipGetDevice(&dev));
  if (dev != g->device) return MOC_EDEVICE;
  return MOC_OK;
}

// The register-resident kernel reads the C copies of a node as one vector: rows must be
// aligned to the vector (they are when the base pointers are, since a row is n vectors).
bool vector_aligned(int C, const int32_t* starts, const int32_t* ends, const uint8_t* active) {
  const uintptr_t se = (uintptr_t)starts | (uintptr_t)ends;
  if (C == 2) return (se & 7) == 0 && ((uintptr_t)active & 1) == 0;
  if (C == 4) return (se & 15) == 0 && ((uintptr_t)active & 3) == 0;
  return true;
}

}  // namespace

int moc_eval_prepare(const moc_graph* g) {
  const LaunchOpts prepare{nullptr, true};
  for (const bool aligned : {true, false}) {
    const int rc = dispatch(g, 1, nullptr, nullptr, nullptr, nullptr, nullptr, aligned, prepare);
    if (rc != MOC_OK) return rc;
  }
  return MOC_OK;
}

extern "C" int moc_eval_batch(const moc_graph* g, int64_t B, const int32_t* starts, const int32_t* ends,
                              const uint8_t* active, moc_result* out, void* hip_stream) {
  const int rc = check_arguments(g, B, starts, ends, active, out);
  if (rc != MOC_OK || B == 0) return rc;
  return dispatch(g, B, starts, ends, active, out, static_cast<hipStream_t>(hip_stream),
                  vector_aligned(g->view.C, starts, ends, active), LaunchOpts{nullptr, false});
}

// ------------------------------------------------------------------ moc_eval_batch_noalloc
// The same evaluation with its work counters in the library's own device image instead of
// memory allocated at upload: one set, kTicketSlotWords words, per GPU.  Host code never uses
// the array's name as an address: the address on each device is asked for once, with that
// device current (moc_eval_static_setup, called by moc_graph_upload), and kept.
static __device__ __align__(256) uint32_t scratch[kTicketSlotWords];

namespace {

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mu;
uint32_t* g_scratch_ptr[kMaxDevices];   // per device: where `scratch` lives there; nullptr = not asked yet

__global__ void clear_counters_kernel(uint32_t* counters) {
  for (int i = threadIdx.x; i < kTicketSlotWords; i += blockDim.x) counters[i] = 0u;
}

}  // namespace

int moc_eval_static_setup(int device) {
  if (device < 0 || device >= kMaxDevices) return MOC_EINVAL;
  std::lock_guard<std::mutex> lock(g_scratch_mu);
  if (g_scratch_ptr[device]) return MOC_OK;
  uint32_t* ptr = nullptr;
  MOC_HIP(hipGetSymbolAddress(reinterpret_cast<void**>(&ptr), HIP_SYMBOL(scratch)));
  if (!ptr) return MOC_EINVAL;
  g_scratch_ptr[device] = ptr;
  return MOC_OK;
}

extern "C" int moc_eval_batch_noalloc(const moc_graph* g, int64_t B, const int32_t* starts, const int32_t* ends,
                                      const uint8_t* active, moc_result* out, void* hip_stream) {
  const int rc = check_arguments(g, B, starts, ends, active, out);
  if (rc != MOC_OK || B == 0) return rc;
  if (B > MOC_NOALLOC_MAX_B) return MOC_EOVERFLOW;
  uint32_t* counters;
  {
    std::lock_guard<std::mutex> lock(g_scratch_mu);
    counters = g_scratch_ptr[g->device];   // set when the graph was uploaded on this device
  }
  if (!counters) return MOC_EINVAL;
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  // the array keeps what the last call left in it: start from zero (a kernel, not a memset,
  // so that the call can be recorded into a HIP graph)
  hipLaunchKernelGGL(clear_counters_kernel, dim3(1), dim3(256), 0, st, counters);
  MOC_HIP(hipGetLastError());
  return dispatch(g, B, starts, ends, active, out, st, vector_aligned(g->view.C, starts, ends, active),
                  LaunchOpts{counters, false});
}
