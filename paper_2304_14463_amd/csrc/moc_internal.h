// Internal declarations shared by the translation units of libmoccasin_hip.so.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <atomic>
#include <mutex>
#include <vector>

#include "moccasin.h"

// A copy that is not live is staged as s = 0xFFFF, e = 0: no position x
// satisfies s < x <= e, so it can never cover a consumer (Eq. (5)).
#define MOC_DEAD 0x0000FFFFu

constexpr int kWave = 64;  // CDNA wavefront

// Device-side view of an uploaded graph, passed to kernels by value.
struct GraphView {
  const int2* size_dur;        // [n] {m_v, w_v}
  const uint32_t* edge_pair;   // edges (u,v) as u*NS | v*NS << 16, NS = moc_node_stride(C), in the order and
                               // with the padding the register-resident kernel reads them (see moc_place_edges)
  const uint32_t* edge_pair_c; // [m] edges as u*C | v*C << 16, ordered by v (kernel for any C)
  const int32_t* in_ptr;       // [n+1] plain CSR by in-edges
  const int32_t* in_idx;       // [m]
  const int32_t* out_ptr;      // [n+1] CSR by out-edges
  const int32_t* out_idx;      // [m]
  int64_t budget;
  int32_t n, m, C, T;
};

constexpr int kTicketSlots = 16;   // sets of work counters per graph handle = streams that get one of their own
constexpr int kTicketGroups = 64;  // counters a launch draws candidates from (+1: workgroups that have left)
constexpr int kTicketStride = 16;  // words from one counter to the next
constexpr int kTicketSlotWords = (kTicketGroups + 1) * kTicketStride;

struct moc_graph {
  int device;
  int num_cu;
  int max_lds;       // bytes of LDS one workgroup may use
  int has_self_loop; // an edge (v,v) exists: the neighbourhood kernel does not take such graphs
  GraphView view;    // device pointers
  void* allocs[8];   // device allocations backing `view`, and `tickets`
  int n_allocs;
  int32_t* place;    // device, [n]: place of every node in the order given to moc_graph_set_order; null before
  // Work counters of the evaluation kernel: kTicketSlots sets of kTicketGroups + 1 counters,
  // each counter on a 64-byte line of its own, all zero between launches (a launch leaves its
  // set at zero when it ends).  A set belongs to a stream: launches on one stream follow each
  // other, so they may share counters; launches on different streams may run at the same time
  // and must not.  The first kTicketSlots streams seen with this handle get a set each
  // (ticket_stream[i] owns set i); launches on further streams are split statically and touch
  // no counters.
  uint32_t* tickets;
  mutable std::mutex mu;   // guards ticket_stream, n_ticket_streams and occupancy
  mutable hipStream_t ticket_stream[kTicketSlots];
  mutable int n_ticket_streams;
  // workgroups per compute unit of (kernel, workgroup size, dynamic LDS bytes), asked once each
  struct Occupancy { const void* kern; int nt, lds_bytes, per_cu; };
  mutable std::vector<Occupancy> occupancy;
};

// The set of work counters that launches of this handle on `stream` draw from, or nullptr
// when all sets belong to other streams (the launch is then split statically).
uint32_t* moc_ticket_set(const moc_graph* g, hipStream_t stream);

// Workgroups of `kern` with nt threads and lds_bytes of dynamic LDS that a compute unit of
// the graph's device holds (at least 1).  On the first use of a kernel on a device its
// dynamic-LDS limit is raised to all the LDS a workgroup can have; with no_static_lds the
// kernel must declare no static LDS (MOC_EINVAL otherwise).  Results are kept per handle.
int moc_kernel_occupancy(const moc_graph* g, const void* kern, int nt, int lds_bytes, bool no_static_lds,
                         int* per_cu);

// Unit of the node indices in GraphView::edge_pair = words per node in the first record array
// of the register-resident kernel: C for C <= 2 (all copies of a node in one record), 1 for
// C >= 3 (first copies only; the other copies are kept in a second array).
int moc_node_stride(int C);

// LDS bytes one workgroup of the evaluation kernel needs for a graph of n nodes, m edges, C copies
// when max_lds bytes are available (optional buffers shrink to fit).
int moc_eval_lds_bytes(int n, int m, int C, int max_lds);

// Workgroup size and edges per lane of the register-resident evaluation kernel for this
// graph (the list holds edges_per_lane entries per lane, of which the first
// edges_per_lane_used are looked at); false if the graph does not take that kernel.
bool moc_eval_shape(int n, int m, int C, int* nt, int* edges_per_lane, int* edges_per_lane_used);

// First-use set-up of the evaluation kernels this graph takes (called at upload, so that
// moc_eval_batch finds everything in the handle).
int moc_eval_prepare(const moc_graph* g);

// Asks the current device (which must be `device`) for the address of the work counters of
// moc_eval_batch_noalloc; once per device.
int moc_eval_static_setup(int device);

int moc_set_hip_error(hipError_t e);  // records e, returns MOC_EHIP

#define MOC_HIP(call)                                  \
  do {                                                 \
    hipError_t moc_e_ = (call);                        \
    if (moc_e_ != hipSuccess) return moc_set_hip_error(moc_e_); \
  } while (0)
