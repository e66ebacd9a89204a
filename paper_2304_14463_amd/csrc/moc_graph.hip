// moc_graph_upload / moc_graph_free / error reporting: host-side validation
// and preprocessing of the problem instance (paper, Section 1 problem
// statement and Section 2.1: DAG, durations w_v, sizes m_v, budget M, C).
//
// The evaluation kernel checks precedence constraints (Eq. (5)) one lane per
// edge, so the edges are also stored as a flat list of packed (u*C, v*C)
// pairs in consumer order; the neighbourhood kernel walks the in- and
// out-edge CSR of single nodes.
#include <algorithm>
#include <cstring>
#include <new>
#include <vector>

#include "moc_internal.h"

static thread_local int g_last_hip_error = 0;

int moc_set_hip_error(hipError_t e) {
  g_last_hip_error = (int)e;
  return MOC_EHIP;
}

uint32_t* moc_ticket_set(const moc_graph* g, hipStream_t stream) {
  std::lock_guard<std::mutex> lock(g->mu);
  int i = 0;
  while (i < g->n_ticket_streams && g->ticket_stream[i] != stream) ++i;
  if (i == g->n_ticket_streams) {
    if (i == kTicketSlots) return nullptr;
    g->ticket_stream[g->n_ticket_streams++] = stream;
  }
  return g->tickets + (size_t)i * kTicketSlotWords;
}

int moc_kernel_occupancy(const moc_graph* g, const void* kern, int nt, int lds_bytes, bool no_static_lds,
                         int* per_cu) {
  std::lock_guard<std::mutex> lock(g->mu);
  for (const moc_graph::Occupancy& o : g->occupancy)
    if (o.kern == kern && o.nt == nt && o.lds_bytes == lds_bytes) {
      *per_cu = o.per_cu;
      return MOC_OK;
    }
  // first use of this kernel on this device, by any handle
  static std::mutex prepared_mu;
  static std::vector<std::pair<const void*, int>> prepared;
  {
    std::lock_guard<std::mutex> plock(prepared_mu);
    const std::pair<const void*, int> key(kern, g->device);
    if (std::find(prepared.begin(), prepared.end(), key) == prepared.end()) {
      if (no_static_lds) {
        hipFuncAttributes attr;
        MOC_HIP(hipFuncGetAttributes(&attr, kern));
        if (attr.sharedSizeBytes != 0) return MOC_EINVAL;
      }
      MOC_HIP(hipFuncSetAttribute(kern, hipFuncAttributeMaxDynamicSharedMemorySize, g->max_lds));
      prepared.push_back(key);
    }
  }
  int blocks = 0;
  MOC_HIP(hipOccupancyMaxActiveBlocksPerMultiprocessor(&blocks, kern, nt, (size_t)lds_bytes));
  if (blocks < 1) blocks = 1;
  g->occupancy.push_back(moc_graph::Occupancy{kern, nt, lds_bytes, blocks});
  *per_cu = blocks;
  return MOC_OK;
}


// The edge list of the register-resident kernel.  Lane `tid` of a workgroup of nt threads
// owns the entries j*nt + tid, j < edges_per_lane, and a wave fetches the records of the two
// ends of its 64 entries with one LDS read each.  LDS serves 32 lanes at a time from 32
// four-byte banks (16 lanes at a time for the eight-byte records of C = 2), so the edges are
// dealt out such that, within every aligned group of 32 (16) lanes, the providers fall into
// distinct banks and so do the consumers: such a read costs 2.8 clocks per wave instead of
// the 7.3 of arbitrary indices.  Greedy: a group takes, bank of u by bank of u (fullest row
// first), an edge whose bank of v is still free; what does not fit that way while spare
// entries remain is left for later groups.  Entries without an edge hold a dummy that never
// counts (see the kernel's LDS layout).
static std::vector<uint32_t> place_edges(int n, int C, const int32_t* in_ptr, const int32_t* in_idx, int nt,
                                         int edges_per_lane, int edges_per_lane_used) {
  const int ns = moc_node_stride(C);
  const int banks = ns == 2 ? 16 : 32;   // also the lanes LDS serves at a time
  const size_t slots = (size_t)nt * edges_per_lane_used;   // the kernel skips the entries beyond
  // padding: C <= 2 the node n, which is never live; C >= 3 the satisfied edge (n + 1, n)
  const uint32_t dummy = C >= 3 ? (uint32_t)(n + 1) | ((uint32_t)n << 16) : (uint32_t)(n * ns) | ((uint32_t)(n * ns) << 16);
  std::vector<uint32_t> out((size_t)nt * edges_per_lane, dummy);
  std::vector<std::vector<uint32_t>> bucket((size_t)banks * banks);   // [bank of u][bank of v] -> pairs
  // C >= 3: the first pass over an edge reads the consumer's 16-bit entry, two to a bank word
  auto bank_of_consumer = [&](int v) { return C >= 3 ? (v >> 1) % banks : v % banks; };
  std::vector<int> row(banks, 0);
  size_t left = 0;
  for (int v = 0; v < n; ++v)
    for (int q = in_ptr[v]; q < in_ptr[v + 1]; ++q) {
      const int u = in_idx[q];
      bucket[(size_t)(u % banks) * banks + bank_of_consumer(v)].push_back((uint32_t)(u * ns) | ((uint32_t)(v * ns) << 16));
      ++row[u % banks];
      ++left;
    }
  size_t spare = slots - left;   // entries that may stay empty
  std::vector<int> order(banks);
  for (size_t at = 0; at < slots && left > 0; at += banks) {
    const size_t group = std::min<size_t>(banks, slots - at);
    for (int i = 0; i < banks; ++i) order[i] = i;
    std::sort(order.begin(), order.end(), [&](int a, int b) { return row[a] > row[b]; });
    uint64_t v_used = 0, u_used = 0;
    size_t filled = 0;
    for (int k = 0; k < banks && filled < group; ++k) {
      const int bu = order[k];
      int best = -1;
      size_t best_size = 0;
      for (int bv = 0; bv < banks; ++bv) {
        const size_t sz = bucket[(size_t)bu * banks + bv].size();
        if (!(v_used >> bv & 1) && sz > best_size) best = bv, best_size = sz;
      }
      if (best < 0) continue;
      std::vector<uint32_t>& b = bucket[(size_t)bu * banks + best];
      out[at + filled++] = b.back();
      b.pop_back();
      --row[bu]; --left;
      v_used |= (uint64_t)1 << best;
      u_used |= (uint64_t)1 << bu;
    }
    // fill up with conflicting edges once the spare entries are used up
    while (filled < group && left > 0) {
      const size_t holes = group - filled;
      if (spare >= holes) { spare -= holes; break; }
      int bu = -1, bv = -1;
      size_t best_size = 0;
      for (int i = 0; i < banks * banks; ++i) {   // prefer free banks, then the fullest bucket
        const size_t sz = bucket[i].size();
        if (sz == 0) continue;
        const size_t score = sz + ((u_used >> (i / banks) & 1) ? 0 : slots) + ((v_used >> (i % banks) & 1) ? 0 : slots);
        if (score > best_size) best_size = score, bu = i / banks, bv = i % banks;
      }
      std::vector<uint32_t>& b = bucket[(size_t)bu * banks + bv];
      out[at + filled++] = b.back();
      b.pop_back();
      --row[bu]; --left;
      u_used |= (uint64_t)1 << bu;
      v_used |= (uint64_t)1 << bv;
    }
  }
  return out;
}

template <typename T>
static int upload(moc_graph* g, const std::vector<T>& host, const T** dev) {
  void* p = nullptr;
  const size_t bytes = std::max<size_t>(host.size(), 1) * sizeof(T);
  hipError_t e = hipMalloc(&p, bytes);
  if (e == hipErrorOutOfMemory) return MOC_ENOMEM;
  if (e != hipSuccess) return moc_set_hip_error(e);
  g->allocs[g->n_allocs++] = p;
  if (!host.empty()) MOC_HIP(hipMemcpy(p, host.data(), host.size() * sizeof(T), hipMemcpyHostToDevice));
  *dev = (const T*)p;
  return MOC_OK;
}

extern "C" {

int moc_graph_upload(int32_t n, const int32_t* in_ptr, const int32_t* in_idx, const int32_t* size,
                     const int32_t* dur, int64_t budget, int32_t C, moc_graph** out) {
  if (!out) return MOC_EINVAL;
  *out = nullptr;
  if (n < 1 || C < 1 || !in_ptr || !size || !dur) return MOC_EINVAL;
  if ((int64_t)n * C > MOC_MAX_T) return MOC_EOVERFLOW;
  if (in_ptr[0] != 0) return MOC_EINVAL;
  for (int v = 0; v < n; ++v)
    if (in_ptr[v + 1] < in_ptr[v]) return MOC_EINVAL;
  const int32_t m = in_ptr[n];
  if (m > 0 && !in_idx) return MOC_EINVAL;
  for (int q = 0; q < m; ++q)
    if (in_idx[q] < 0 || in_idx[q] >= n) return MOC_EINVAL;
  int64_t sum_size = 0, sum_dur = 0;
  for (int v = 0; v < n; ++v) {
    if (size[v] < 0 || dur[v] < 0) return MOC_EINVAL;
    sum_size += size[v];
    sum_dur += dur[v];
  }
  // The memory profile and the objective are accumulated in int32 on the device.
  if (sum_size * C >= (int64_t)1 << 31 || sum_dur * C >= (int64_t)1 << 31) return MOC_EOVERFLOW;

  try {
    const int T = n * C;
    std::vector<int2> size_dur(n);
    for (int v = 0; v < n; ++v) size_dur[v] = make_int2(size[v], dur[v]);

    std::vector<uint32_t> edge_pair_c(m);
    for (int v = 0; v < n; ++v)
      for (int q = in_ptr[v]; q < in_ptr[v + 1]; ++q)
        edge_pair_c[q] = (uint32_t)(in_idx[q] * C) | ((uint32_t)(v * C) << 16);
    int nt = 0, edges_per_lane = 0, edges_per_lane_used = 0;
    std::vector<uint32_t> edge_pair;
    if (moc_eval_shape(n, m, C, &nt, &edges_per_lane, &edges_per_lane_used))
      edge_pair = place_edges(n, C, in_ptr, in_idx, nt, edges_per_lane, edges_per_lane_used);

    // out-edge CSR (consumers of every node), used by the neighbourhood kernel
    std::vector<int32_t> out_ptr(n + 1, 0), out_idx(m);
    for (int q = 0; q < m; ++q) ++out_ptr[in_idx[q] + 1];
    for (int v = 0; v < n; ++v) out_ptr[v + 1] += out_ptr[v];
    {
      std::vector<int32_t> fill(out_ptr.begin(), out_ptr.end() - 1);
      for (int v = 0; v < n; ++v)
        for (int q = in_ptr[v]; q < in_ptr[v + 1]; ++q) out_idx[fill[in_idx[q]]++] = v;
    }
    std::vector<int32_t> in_ptr_v(in_ptr, in_ptr + n + 1), in_idx_v(in_idx, in_idx + m);

    moc_graph* g = new moc_graph();   // all members zero
    int rc = MOC_OK;
    hipError_t e = hipGetDevice(&g->device);
    hipDeviceProp_t prop;
    if (e == hipSuccess) e = hipGetDeviceProperties(&prop, g->device);
    if (e != hipSuccess) {
      delete g;
      return moc_set_hip_error(e);
    }
    for (int v = 0; v < n; ++v)
      for (int q = in_ptr[v]; q < in_ptr[v + 1]; ++q)
        if (in_idx[q] == v) g->has_self_loop = 1;
    g->num_cu = prop.multiProcessorCount;
    g->max_lds = (int)prop.sharedMemPerBlock;
    if (moc_eval_lds_bytes(n, m, C, g->max_lds) > g->max_lds) {
      delete g;
      return MOC_EOVERFLOW;
    }
    GraphView& w = g->view;
    w.budget = budget; w.n = n; w.m = m; w.C = C; w.T = T;
    if (rc == MOC_OK) rc = upload(g, size_dur, &w.size_dur);
    if (rc == MOC_OK) rc = upload(g, edge_pair, &w.edge_pair);
    if (rc == MOC_OK) rc = upload(g, edge_pair_c, &w.edge_pair_c);
    if (rc == MOC_OK) rc = upload(g, in_ptr_v, &w.in_ptr);
    if (rc == MOC_OK) rc = upload(g, in_idx_v, &w.in_idx);
    if (rc == MOC_OK) rc = upload(g, out_ptr, &w.out_ptr);
    if (rc == MOC_OK) rc = upload(g, out_idx, &w.out_idx);
    if (rc == MOC_OK) {
      const std::vector<uint32_t> zeros((size_t)kTicketSlots * kTicketSlotWords, 0u);
      const uint32_t* dev = nullptr;
      rc = upload(g, zeros, &dev);
      g->tickets = const_cast<uint32_t*>(dev);
    }
    if (rc == MOC_OK) {
      g->occupancy.reserve(16);
      rc = moc_eval_prepare(g);
    }
    if (rc == MOC_OK) rc = moc_eval_static_setup(g->device);
    if (rc != MOC_OK) {
      for (int i = 0; i < g->n_allocs; ++i) (void)hipFree(g->allocs[i]);
      delete g;
      return rc;
    }
    *out = g;
    return MOC_OK;
  } catch (const std::bad_alloc&) {
    return MOC_ENOMEM;
  }
}

int moc_graph_set_order(moc_graph* g, const int32_t* order) {
  if (!g || !order) return MOC_EINVAL;
  int dev = -1;
  MOC_HIP(hipGetDevice(&dev));
  if (dev != g->device) return MOC_EDEVICE;
  const int n = g->view.n, m = g->view.m;
  try {
    std::vector<int32_t> place(n, -1);
    for (int j = 0; j < n; ++j) {
      if (order[j] < 0 || order[j] >= n || place[order[j]] >= 0) return MOC_EINVAL;   // not a permutation
      place[order[j]] = j;
    }
    // topological: every edge (u, v) has u before v (the graph's arrays are read back from the device)
    std::vector<int32_t> in_ptr(n + 1), in_idx(m);
    MOC_HIP(hipMemcpy(in_ptr.data(), g->view.in_ptr, sizeof(int32_t) * (n + 1), hipMemcpyDeviceToHost));
    if (m) MOC_HIP(hipMemcpy(in_idx.data(), g->view.in_idx, sizeof(int32_t) * m, hipMemcpyDeviceToHost));
    for (int v = 0; v < n; ++v)
      for (int q = in_ptr[v]; q < in_ptr[v + 1]; ++q)
        if (place[in_idx[q]] >= place[v]) return MOC_EINVAL;
    if (!g->place) {
      void* p = nullptr;
      const hipError_t e = hipMalloc(&p, sizeof(int32_t) * n);
      if (e == hipErrorOutOfMemory) return MOC_ENOMEM;
      if (e != hipSuccess) return moc_set_hip_error(e);
      g->place = static_cast<int32_t*>(p);
    } else {
      MOC_HIP(hipDeviceSynchronize());   // launches that read the previous order have finished
    }
    MOC_HIP(hipMemcpy(g->place, place.data(), sizeof(int32_t) * n, hipMemcpyHostToDevice));
    return MOC_OK;
  } catch (const std::bad_alloc&) {
    return MOC_ENOMEM;
  }
}

int moc_graph_info(const moc_graph* g, int32_t* n, int32_t* m, int32_t* C, int32_t* T) {
  if (!g) return MOC_EINVAL;
  if (n) *n = g->view.n;
  if (m) *m = g->view.m;
  if (C) *C = g->view.C;
  if (T) *T = g->view.T;
  return MOC_OK;
}

void moc_graph_free(moc_graph* g) {
  if (!g) return;
  int cur = -1;
  if (hipGetDevice(&cur) == hipSuccess && cur == g->device) (void)hipDeviceSynchronize();
  for (int i = 0; i < g->n_allocs; ++i) (void)hipFree(g->allocs[i]);
  if (g->place) (void)hipFree(g->place);
  delete g;
}

const char* moc_strerror(int code) {
  switch (code) {
    case MOC_OK: return "ok";
    case MOC_EINVAL: return "invalid argument";
    case MOC_EOVERFLOW: return "size limit exceeded (int32 sums or T too large for LDS)";
    case MOC_ENOMEM: return "out of memory";
    case MOC_EHIP: return "HIP runtime error (see moc_last_hip_error)";
    case MOC_EDEVICE: return "graph was uploaded on a different device than the current one";
    default: return "unknown error";
  }
}

int moc_last_hip_error(void) { return g_last_hip_error; }

}  // extern "C"
