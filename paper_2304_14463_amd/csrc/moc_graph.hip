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

    const int ns = moc_node_stride(C);
    const bool wide_ok = (int64_t)(n + 1) * ns <= 0xFFFF;   // else only the kernel for any C runs
    std::vector<uint32_t> edge_pair(m), edge_pair_c(m);
    for (int v = 0; v < n; ++v)
      for (int q = in_ptr[v]; q < in_ptr[v + 1]; ++q) {
        edge_pair_c[q] = (uint32_t)(in_idx[q] * C) | ((uint32_t)(v * C) << 16);
        edge_pair[q] = wide_ok ? (uint32_t)(in_idx[q] * ns) | ((uint32_t)(v * ns) << 16) : 0u;
      }

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
