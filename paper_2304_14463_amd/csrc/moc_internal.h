// Internal declarations shared by the translation units of libmoccasin_hip.so.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "moccasin.h"

// A copy that is not live is staged as s = 0xFFFF, e = 0: no position x
// satisfies s < x <= e, so it can never cover a consumer (Eq. (5)).
#define MOC_DEAD 0x0000FFFFu

constexpr int kWave = 64;  // CDNA wavefront

// Device-side view of an uploaded graph, passed to kernels by value.
struct GraphView {
  const int2* size_dur;        // [n] {m_v, w_v}
  const uint32_t* slot_info;   // [n_slices*64] (v*C) | in-degree << 16, nodes sorted by in-degree (desc)
  const uint16_t* ell_pred;    // sliced ELL: slice sl, edge j, lane l at ell_ptr[sl] + j*64 + l -> u*C
  const int32_t* ell_ptr;      // [n_slices+1]
  const int32_t* in_ptr;       // [n+1] plain CSR by in-edges
  const int32_t* in_idx;       // [m]
  const int32_t* out_ptr;      // [n+1] CSR by out-edges
  const int32_t* out_idx;      // [m]
  int64_t budget;
  int32_t n, m, C, T, n_slices;
};

struct moc_graph {
  int device;
  int num_cu;
  int max_lds;       // bytes of LDS one workgroup may use
  GraphView view;    // device pointers
  void* allocs[8];   // device allocations backing `view`
  int n_allocs;
};

int moc_set_hip_error(hipError_t e);  // records e, returns MOC_EHIP

#define MOC_HIP(call)                                  \
  do {                                                 \
    hipError_t moc_e_ = (call);                        \
    if (moc_e_ != hipSuccess) return moc_set_hip_error(moc_e_); \
  } while (0)
