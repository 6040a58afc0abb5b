// Host-side launch interfaces between the C ABI (lessdec_api.hip) and the kernel files.
#pragma once

#include <hip/hip_fp16.h>
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "lessdec.h"

namespace lessdec {

// Feature-map evaluation over rows of D values (Eq. 1 when W3 == NULL, Eq. 2 otherwise).
// Row (u * rpu + p) of x / out belongs to unit u = b * Hh + h and uses head h's weights.
struct FeatmapArgs {
  const void *x;
  const void *W1, *W2, *W3;
  void *out;       // [rows, R], double if out_f64 else float
  int out_f64;
  int B, Hh, rpu;  // batch, heads, rows per unit
  int D, Rp, R;
};
hipError_t launch_featmap_generic(const FeatmapArgs &a, int dtype, hipStream_t st);

// Matrix-core feature maps (fp16 storage): up to two maps (phi of q and psi of k) in one
// launch, same row-to-unit convention as above.
struct FeatmapMfmaArgs {
  struct Map {
    const __half *x, *W1, *W2, *W3;   // W3 == NULL: Eq. 1, else Eq. 2
    void *out;
    int out_f64;
  };
  Map map[2];
  int B, Hh, rpu, D, Rp, R;
  int nchunk;                           // set by the launcher
};
bool featmap_mfma_supported(int dtype, int D, int Rp, int R);
hipError_t launch_featmap_mfma(FeatmapMfmaArgs a, int n_maps, hipStream_t st);

struct StepArgs {
  int C, Nh, Nr, R;
  uint32_t flags;
  void *k_cache, *v_cache;
  double *acc;
  int32_t *pos;
  float *psi;
  float *H;
  double *z;
  int32_t *n_seen;
  int32_t *pend_slot;    // [U] fold left pending by the last step (see step_unit_kernel)
  void *pend_v;          // [U,D] value row of the pending discarded pair
  float *pend_psi;       // [U,R] psi of the last step's key while its slot write is pending
  const void *q, *k, *v;
  void *out;
  int32_t *evicted_pos;
  const double *f_phi;   // [U,R] phi(q) of this step
  const float *psi_new;  // [U,R] psi(k) of this step
};
hipError_t launch_step(const StepArgs &a, int units, int dtype, int D, hipStream_t st);
hipError_t launch_state_sync(const StepArgs &a, int units, int dtype, int D, hipStream_t st);

hipError_t launch_reset(const lessdec_desc *d, hipStream_t st);

struct PrefillArgs {
  const lessdec_desc *d;
  const void *Q, *K, *V;
  int P;
  void *out;
  // workspace carve-up
  double *rowmax, *rowsum;  // [U,P]
  double *colsum;           // [U,P]
  int32_t *slot_of;         // [U,P] slot index of a kept token, -1 if discarded
  float *psi_all;           // [U,P,R]
};
hipError_t launch_prefill(const PrefillArgs &a, hipStream_t st);

}  // namespace lessdec
