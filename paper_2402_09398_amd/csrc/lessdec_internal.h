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

// Matrix-core feature maps (fp16 storage, D in {64,128}, R' a multiple of 128, R <= 16).
// Row convention as above.  Two kinds of blocks in one launch:
//  - part blocks (map[0], phi): 16 rows x 128 hidden units each, writing the layer-2
//    pre-activation partial sums out[(part * rows + row) * 16 + r] (fp32); the reader adds
//    the R'/128 parts and applies the last activation of Eq. 1.
//  - full blocks (map[1], psi): 16 rows x all hidden units, writing psi [rows, R] itself.
constexpr int kMlpPartHidden = 128;
constexpr int kMlpPartStride = 16;      // floats per row in a partial-sum buffer
struct MlpArgs {
  struct Map {
    const __half *x, *W1, *W2, *W3;
    float *out;                          // parts: partial sums; full: psi [rows, R]
  };
  Map map[2];
  int B, Hh, rpu, D, Rp, R;
  int nchunk, nparts, n_part_blocks;     // set by the launcher
};
bool mlp_mfma_supported(int dtype, int D, int Rp, int R);
hipError_t launch_mlp(MlpArgs a, bool parts, bool fulls, hipStream_t st);

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
  // feature maps of this step's q and k: either final values (generic path) ...
  const double *f_phi;   // [U,R] phi(q)
  const float *psi_new;  // [U,R] psi(k)
  // ... or layer-2 partial sums from the matrix-core path (nparts > 0)
  const float *part_phi;              // [nparts, U, 16]
  int nparts, U;
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
