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

// Matrix-core psi (Eq. 2) for many rows: fp16 storage, D in {64,128}, R' a multiple of 32,
// R <= 16.  Row convention as above; out is [rows, R] fp32.
struct MlpArgs {
  const __half *x, *W1, *W2, *W3;
  float *out;
  int B, Hh, rpu, D, Rp, R;
};
bool mlp_mfma_supported(int dtype, int D, int Rp, int R);
hipError_t launch_mlp(const MlpArgs &a, hipStream_t st);
hipError_t launch_mlp_pair(const MlpArgs &a, const MlpArgs &b, hipStream_t st);   // both in one launch (same D, R', R)

// Both feature maps of one decode step, up to the layer-2 sums: phi of q and psi of k for
// every unit, the hidden units split into parts of kMlpPartHidden.  out[((u * 2 + map) * nparts +
// part) * mlp_entry_stride(R) + r] is part's share of the layer-2 pre-activation r of unit u (map 0:
// q with Wq, map 1: k with Wk); the reader adds the parts and finishes Eq. 1 / Eq. 2.
constexpr int kMlpPartHidden = 64;
struct MlpPartsArgs {
  const __half *q, *k, *Wq1, *Wq2, *Wk1, *Wk2;
  float *out;
  int B, Hh, D, Rp, R;
  int x_stride = 0;      // elements from a unit's q / k row to the next unit's (0: D, rows packed)
};
__host__ __device__ inline int mlp_nparts(int Rp) { return (Rp + kMlpPartHidden - 1) / kMlpPartHidden; }
// Entries per (map, part, unit) in the exchange array: the rank rounded up to the four outputs a
// lane of the matrix tile holds.
__host__ __device__ inline int mlp_entry_stride(int R) { return (R + 3) / 4 * 4; }
hipError_t launch_mlp_parts(const MlpPartsArgs &a, hipStream_t st);
// G query heads per key head (a.Hh key heads): entries [query row][part] for phi, then [unit][part]
// for psi, (G + 1) * B * Hh * nparts * mlp_entry_stride(R) floats
hipError_t launch_mlp_parts_gq(const MlpPartsArgs &a, int G, hipStream_t st);

// pend_slot: -1 nothing; else slot index (C = the step's own pair) | kPendNoFold
constexpr int kPendNoFold = 1 << 30;

struct StepArgs {
  int C, Nh, Nr, R, Rp;
  uint32_t flags;
  void *k_cache, *v_cache;
  double *acc;
  int32_t *pos;
  float *psi;
  float *H;
  double *z;
  int32_t *n_seen;
  int32_t *pend_slot;    // [U] work left pending by the last step (see lessdec_step.hip)
  void *pend_v;          // [U,D] value row of the pending discarded pair
  float *pend_psi;       // [U,R] psi of the last step's key
  const void *q, *k, *v;
  void *out;
  int32_t *evicted_pos;
  int x_stride;          // wave-per-unit path: elements from a unit's q / k / v / out row to the next unit's
                         // (D for packed rows; P D when the rows are token t of [U,P,D] prompt arrays)
  int U, Hh, B;
  // generic path: feature maps of this step's q and k from the launches before it
  const double *f_phi;   // [U,R] ([U,G,R] with several query heads per unit)
  const float *f_phi32;  // the same in fp32 from the matrix-core feature maps, or NULL
  double *gqa_parts;     // [U, head blocks, C+2] a step's probability sums per block of heads
  const float *f_psi;    // [U,R]
  // wave-per-unit path: layer-2 sums of both feature maps by parts (launch_mlp_parts), and W3
  const float *mlp_parts;
  float *mlp_out;        // the same array, for handing entries back empty (and, fused, for writing them)
  const void *Wk3;
  const void *Wk2;       // fused launch only (the other weight pointers are kernel arguments of their own)
};
hipError_t launch_step(const StepArgs &a, int dtype, int D, hipStream_t st);
// several query heads per unit: q, out [U,G,D], f_phi [U,G,R]
hipError_t launch_step_gqa(const StepArgs &a, int G, int dtype, int D, hipStream_t st);
constexpr int kGqaMaxHeadBlocks = 8;
int gqa_head_blocks(long units, int G);
hipError_t launch_state_sync(const StepArgs &a, int dtype, int D, hipStream_t st);
// several query heads per unit, streaming form: one block per unit, one wave per query head
// (lessdec_gqs.hip); leaves the discarded pair pending like the single-head streaming path
bool gqs_supported(int dtype, int D, int C, int R, int G);
// whether that kernel finishes the feature maps itself from the parts of launch_mlp_parts_gq
// (StepArgs::mlp_parts set) instead of taking them complete (f_phi32, f_psi)
bool gqs_takes_parts(int Rp);
// fm: the step's feature-map jobs run as the first workgroups of the same launch (gqs_fusable shapes)
hipError_t launch_step_gqs(const StepArgs &a, int G, int D, hipStream_t st, const MlpPartsArgs *fm = nullptr);
bool gqs_fusable(int D, int C, int Rp, int R, int G);

// One wave per unit, K and V streamed through a register ring (lessdec_wpu.hip).
bool wpu_supported(int dtype, int D, int C, int Rp, int R);
// fm == nullptr: the step's feature-map sums are in a.mlp_parts already (launch_mlp_parts ran
// before).  fm != nullptr (only where wpu_fusable says so): one launch does both.
hipError_t launch_step_wpu(const StepArgs &a, int D, hipStream_t st, const MlpPartsArgs *fm = nullptr);
// Whether the whole step of this shape runs as one launch: the exchange array must then hold
// kMlpEmpty everywhere when the step starts (launch_fill_empty; every step leaves it so).
bool wpu_fusable(int B, int Hh, int D, int C, int Rp, int R);
hipError_t launch_fill_empty(float *parts, size_t count, hipStream_t st);

hipError_t launch_reset(const lessdec_desc *d, hipStream_t st);

struct PrefillArgs {
  const lessdec_desc *d;
  const void *Q, *K, *V;
  int P;
  void *out;
  // workspace carve-up
  double *lse;              // [U,P] ln sum_j e^{s_ij} of every causal row
  double *colsum;           // [U,P]
  int32_t *slot_of;         // [U,P] slot index of a kept token, -1 if discarded
  float *approx;            // [U,P] cheap column sums (selection band only)
  int32_t *list;            // [U,P] tokens whose exact column sum is wanted; later keep flags
  int32_t *count;           // [U] length of each unit's list
  float *bound;             // [U] largest score magnitude the unit's prompt can produce (selection band)
  float *psi_all;           // [U,P,R]
  float *phi_all = nullptr; // [U*G,P,R], only for the masked form
  float *psimax = nullptr;  // [U,R] feature-wise maximum of psi over the prompt, only for the masked form
  float *hpre = nullptr;    // [U, P/64+1, R, D] prefix sums of psi^T v, only for the masked form
  float *zpre = nullptr;    // [U, P/64+1, R] prefix sums of psi, only for the masked form
  int masked = 0;           // Lambda-masking through the prompt token by token, all rows at once
};
hipError_t launch_prefill(const PrefillArgs &a, hipStream_t st);

// Row staging for the prompt phase taken token by token: rows [U,P,D] <-> one step's [U,D].
struct PromptRowsArgs {
  const void *Q, *K, *V;   // [U,P,D] dtype
  void *out;               // [U,P,D] dtype or NULL
  void *qs, *ks, *vs;      // [U,G,D], [U,D], [U,D] dtype: token `gather`'s rows
  void *outs;              // [U,G,D] dtype: the output of token `scatter`
  int P, D, dtype, G;      // Q and out are [U,G,P,D]
  unsigned U;
};
// gather < 0: nothing staged; scatter < 0: nothing written back
hipError_t launch_prompt_rows(const PromptRowsArgs &a, int gather, int scatter, hipStream_t st);

}  // namespace lessdec
