// Feature maps phi, psi (Eq. 1, Eq. 2) on the matrix cores, fp16 storage.
//
// Both layers of the MLP run on v_mfma_f32_16x16x32_f16 (wave64; lane = 16 g + c; A and B
// take 8 consecutive k from lane (g, i) for matrix row / column i; result register w of
// lane (g, c) is element [4 g + w][c]).
//
// Layer 1, H1 = W1 X^T with M = hidden units, N = 16 rows of x, K = D: fp16 x fp16 products
// are exact in fp32, only the fp32 accumulation rounds.  A wave takes 32 hidden units (two
// M-tiles) at a time, applies GELU in registers, and feeds the result straight into
// layer 2, out = W2 gelu(H1), as the B operand: lane group g already holds the hidden units
// {4 g .. 4 g + 3} of each of the two tiles, which become its 8 k-slots (the A operand, W2,
// is loaded in the same order).  The activations are fp32, so they go through the fp16
// matrix core as hi + lo (two MFMAs): hi = fp16(a), lo = fp16(a - hi) keeps 22 bits, the
// same class of error as the fp32 accumulation.  The hidden activations never leave the
// registers.
#pragma once

#include "lessdec_common.h"

namespace lessdec {

typedef _Float16 v8h __attribute__((ext_vector_type(8)));
typedef _Float16 v4h __attribute__((ext_vector_type(4)));
typedef float v4f __attribute__((ext_vector_type(4)));

// Weights of one group of 32 hidden units, in operand order.
template <int D>
struct MlpTiles {
  v8h a0[D / 32], a1[D / 32];   // layer 1: hidden units hid + c and hid + 16 + c, all of D
  v8h a2;                       // layer 2: row r = c of W2 (c < R), the 8 hidden units of lane group g
};

template <int D>
__device__ inline MlpTiles<D> mlp_load_tiles(const __half *__restrict__ W1, const __half *__restrict__ W2,
                                             int Rp, int R, int hid, int g, int c)
{
  MlpTiles<D> t;
  const __half *w1a = W1 + (size_t)(hid + c) * D + 8 * g;
  const __half *w1b = w1a + (size_t)16 * D;
#pragma unroll
  for (int ks = 0; ks < D / 32; ++ks) {
    t.a0[ks] = *reinterpret_cast<const v8h *>(w1a + 32 * ks);
    t.a1[ks] = *reinterpret_cast<const v8h *>(w1b + 32 * ks);
  }
  // rows c >= R of the layer-2 operand repeat row 0 (loaded unconditionally, so that nothing
  // here waits for a load): their outputs are never looked at
  const __half *w2 = W2 + (size_t)(c < R ? c : 0) * Rp + hid + 4 * g;
  const v4h lo = *reinterpret_cast<const v4h *>(w2);
  const v4h hi = *reinterpret_cast<const v4h *>(w2 + 16);
  t.a2 = v8h{lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
  return t;
}

// One wave, one group of 32 hidden units, 16 rows of x held in bx (lane (g, c): row c,
// elements 32 ks + 8 g ..): adds W2[:, group] gelu(W1[group] x^T) to c2, whose register w
// is output r = 4 g + w of row c.
template <int D>
__device__ inline void mlp_apply_tiles(const MlpTiles<D> &t, const v8h (&bx)[D / 32], v4f &c2)
{
  v4f h0 = {0.f, 0.f, 0.f, 0.f}, h1 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int ks = 0; ks < D / 32; ++ks) {
    h0 = __builtin_amdgcn_mfma_f32_16x16x32_f16(t.a0[ks], bx[ks], h0, 0, 0, 0);
    h1 = __builtin_amdgcn_mfma_f32_16x16x32_f16(t.a1[ks], bx[ks], h1, 0, 0, 0);
  }
  // h0[w], h1[w]: hidden units hid + 4 g + w and hid + 16 + 4 g + w of row c
  v8h bhi, blo;
#pragma unroll
  for (int w = 0; w < 4; ++w) {
    const float x0 = gelu_fast_f32(h0[w]), x1 = gelu_fast_f32(h1[w]);
    const _Float16 s0 = (_Float16)x0, s1 = (_Float16)x1;
    bhi[w] = s0;
    bhi[4 + w] = s1;
    blo[w] = (_Float16)(x0 - (float)s0);
    blo[4 + w] = (_Float16)(x1 - (float)s1);
  }
  c2 = __builtin_amdgcn_mfma_f32_16x16x32_f16(t.a2, bhi, c2, 0, 0, 0);
  c2 = __builtin_amdgcn_mfma_f32_16x16x32_f16(t.a2, blo, c2, 0, 0, 0);
}

// Row c of x in operand order.  The loads are unconditional (a select on validity would
// make the caller wait for them on the spot): for a padding row pass any readable row, its
// outputs are never looked at.
template <int D>
__device__ inline void mlp_load_row(const __half *xr, int g, v8h (&bx)[D / 32])
{
#pragma unroll
  for (int ks = 0; ks < D / 32; ++ks) bx[ks] = *reinterpret_cast<const v8h *>(xr + 32 * ks + 8 * g);
}

}  // namespace lessdec
