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
#include "lessdec_common.h"
#include "lessdec_internal.h"

namespace lessdec {

typedef _Float16 v8h __attribute__((ext_vector_type(8)));
typedef _Float16 v4h __attribute__((ext_vector_type(4)));
typedef float v4f __attribute__((ext_vector_type(4)));

// One wave, 32 hidden units starting at `hid`, 16 rows held in bx: adds W2[:, hid..hid+32)
// gelu(W1[hid..hid+32) x^T) to c2.
template <int D>
__device__ inline void mlp_group(const __half *__restrict__ W1, const __half *__restrict__ W2, int Rp,
                                 int R, int hid, const v8h (&bx)[D / 32], v4f &c2, int g, int c)
{
  constexpr int KS = D / 32;
  v8h a0[KS], a1[KS];
  const __half *w1a = W1 + (size_t)(hid + c) * D + 8 * g;
  const __half *w1b = w1a + (size_t)16 * D;
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) {
    a0[ks] = *reinterpret_cast<const v8h *>(w1a + 32 * ks);
    a1[ks] = *reinterpret_cast<const v8h *>(w1b + 32 * ks);
  }
  // layer-2 A operand: row r = c of W2, the 8 hidden units this lane group owns
  v8h a2 = {0, 0, 0, 0, 0, 0, 0, 0};
  if (c < R) {
    const __half *w2 = W2 + (size_t)c * Rp + hid + 4 * g;
    const v4h lo = *reinterpret_cast<const v4h *>(w2);
    const v4h hi = *reinterpret_cast<const v4h *>(w2 + 16);
    a2 = v8h{lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
  }
  v4f h0 = {0.f, 0.f, 0.f, 0.f}, h1 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) {
    h0 = __builtin_amdgcn_mfma_f32_16x16x32_f16(a0[ks], bx[ks], h0, 0, 0, 0);
    h1 = __builtin_amdgcn_mfma_f32_16x16x32_f16(a1[ks], bx[ks], h1, 0, 0, 0);
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
  c2 = __builtin_amdgcn_mfma_f32_16x16x32_f16(a2, bhi, c2, 0, 0, 0);
  c2 = __builtin_amdgcn_mfma_f32_16x16x32_f16(a2, blo, c2, 0, 0, 0);
}

template <int D>
__device__ inline void load_rows(const __half *x, long i, long rows_head, long grow, int g,
                                 v8h (&bx)[D / 32])
{
  if (i < rows_head) {
    const __half *xr = x + grow * D;
#pragma unroll
    for (int ks = 0; ks < D / 32; ++ks) bx[ks] = *reinterpret_cast<const v8h *>(xr + 32 * ks + 8 * g);
  } else {
#pragma unroll
    for (int ks = 0; ks < D / 32; ++ks) bx[ks] = v8h{0, 0, 0, 0, 0, 0, 0, 0};
  }
}

// One launch serves two kinds of blocks (256 threads each, head fastest in the block index:
// with Hh a multiple of 8 every block of a head lands on the same XCD and shares its L2
// copy of the head's weights):
//   blocks [0, n_part_blocks): "part" blocks of map[0], 16 rows x 128 hidden units each,
//     writing fp32 partial sums of layer 2.  This is the form for phi of the step's query,
//     which the step kernel is waiting for: four times as many, four times shorter blocks.
//   the rest: "full" blocks of map[1], 16 rows x all hidden units, finishing psi (Eq. 2)
//     themselves.  Nothing waits for psi within a step, and the prompt needs nothing else.
template <int D>
__global__ __launch_bounds__(256) void mlp_mfma_kernel(const MlpArgs a)
{
  __shared__ float s_red[4][16][16];              // [wave][r][row]
  __shared__ double s_h2[16][16];                 // [row][r]
  const int tid = threadIdx.x, wave = tid / 64, l = tid % 64, g = l / 16, c = l % 16;
  const int Hh = a.Hh, Rp = a.Rp, R = a.R;
  const bool full = (int)blockIdx.x >= a.n_part_blocks;
  int b = full ? (int)blockIdx.x - a.n_part_blocks : (int)blockIdx.x;
  const int h = b % Hh; b /= Hh;
  const int chunk = b % a.nchunk; b /= a.nchunk;
  const int part = b;                              // part blocks only
  const MlpArgs::Map mp = a.map[full ? 1 : 0];
  const __half *W1 = mp.W1 + (size_t)h * Rp * D;
  const __half *W2 = mp.W2 + (size_t)h * R * Rp;
  const long rows_head = (long)a.B * a.rpu;
  auto global_row = [&](long i) -> long {
    const long bb = i / a.rpu, p = i % a.rpu;
    return (bb * Hh + h) * (long)a.rpu + p;
  };
  v8h bx[D / 32];
  {
    const long i = (long)chunk * 16 + c;
    load_rows<D>(mp.x, i, rows_head, i < rows_head ? global_row(i) : 0, g, bx);
  }
  v4f c2 = {0.f, 0.f, 0.f, 0.f};
  if (full) {
    for (int p = 0; p < a.nparts; ++p)
      mlp_group<D>(W1, W2, Rp, R, p * kMlpPartHidden + 32 * wave, bx, c2, g, c);
  } else {
    mlp_group<D>(W1, W2, Rp, R, part * kMlpPartHidden + 32 * wave, bx, c2, g, c);
  }
  // c2[w]: output r = 4 g + w of row c, summed over this wave's hidden units
#pragma unroll
  for (int w = 0; w < 4; ++w) s_red[wave][4 * g + w][c] = c2[w];
  __syncthreads();
  const int row = tid / 16, r = tid % 16;
  const long i = (long)chunk * 16 + row;
  const float sum = ((s_red[0][r][row] + s_red[1][r][row]) + s_red[2][r][row]) + s_red[3][r][row];
  if (!full) {
    if (i < rows_head) {
      const size_t rows_total = (size_t)a.B * Hh * a.rpu;
      mp.out[((size_t)part * rows_total + (size_t)global_row(i)) * kMlpPartStride + r] = (r < R) ? sum : 0.f;
    }
  } else {                                         // block-uniform branch
    s_h2[row][r] = (r < R) ? gelu_f64((double)sum) : 0.0;
    __syncthreads();
    if (r < R && i < rows_head) {
      const __half *W3 = mp.W3 + ((size_t)h * R + r) * R;
      double acc3 = 0.0;
      for (int j = 0; j < R; ++j) acc3 = fma(s_h2[row][j], (double)__half2float(W3[j]), acc3);
      mp.out[(size_t)global_row(i) * R + r] = (float)fabs(acc3);
    }
  }
}

bool mlp_mfma_supported(int dtype, int D, int Rp, int R)
{
  return dtype == LESSDEC_DTYPE_F16 && (D == 64 || D == 128) && Rp % kMlpPartHidden == 0 &&
         Rp >= kMlpPartHidden && R <= 16;
}

// map[0] (may be unused: parts = false) in part blocks, map[1] in full blocks.
hipError_t launch_mlp(MlpArgs a, bool parts, bool fulls, hipStream_t st)
{
  const long rows_head = (long)a.B * a.rpu;
  a.nchunk = (int)((rows_head + 15) / 16);
  a.nparts = a.Rp / kMlpPartHidden;
  a.n_part_blocks = parts ? a.nparts * a.nchunk * a.Hh : 0;
  const unsigned grid = (unsigned)(a.n_part_blocks + (fulls ? a.nchunk * a.Hh : 0));
  if (a.D == 128) mlp_mfma_kernel<128><<<grid, 256, 0, st>>>(a);
  else mlp_mfma_kernel<64><<<grid, 256, 0, st>>>(a);
  return hipGetLastError();
}

}  // namespace lessdec
