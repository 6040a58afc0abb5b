// psi (Eq. 2) of many rows on the matrix cores: used by the prompt phase for every prompt key.
#include "lessdec_internal.h"
#include "lessdec_mlp.h"

namespace lessdec {

// One block = 16 rows that share a head (head fastest in blockIdx: with Hh a multiple of 8
// every block of a head lands on the same XCD and shares its L2 copy of the weights).  The
// four waves split the groups of 32 hidden units, add their layer-2 sums through the LDS, and
// 256 threads finish the 16 x 16 outputs (activation, W3, absolute value) in fp64.
template <int D>
__global__ __launch_bounds__(256) void mlp_psi_kernel(const MlpArgs a)
{
  __shared__ float s_red[4][16][16];              // [wave][r][row]
  __shared__ double s_h2[16][16];                 // [row][r]
  const int tid = threadIdx.x, wave = tid / 64, l = tid % 64, g = l / 16, c = l % 16;
  const int Hh = a.Hh, Rp = a.Rp, R = a.R;
  const int h = blockIdx.x % Hh, chunk = blockIdx.x / Hh;
  const __half *W1 = a.W1 + (size_t)h * Rp * D;
  const __half *W2 = a.W2 + (size_t)h * R * Rp;
  const long rows_head = (long)a.B * a.rpu;
  auto global_row = [&](long i) -> long {
    const long bb = i / a.rpu, p = i % a.rpu;
    return (bb * Hh + h) * (long)a.rpu + p;
  };
  v8h bx[D / 32];
  {
    const long i = (long)chunk * 16 + c;
    mlp_load_row<D>(a.x + (i < rows_head ? global_row(i) : 0) * D, g, bx);    // padding: any row
  }
  v4f c2 = {0.f, 0.f, 0.f, 0.f};
  for (int grp = wave; grp < Rp / 32; grp += 4) {
    const MlpTiles<D> t = mlp_load_tiles<D>(W1, W2, Rp, R, 32 * grp, g, c);
    mlp_apply_tiles<D>(t, bx, c2);
  }
#pragma unroll
  for (int w = 0; w < 4; ++w) s_red[wave][4 * g + w][c] = c2[w];
  __syncthreads();
  const int row = tid / 16, r = tid % 16;
  const long i = (long)chunk * 16 + row;
  const float sum = ((s_red[0][r][row] + s_red[1][r][row]) + s_red[2][r][row]) + s_red[3][r][row];
  s_h2[row][r] = (r < R) ? gelu_poly_f64((double)sum) : 0.0;
  __syncthreads();
  if (r < R && i < rows_head) {
    const __half *W3 = a.W3 + ((size_t)h * R + r) * R;
    double acc3 = 0.0;
    for (int j = 0; j < R; ++j) acc3 = fma(s_h2[row][j], (double)__half2float(W3[j]), acc3);
    a.out[(size_t)global_row(i) * R + r] = (float)fabs(acc3);
  }
}

bool mlp_mfma_supported(int dtype, int D, int Rp, int R)
{
  return dtype == LESSDEC_DTYPE_F16 && (D == 64 || D == 128) && Rp % 32 == 0 && Rp >= 32 && R <= 16;
}

hipError_t launch_mlp(const MlpArgs &a, hipStream_t st)
{
  const long rows_head = (long)a.B * a.rpu;
  const unsigned grid = (unsigned)(((rows_head + 15) / 16) * a.Hh);
  if (a.D == 128) mlp_psi_kernel<128><<<grid, 256, 0, st>>>(a);
  else mlp_psi_kernel<64><<<grid, 256, 0, st>>>(a);
  return hipGetLastError();
}

}  // namespace lessdec
