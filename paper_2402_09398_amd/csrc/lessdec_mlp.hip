// psi (Eq. 2), or phi (Eq. 1) when no third matrix is given, of many rows on the matrix cores:
// used by the prompt phase for every prompt key and by the multi-head decode step.
#include "lessdec_internal.h"
#include "lessdec_mlp.h"

namespace lessdec {

// One block = 16 kTiles rows that share a head, as kTiles tiles of 16 (head fastest in blockIdx: with
// Hh a multiple of 8 every block of a head lands on the same XCD and shares its L2 copy of the
// weights).  The four waves split the groups of 32 hidden units and apply each loaded weight
// tile to all the row tiles, add their layer-2 sums through the LDS, and 256 threads finish
// the rows x 16 outputs (activation, W3, absolute value) in fp64.
constexpr int kPsiTiles = 4;      // prompt phase: 64 rows per block
constexpr int kPairTiles = 1;     // decode step: 16 rows per block, so that a batch of 64 fills more of the chip
template <int D, int kTiles>
__device__ inline void mlp_psi_block(const MlpArgs &a, unsigned bid)
{
  __shared__ float s_red[4][16][16 * kTiles + 1];       // [wave][r][row]
  __shared__ double s_h2[16 * kTiles][17];              // [row][r]
  const int tid = threadIdx.x, wave = tid / 64, l = tid % 64, g = l / 16, c = l % 16;
  const int Hh = a.Hh, Rp = a.Rp, R = a.R;
  const int h = bid % Hh, chunk = bid / Hh;
  const __half *W1 = a.W1 + (size_t)h * Rp * D;
  const __half *W2 = a.W2 + (size_t)h * R * Rp;
  const long rows_head = (long)a.B * a.rpu;
  auto global_row = [&](long i) -> long {
    const long bb = i / a.rpu, p = i % a.rpu;
    return (bb * Hh + h) * (long)a.rpu + p;
  };
  v8h bx[kTiles][D / 32];
#pragma unroll
  for (int t = 0; t < kTiles; ++t) {
    const long i = ((long)chunk * kTiles + t) * 16 + c;
    mlp_load_row<D>(a.x + (i < rows_head ? global_row(i) : 0) * D, g, bx[t]);   // padding: any row
  }
  v4f c2[kTiles];
#pragma unroll
  for (int t = 0; t < kTiles; ++t) c2[t] = v4f{0.f, 0.f, 0.f, 0.f};
  for (int grp = wave; grp < Rp / 32; grp += 4) {
    const MlpTiles<D> w = mlp_load_tiles<D>(W1, W2, Rp, R, 32 * grp, g, c);
#pragma unroll
    for (int t = 0; t < kTiles; ++t) mlp_apply_tiles<D>(w, bx[t], c2[t]);
  }
#pragma unroll
  for (int t = 0; t < kTiles; ++t)
#pragma unroll
    for (int w = 0; w < 4; ++w) s_red[wave][4 * g + w][16 * t + c] = c2[t][w];
  __syncthreads();
  const int r = tid % 16;
  for (int row = tid / 16; row < 16 * kTiles; row += 16) {
    const float sum = ((s_red[0][r][row] + s_red[1][r][row]) + s_red[2][r][row]) + s_red[3][r][row];
    s_h2[row][r] = (r < R) ? gelu_poly_f64((double)sum) : 0.0;
  }
  __syncthreads();
  // W3 == nullptr: the map has no third matrix (phi, Eq. 1)
  const __half *W3 = a.W3 ? a.W3 + ((size_t)h * R + (r < R ? r : 0)) * R : nullptr;
  for (int row = tid / 16; row < 16 * kTiles; row += 16) {
    const long i = (long)chunk * (16 * kTiles) + row;
    if (r < R && i < rows_head) {
      double acc3 = 0.0;
      if (W3 != nullptr) {
        for (int j = 0; j < R; ++j) acc3 = fma(s_h2[row][j], (double)__half2float(W3[j]), acc3);
      } else {
        acc3 = s_h2[row][r];
      }
      a.out[(size_t)global_row(i) * R + r] = (float)fabs(acc3);
    }
  }
}

template <int D>
__global__ __launch_bounds__(256) void mlp_psi_kernel(const MlpArgs a)
{
  mlp_psi_block<D, kPsiTiles>(a, blockIdx.x);
}
// two maps in one launch (phi of the queries and psi of the keys of a multi-head decode step):
// the first na blocks work on a, the rest on b
template <int D>
__global__ __launch_bounds__(256) void mlp_pair_kernel(const MlpArgs a, const MlpArgs b, unsigned na)
{
  if (blockIdx.x < na) mlp_psi_block<D, kPairTiles>(a, blockIdx.x);
  else mlp_psi_block<D, kPairTiles>(b, blockIdx.x - na);
}

// Many rows per head (the prompt phase): a workgroup keeps its head's weights in registers and
// streams rows through them.  Wave w holds the groups of 32 hidden units w, w + 4, ... (NGW of
// them: R' = 128 NGW) for the whole kernel; per chunk of 16 kRowTiles rows it loads the rows,
// applies its groups, and the block adds the four layer-2 sums through the LDS and finishes the
// outputs as above (same arithmetic in the same order as mlp_psi_block: identical results).  The
// next chunk's rows are requested before the current chunk's arithmetic.
// grid = Hh * parts (head fastest), every block a contiguous share of the head's chunks.
constexpr int kRowTiles = 1;
template <int D, int NGW>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2, 2))) void mlp_rows_kernel(const MlpArgs a,
                                                                                                  int parts)
{
  __shared__ float s_red[4][16][16 * kRowTiles + 1];       // [wave][r][row]
  __shared__ double s_h2[16 * kRowTiles][17];              // [row][r]
  const int tid = threadIdx.x, wave = tid / 64, l = tid % 64, g = l / 16, c = l % 16;
  const int Hh = a.Hh, Rp = a.Rp, R = a.R;
  const int h = (int)blockIdx.x % Hh, part = (int)blockIdx.x / Hh;
  const __half *W1 = a.W1 + (size_t)h * Rp * D;
  const __half *W2 = a.W2 + (size_t)h * R * Rp;
  // 32-bit row arithmetic (the launcher checks that a head's rows fit): a 64-bit division per row
  // would be a long instruction sequence
  const unsigned rows_head = (unsigned)a.B * (unsigned)a.rpu, rpu = (unsigned)a.rpu;
  const unsigned nchunk = (rows_head + 16 * kRowTiles - 1) / (16 * kRowTiles);
  const unsigned ch0 = (unsigned)((unsigned long)nchunk * part / parts);
  const unsigned ch1 = (unsigned)((unsigned long)nchunk * (part + 1) / parts);
  auto global_row = [&](unsigned i) -> size_t {
    const unsigned bb = i / rpu, p = i - bb * rpu;
    return ((size_t)bb * Hh + h) * rpu + p;
  };
  MlpTiles<D> w[NGW];
#pragma unroll
  for (int k = 0; k < NGW; ++k) w[k] = mlp_load_tiles<D>(W1, W2, Rp, R, 32 * (wave + 4 * k), g, c);
  const int r = tid % 16;
  __shared__ double s_w3[16][17];                          // W3 of the head, widened once; W3 == nullptr: phi (Eq. 1)
  {
    const int j = tid / 16;
    s_w3[r][j] = (a.W3 != nullptr && r < R && j < R) ? (double)__half2float(a.W3[((size_t)h * R + r) * R + j]) : 0.0;
  }

  auto load_chunk = [&](unsigned ch, v8h (&bx)[kRowTiles][D / 32]) {
#pragma unroll
    for (int t = 0; t < kRowTiles; ++t) {
      const unsigned i = (ch * kRowTiles + t) * 16 + c;
      mlp_load_row<D>(a.x + (i < rows_head ? global_row(i) : 0) * D, g, bx[t]);   // padding: any row
    }
  };
  v8h bx_next[kRowTiles][D / 32];
  if (ch0 < ch1) load_chunk(ch0, bx_next);
  for (unsigned ch = ch0; ch < ch1; ++ch) {
    v8h bx[kRowTiles][D / 32];
#pragma unroll
    for (int t = 0; t < kRowTiles; ++t)
#pragma unroll
      for (int ks = 0; ks < D / 32; ++ks) bx[t][ks] = bx_next[t][ks];
    load_chunk(ch + 1 < ch1 ? ch + 1 : ch, bx_next);
    v4f c2[kRowTiles];
#pragma unroll
    for (int t = 0; t < kRowTiles; ++t) c2[t] = v4f{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int k = 0; k < NGW; ++k)
#pragma unroll
      for (int t = 0; t < kRowTiles; ++t) mlp_apply_tiles<D>(w[k], bx[t], c2[t]);
    __syncthreads();                                       // the previous chunk's readers are done
#pragma unroll
    for (int t = 0; t < kRowTiles; ++t)
#pragma unroll
      for (int q = 0; q < 4; ++q) s_red[wave][4 * g + q][16 * t + c] = c2[t][q];
    __syncthreads();
    for (int row = tid / 16; row < 16 * kRowTiles; row += 16) {
      const float sum = ((s_red[0][r][row] + s_red[1][r][row]) + s_red[2][r][row]) + s_red[3][r][row];
      s_h2[row][r] = (r < R) ? gelu_poly_f64((double)sum) : 0.0;
    }
    __syncthreads();
    for (int row = tid / 16; row < 16 * kRowTiles; row += 16) {
      const unsigned i = ch * (16 * kRowTiles) + row;
      if (r < R && i < rows_head) {
        double acc3 = 0.0;
        if (a.W3 != nullptr) {
          for (int j = 0; j < R; ++j) acc3 = fma(s_h2[row][j], s_w3[r][j], acc3);
        } else {
          acc3 = s_h2[row][r];
        }
        a.out[(size_t)global_row(i) * R + r] = (float)fabs(acc3);
      }
    }
  }
}

// Decode step: both maps for every unit, by parts of 64 hidden units, one job of mlp_parts_job
// per block.
template <int D>
__global__ __launch_bounds__(256) void mlp_parts_kernel(const __half *q, const __half *k, const __half *Wq1,
                                                        const __half *Wk1, const __half *Wq2, const __half *Wk2,
                                                        int Hh, int rrp, int x_stride, int B, float *out)
{
  // Plain scalar arguments, the ones the loads need first: the launch can preload the first
  // sixteen dwords into registers (the compile flag asks for it),
  // which takes the argument fetch out of a kernel that is one chain of latencies.  rrp = R | R' << 8.
  __shared__ __attribute__((aligned(16))) unsigned char s_slabs[2 * mlp_slab_bytes(D)];
  mlp_parts_block<D, false>(q, k, Wq1, Wk1, Wq2, Wk2, Hh, rrp >> 8, rrp & 0xff, B, x_stride, out, (int)blockIdx.x,
                            s_slabs, (int)threadIdx.x / 64, (int)threadIdx.x % 64);
}

// Decode step with G query heads per key head: phi of every query row and psi of every key row by
// parts, one job of mlp_parts_gq_job per block.  hg = Hk | G << 16, rrp = R | R' << 8.
template <int D>
__global__ __launch_bounds__(256) void mlp_parts_gq_kernel(const __half *q, const __half *k, const __half *Wq1,
                                                           const __half *Wk1, const __half *Wq2, const __half *Wk2,
                                                           int hg, int rrp, int B, float *out)
{
  __shared__ __attribute__((aligned(16))) unsigned char s_slab[mlp_slab_bytes(D)];
  mlp_parts_gq_job<D, false>(q, k, Wq1, Wk1, Wq2, Wk2, hg & 0xffff, hg >> 16, rrp >> 8, rrp & 0xff, B, out,
                             (int)blockIdx.x, s_slab, (int)threadIdx.x / 64, (int)threadIdx.x % 64);
}

bool mlp_mfma_supported(int dtype, int D, int Rp, int R)
{
  return dtype == LESSDEC_DTYPE_F16 && (D == 64 || D == 128) && Rp % 32 == 0 && Rp >= 32 && R <= 16;
}

hipError_t launch_mlp(const MlpArgs &a, hipStream_t st)
{
  const long rows_head = (long)a.B * a.rpu;
  // many rows per head and R' = 128, 256, 384 or 512: weights stay in registers, rows stream through
  const int ngw = a.Rp % 128 == 0 ? a.Rp / 128 : 0;
  const long nchunk = (rows_head + 16 * kRowTiles - 1) / (16 * kRowTiles);
  if (ngw >= 1 && ngw <= 4 && nchunk >= 64 && rows_head < (1L << 31) - 64) {
    long parts = 1024 / a.Hh;                              // about four workgroups per compute unit
    if (parts < 1) parts = 1;
    if (parts > nchunk / 8) parts = nchunk / 8;            // at least 8 chunks behind every weight load
    const unsigned grid = (unsigned)(a.Hh * parts);
#define LESSDEC_MLP_ROWS(DD, NG) mlp_rows_kernel<DD, NG><<<grid, 256, 0, st>>>(a, (int)parts)
    if (a.D == 128) {
      if (ngw == 1) LESSDEC_MLP_ROWS(128, 1); else if (ngw == 2) LESSDEC_MLP_ROWS(128, 2);
      else if (ngw == 3) LESSDEC_MLP_ROWS(128, 3); else LESSDEC_MLP_ROWS(128, 4);
    } else {
      if (ngw == 1) LESSDEC_MLP_ROWS(64, 1); else if (ngw == 2) LESSDEC_MLP_ROWS(64, 2);
      else if (ngw == 3) LESSDEC_MLP_ROWS(64, 3); else LESSDEC_MLP_ROWS(64, 4);
    }
#undef LESSDEC_MLP_ROWS
    return hipGetLastError();
  }
  const unsigned grid = (unsigned)(((rows_head + 16 * kPsiTiles - 1) / (16 * kPsiTiles)) * a.Hh);
  if (a.D == 128) mlp_psi_kernel<128><<<grid, 256, 0, st>>>(a);
  else mlp_psi_kernel<64><<<grid, 256, 0, st>>>(a);
  return hipGetLastError();
}

hipError_t launch_mlp_pair(const MlpArgs &a, const MlpArgs &b, hipStream_t st)
{
  const unsigned na = (unsigned)((((long)a.B * a.rpu + 16 * kPairTiles - 1) / (16 * kPairTiles)) * a.Hh);
  const unsigned nb = (unsigned)((((long)b.B * b.rpu + 16 * kPairTiles - 1) / (16 * kPairTiles)) * b.Hh);
  if (a.D == 128) mlp_pair_kernel<128><<<na + nb, 256, 0, st>>>(a, b, na);
  else mlp_pair_kernel<64><<<na + nb, 256, 0, st>>>(a, b, na);
  return hipGetLastError();
}

hipError_t launch_mlp_parts(const MlpPartsArgs &a, hipStream_t st)
{
  const unsigned grid = (unsigned)mlp_parts_blocks(a.Hh, a.Rp, a.B);
  const int rrp = a.R | (a.Rp << 8), xs = a.x_stride ? a.x_stride : a.D;
  if (a.D == 128)
    mlp_parts_kernel<128><<<grid, 256, 0, st>>>(a.q, a.k, a.Wq1, a.Wk1, a.Wq2, a.Wk2, a.Hh, rrp, xs, a.B, a.out);
  else
    mlp_parts_kernel<64><<<grid, 256, 0, st>>>(a.q, a.k, a.Wq1, a.Wk1, a.Wq2, a.Wk2, a.Hh, rrp, xs, a.B, a.out);
  return hipGetLastError();
}

// a.Hh: key heads; G query heads each (q rows [B, Hh, G, D], Wq per query head)
hipError_t launch_mlp_parts_gq(const MlpPartsArgs &a, int G, hipStream_t st)
{
  const unsigned grid = (unsigned)mlp_parts_gq_jobs(a.Hh, G, a.Rp, a.B);
  const int rrp = a.R | (a.Rp << 8), hg = a.Hh | (G << 16);
  if (a.D == 128)
    mlp_parts_gq_kernel<128><<<grid, 256, 0, st>>>(a.q, a.k, a.Wq1, a.Wk1, a.Wq2, a.Wk2, hg, rrp, a.B, a.out);
  else
    mlp_parts_gq_kernel<64><<<grid, 256, 0, st>>>(a.q, a.k, a.Wq1, a.Wk1, a.Wq2, a.Wk2, hg, rrp, a.B, a.out);
  return hipGetLastError();
}

}  // namespace lessdec
