// Generic feature-map kernel (Eq. 1, Eq. 2) for any shape and storage type, and the state
// reset.  Weights are stored output-major: W1 [R'][D], W2 [R][R'], W3 [R][R] per head.
#include "lessdec_common.h"
#include "lessdec_internal.h"

namespace lessdec {

// =====================================================================================
// Feature maps, generic path: any D, R', R, either storage type, fp64 accumulation in the
// oracle's summation order.  One block evaluates TM rows that share a head, so the
// head's weights are read once per TM rows.
//   x    : rows of D values; row (u * rpu + p) belongs to unit u = b * Hh + h
//   out  : [rows, R] as double (out_f64) or float
//   W3   : NULL for phi (Eq. 1), the R x R matrix for psi (Eq. 2)
// grid = Hh * ceil(B * rpu / TM) (head fastest), block = 256, dynamic LDS = TM * (D + R' + R) doubles
// =====================================================================================
template <typename T, int TM>
__global__ __launch_bounds__(256) void featmap_generic_kernel(
    const T *__restrict__ x, const T *__restrict__ W1, const T *__restrict__ W2,
    const T *__restrict__ W3, void *__restrict__ out, int out_f64,
    int B, int Hh, int rpu, int D, int Rp, int R)
{
  extern __shared__ double sm[];
  double *xs = sm;                 // [TM][D]
  double *hs = xs + TM * D;        // [TM][Rp]
  double *h2 = hs + TM * Rp;       // [TM][R]
  const int h = blockIdx.x % Hh;
  const long rows_head = (long)B * rpu;
  const long i0 = (long)(blockIdx.x / Hh) * TM;
  const int tid = threadIdx.x;
  const T *W1h = W1 + (size_t)h * D * Rp;
  const T *W2h = W2 + (size_t)h * Rp * R;

  auto global_row = [&](long i) -> long {   // i-th row of this head -> row in x / out
    long b = i / rpu, p = i % rpu;
    return (b * Hh + h) * (long)rpu + p;
  };

  for (int idx = tid; idx < TM * D; idx += 256) {
    int m = idx / D, d = idx % D;
    long i = i0 + m;
    xs[idx] = (i < rows_head) ? (double)Store<T>::to_float(x[global_row(i) * D + d]) : 0.0;
  }
  __syncthreads();

  for (int i = tid; i < Rp; i += 256) {
    double a[TM];
#pragma unroll
    for (int m = 0; m < TM; ++m) a[m] = 0.0;
    for (int d = 0; d < D; ++d) {
      double w = (double)Store<T>::to_float(W1h[(size_t)i * D + d]);
#pragma unroll
      for (int m = 0; m < TM; ++m) a[m] = fma(xs[m * D + d], w, a[m]);
    }
#pragma unroll
    for (int m = 0; m < TM; ++m) hs[m * Rp + i] = gelu_f64(a[m]);
  }
  __syncthreads();

  for (int pr = tid; pr < TM * R; pr += 256) {
    int m = pr / R, r = pr % R;
    double a = 0.0;
    for (int i = 0; i < Rp; ++i)
      a = fma(hs[m * Rp + i], (double)Store<T>::to_float(W2h[(size_t)r * Rp + i]), a);
    h2[pr] = gelu_f64(a);
  }
  __syncthreads();

  for (int pr = tid; pr < TM * R; pr += 256) {
    int m = pr / R, r = pr % R;
    long i = i0 + m;
    if (i >= rows_head) continue;
    double g;
    if (W3 == nullptr) {
      g = fabs(h2[pr]);
    } else {
      const T *W3h = W3 + (size_t)h * R * R;
      double a = 0.0;
      for (int j = 0; j < R; ++j)
        a = fma(h2[m * R + j], (double)Store<T>::to_float(W3h[(size_t)r * R + j]), a);
      g = fabs(a);
    }
    const size_t o = (size_t)global_row(i) * R + r;
    if (out_f64) reinterpret_cast<double *>(out)[o] = g;
    else reinterpret_cast<float *>(out)[o] = (float)g;
  }
}

template <typename T>
static hipError_t launch_featmap_generic_t(const FeatmapArgs &a, hipStream_t st)
{
  const long rows_head = (long)a.B * a.rpu;
  if (a.Rp <= 512) {
    constexpr int TM = 8;
    const unsigned grid = (unsigned)(a.Hh * ((rows_head + TM - 1) / TM));
    size_t lds = sizeof(double) * TM * (size_t)(a.D + a.Rp + a.R);
    featmap_generic_kernel<T, TM><<<grid, 256, lds, st>>>(
        (const T *)a.x, (const T *)a.W1, (const T *)a.W2, (const T *)a.W3, a.out, a.out_f64,
        a.B, a.Hh, a.rpu, a.D, a.Rp, a.R);
  } else {
    constexpr int TM = 2;
    const unsigned grid = (unsigned)(a.Hh * ((rows_head + TM - 1) / TM));
    size_t lds = sizeof(double) * TM * (size_t)(a.D + a.Rp + a.R);
    featmap_generic_kernel<T, TM><<<grid, 256, lds, st>>>(
        (const T *)a.x, (const T *)a.W1, (const T *)a.W2, (const T *)a.W3, a.out, a.out_f64,
        a.B, a.Hh, a.rpu, a.D, a.Rp, a.R);
  }
  return hipGetLastError();
}

hipError_t launch_featmap_generic(const FeatmapArgs &a, int dtype, hipStream_t st)
{
  return dtype == LESSDEC_DTYPE_F16 ? launch_featmap_generic_t<__half>(a, st)
                                    : launch_featmap_generic_t<float>(a, st);
}

// =====================================================================================
// Reset: H = 0, z = 0, acc = 0, psi = 0, pos = -1, n_seen = 0, nothing pending (a fill kernel,
// so the call can be recorded into a HIP graph).
// =====================================================================================
__global__ void reset_kernel(float *H, size_t nH, double *z, size_t nz, double *acc, size_t nacc,
                             int32_t *pos, size_t npos, float *psi, size_t npsi, int32_t *n_seen,
                             int32_t *pend_slot, size_t nn)
{
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  const size_t t0 = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  for (size_t i = t0; i < nH; i += stride) H[i] = 0.f;
  for (size_t i = t0; i < nz; i += stride) z[i] = 0.0;
  for (size_t i = t0; i < nacc; i += stride) acc[i] = 0.0;
  for (size_t i = t0; i < npos; i += stride) pos[i] = -1;
  for (size_t i = t0; i < npsi; i += stride) psi[i] = 0.f;
  for (size_t i = t0; i < nn; i += stride) {
    n_seen[i] = 0;
    pend_slot[i] = -1;
  }
}

hipError_t launch_reset(const lessdec_desc *d, hipStream_t st)
{
  const size_t U = (size_t)d->batch * d->heads, C = (size_t)d->n_heavy + d->n_recent;
  const size_t R = d->rank, D = d->head_dim;
  reset_kernel<<<1024, 256, 0, st>>>(d->H, U * R * D, d->z, U * R, d->acc, U * C, d->pos, U * C,
                                     d->psi, U * C * R, d->n_seen, d->pend_slot, U);
  return hipGetLastError();
}

}  // namespace lessdec
