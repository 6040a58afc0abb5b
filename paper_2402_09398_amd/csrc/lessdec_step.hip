// Decode-step kernels: feature maps of the step's q and k (Eq. 1, Eq. 2) and the fused
// attention / score-accumulate / evict / state-update kernel (Algorithm 1, Eq. 3-5).
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
    const T *__restrict__ W3, void *__restrict__ out, int out_f64, int B, int Hh, int rpu, int D,
    int Rp, int R)
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
      double w = (double)Store<T>::to_float(W1h[(size_t)d * Rp + i]);
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
      a = fma(hs[m * Rp + i], (double)Store<T>::to_float(W2h[(size_t)i * R + r]), a);
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
        a = fma(h2[m * R + j], (double)Store<T>::to_float(W3h[(size_t)j * R + r]), a);
      g = fabs(a);
    }
    size_t o = (size_t)global_row(i) * R + r;
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
        (const T *)a.x, (const T *)a.W1, (const T *)a.W2, (const T *)a.W3, a.out, a.out_f64, a.B,
        a.Hh, a.rpu, a.D, a.Rp, a.R);
  } else {
    constexpr int TM = 2;
    const unsigned grid = (unsigned)(a.Hh * ((rows_head + TM - 1) / TM));
    size_t lds = sizeof(double) * TM * (size_t)(a.D + a.Rp + a.R);
    featmap_generic_kernel<T, TM><<<grid, 256, lds, st>>>(
        (const T *)a.x, (const T *)a.W1, (const T *)a.W2, (const T *)a.W3, a.out, a.out_f64, a.B,
        a.Hh, a.rpu, a.D, a.Rp, a.R);
  }
  return hipGetLastError();
}

hipError_t launch_featmap_generic(const FeatmapArgs &a, int dtype, hipStream_t st)
{
  return dtype == LESSDEC_DTYPE_F16 ? launch_featmap_generic_t<__half>(a, st)
                                    : launch_featmap_generic_t<float>(a, st);
}

// =====================================================================================
// Fused step kernel: one block of 256 threads per unit.
//
// Phase 1  scores s_j = q . K_j / sqrt(D) of the live slots and of the appended key, fp64.
//          A cache row is D * sizeof(T) bytes = LPR lanes of 16 bytes; the block reads
//          256 / LPR rows per iteration with fully coalesced 16-byte loads.
// Phase 2  one thread per row: shift, exponentials, denominator of Eq. 3 including
//          phi(q) z^T, probabilities, H2O score accumulation, eviction argmin.
// Phase 3  p . V in fp32 with the same row mapping as phase 1.
// Phase 4  one thread per column: out = p V + phi(q) H / den (Eq. 3), H += psi_e^T v_e,
//          z += psi_e (Eq. 4, Eq. 5), new pair written into the freed slot.
// =====================================================================================
template <typename T, int D>
__global__ __launch_bounds__(256) void step_kernel(const StepArgs a)
{
  constexpr int kThreads = 256, kWaves = kThreads / kWave;
  constexpr int EPL = Store<T>::kPerVec;   // elements per lane
  constexpr int LPR = D / EPL;             // lanes per row
  constexpr int RPB = kThreads / LPR;      // rows per block iteration
  static_assert(LPR >= 8 && LPR <= 32, "row must span 8..32 lanes");

  extern __shared__ double dyn[];
  const int C = a.C;
  double *s_sc = dyn;                                        // [C+1] scores, then e_j, then new acc
  float *s_p = reinterpret_cast<float *>(dyn + (C + 1));     // [C+1] probabilities (fp32)
  __shared__ double s_red[kWaves];
  __shared__ Cand s_cand[kWaves];
  __shared__ float s_o[kWaves][D];
  __shared__ float s_psie[LESSDEC_MAX_RANK];

  const int u = blockIdx.x;
  const int tid = threadIdx.x;
  const int lr = tid % LPR, rb = tid / LPR;
  const int R = a.R;
  const int n = a.n_seen[u];
  const int m = n < C ? n : C;          // live slots are 0..m-1 (slots fill in order)
  const int rows = m + 1;               // + the appended pair (K', V' of Eq. 3)
  const bool full = (m == C);

  const T *kc = reinterpret_cast<const T *>(a.k_cache) + (size_t)u * C * D;
  const T *vc = reinterpret_cast<const T *>(a.v_cache) + (size_t)u * C * D;
  const T *qn = reinterpret_cast<const T *>(a.q) + (size_t)u * D;
  const T *kn = reinterpret_cast<const T *>(a.k) + (size_t)u * D;
  const T *vn = reinterpret_cast<const T *>(a.v) + (size_t)u * D;

  // ---- phase 1: scores ---------------------------------------------------------------
  {
    double qd[EPL];
    auto qv = load_vec<T>(qn + lr * EPL);
#pragma unroll
    for (int i = 0; i < EPL; ++i) qd[i] = (double)Store<T>::get(qv, i);
    const double sqrt_d = sqrt((double)D);
    for (int r = rb; r < rows; r += RPB) {
      const T *src = (r < m) ? kc + (size_t)r * D : kn;
      auto kv = load_vec<T>(src + lr * EPL);
      double part = 0.0;
#pragma unroll
      for (int i = 0; i < EPL; ++i) part = fma(qd[i], (double)Store<T>::get(kv, i), part);
#pragma unroll
      for (int o = LPR / 2; o > 0; o >>= 1) part += __shfl_xor(part, o);
      if (lr == 0) s_sc[r] = part / sqrt_d;
    }
  }
  __syncthreads();

  // ---- phase 2: softmax pieces, H2O accumulation, eviction choice ----------------------
  double lmax = -__builtin_inf();
  for (int j = tid; j < rows; j += kThreads) lmax = fmax(lmax, s_sc[j]);
  const double M = block_max<kWaves>(lmax, s_red);

  double lsum = 0.0;
  for (int j = tid; j < rows; j += kThreads) {
    double e = exp(s_sc[j] - M);
    s_sc[j] = e;
    lsum += e;
  }
  const double S = block_sum<kWaves>(lsum, s_red);       // sparse part of the denominator, shifted

  double fz = 0.0;                                        // phi(q) z^T
  for (int r = 0; r < R; ++r) fz = fma(a.f_phi[(size_t)u * R + r], a.z[(size_t)u * R + r], fz);

  // den = phi(q) z^T + sum_j e^{s_j}; evaluated in whichever scaling cannot overflow:
  //   M > 0 (or no low-rank term): everything times e^{-M}
  //   M <= 0 with a low-rank term: unscaled, e^{M} <= 1
  double pscale, lscale;
  if (fz > 0.0 && M <= 0.0) {
    const double w = exp(M);
    const double den = fz + w * S;
    pscale = w / den;
    lscale = 1.0 / den;
  } else {
    const double eM = (fz > 0.0) ? exp(-M) : 0.0;
    const double den = fz * eM + S;
    pscale = 1.0 / den;
    lscale = eM / den;
  }
  const double ascale = (a.flags & LESSDEC_FLAG_SPARSE_DENOM) ? 1.0 / S : pscale;

  Cand best = cand_none();
  for (int j = tid; j < rows; j += kThreads) {
    const double e = s_sc[j];
    s_p[j] = (float)(e * pscale);
    double na = e * ascale;
    int pj = n;
    if (j < m) {
      na += a.acc[(size_t)u * C + j];
      pj = a.pos[(size_t)u * C + j];
    }
    s_sc[j] = na;
    if (full) {
      const bool is_cand = (j < m) ? (pj <= n - a.Nr) : (a.Nr == 0);
      Cand c{na, pj, j};
      if (is_cand && cand_less(c, best)) best = c;
    }
  }
  const Cand ev = block_argmin<kWaves>(best, s_cand);      // its barriers also publish s_sc / s_p
  const int eslot = full ? ev.slot : -1;                   // m means: the new pair itself
  const bool evict = full && eslot >= 0;
  const int ins_slot = full ? ((eslot >= 0 && eslot < m) ? eslot : -1) : m;

  // ---- phase 3: p . V, and staging of the discarded pair's psi --------------------------
  if (evict && tid < R)
    s_psie[tid] = (eslot < m) ? a.psi[((size_t)u * C + eslot) * R + tid] : a.psi_new[(size_t)u * R + tid];
  {
    float o[EPL];
#pragma unroll
    for (int i = 0; i < EPL; ++i) o[i] = 0.f;
    for (int r = rb; r < rows; r += RPB) {
      const T *src = (r < m) ? vc + (size_t)r * D : vn;
      auto vv = load_vec<T>(src + lr * EPL);
      const float p = s_p[r];
#pragma unroll
      for (int i = 0; i < EPL; ++i) o[i] = fmaf(p, Store<T>::get(vv, i), o[i]);
    }
    // rows of one wave: lanes lr, lr + LPR, ... hold the same columns
#pragma unroll
    for (int i = 0; i < EPL; ++i) {
#pragma unroll
      for (int off = LPR; off < kWave; off <<= 1) o[i] += __shfl_xor(o[i], off);
    }
    if ((tid & (kWave - 1)) < LPR) {
#pragma unroll
      for (int i = 0; i < EPL; ++i) s_o[tid / kWave][lr * EPL + i] = o[i];
    }
  }
  __syncthreads();

  // ---- phase 4: output, state update, in-place insert -----------------------------------
  if (tid < D) {
    const int c = tid;
    float pv = 0.f;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) pv += s_o[w][c];
    float *Hu = a.H + (size_t)u * R * D;
    float fh = 0.f;
    for (int r = 0; r < R; ++r) fh = fmaf((float)a.f_phi[(size_t)u * R + r], Hu[(size_t)r * D + c], fh);
    const double o = (double)pv + lscale * (double)fh;
    reinterpret_cast<T *>(a.out)[(size_t)u * D + c] = Store<T>::from_float((float)o);

    if (evict) {
      const float ve = (eslot < m) ? Store<T>::to_float(vc[(size_t)eslot * D + c])
                                   : Store<T>::to_float(vn[c]);
      for (int r = 0; r < R; ++r) Hu[(size_t)r * D + c] = fmaf(s_psie[r], ve, Hu[(size_t)r * D + c]);
      if (c < R) a.z[(size_t)u * R + c] += (double)s_psie[c];
    }
    if (ins_slot >= 0) {
      T *kw = reinterpret_cast<T *>(a.k_cache) + ((size_t)u * C + ins_slot) * D;
      T *vw = reinterpret_cast<T *>(a.v_cache) + ((size_t)u * C + ins_slot) * D;
      kw[c] = kn[c];
      vw[c] = vn[c];
      if (c < R) a.psi[((size_t)u * C + ins_slot) * R + c] = a.psi_new[(size_t)u * R + c];
    }
  }
  // accumulated scores and positions
  for (int j = tid; j < rows; j += kThreads) {
    if (j < m) {
      if (j != ins_slot) a.acc[(size_t)u * C + j] = s_sc[j];
    } else {
      int old = -1;
      if (evict) old = (eslot < m) ? a.pos[(size_t)u * C + eslot] : n;
      if (ins_slot >= 0) {
        a.acc[(size_t)u * C + ins_slot] = s_sc[m];
        a.pos[(size_t)u * C + ins_slot] = n;
      }
      if (a.evicted_pos) a.evicted_pos[u] = old;
      a.n_seen[u] = n + 1;
    }
  }
}

template <typename T, int D>
static hipError_t launch_step_t(const StepArgs &a, int units, hipStream_t st)
{
  size_t lds = (size_t)(a.C + 1) * (sizeof(double) + sizeof(float));
  step_kernel<T, D><<<units, 256, lds, st>>>(a);
  return hipGetLastError();
}

hipError_t launch_step(const StepArgs &a, int units, int dtype, int D, hipStream_t st)
{
  if (dtype == LESSDEC_DTYPE_F16) {
    return D == 128 ? launch_step_t<__half, 128>(a, units, st) : launch_step_t<__half, 64>(a, units, st);
  }
  return D == 128 ? launch_step_t<float, 128>(a, units, st) : launch_step_t<float, 64>(a, units, st);
}

// =====================================================================================
// Reset: H = 0, z = 0, acc = 0, psi = 0, pos = -1, n_seen = 0 (fill kernels, so the call
// can be recorded into a HIP graph).
// =====================================================================================
__global__ void reset_kernel(float *H, size_t nH, double *z, size_t nz, double *acc, size_t nacc,
                             int32_t *pos, size_t npos, float *psi, size_t npsi, int32_t *n_seen,
                             size_t nn)
{
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  const size_t t0 = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  for (size_t i = t0; i < nH; i += stride) H[i] = 0.f;
  for (size_t i = t0; i < nz; i += stride) z[i] = 0.0;
  for (size_t i = t0; i < nacc; i += stride) acc[i] = 0.0;
  for (size_t i = t0; i < npos; i += stride) pos[i] = -1;
  for (size_t i = t0; i < npsi; i += stride) psi[i] = 0.f;
  for (size_t i = t0; i < nn; i += stride) n_seen[i] = 0;
}

hipError_t launch_reset(const lessdec_desc *d, hipStream_t st)
{
  const size_t U = (size_t)d->batch * d->heads, C = (size_t)d->n_heavy + d->n_recent;
  const size_t R = d->rank, D = d->head_dim;
  reset_kernel<<<1024, 256, 0, st>>>(d->H, U * R * D, d->z, U * R, d->acc, U * C, d->pos, U * C,
                                     d->psi, U * C * R, d->n_seen, U);
  return hipGetLastError();
}

}  // namespace lessdec
