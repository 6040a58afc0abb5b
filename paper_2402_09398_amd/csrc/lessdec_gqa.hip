// Decode step (Algorithm 1) for several query heads per key/value head (multi-query and
// grouped-query attention; Sec. 3.2, "Inexpensive Training", extends H2O to the attention
// scores of all query heads).  The G query heads of a unit share its sparse cache and its state
// H, z (psi acts on keys); each has its own phi and its own Eq. 3; a pair's accumulated score
// grows by its probability under every head.
//
// First form of this path: one block of 256 threads per unit, the heads one after the other,
// all arithmetic fp64 in the order of the equations, cache rows read straight from memory.
// It folds the discarded pair into H, z within the step (nothing is left pending).
#include "lessdec_common.h"
#include "lessdec_internal.h"

namespace lessdec {

namespace {

__device__ inline double block_max(double v, double *s_red, int tid)
{
  s_red[tid] = v;
  __syncthreads();
  for (int o = 128; o > 0; o >>= 1) {
    if (tid < o) s_red[tid] = fmax(s_red[tid], s_red[tid + o]);
    __syncthreads();
  }
  const double r = s_red[0];
  __syncthreads();
  return r;
}
__device__ inline double block_sum(double v, double *s_red, int tid)
{
  s_red[tid] = v;
  __syncthreads();
  for (int o = 128; o > 0; o >>= 1) {
    if (tid < o) s_red[tid] += s_red[tid + o];
    __syncthreads();
  }
  const double r = s_red[0];
  __syncthreads();
  return r;
}

}  // namespace

// q, out: [U,G,D]; k, v: [U,D]; f_phi: [U,G,R] fp64; f_psi: [U,R] fp32.
// grid = U, block = 256, dynamic LDS = (2 (C + 2) + D + 64) doubles.
template <typename T, int D>
__global__ __launch_bounds__(256) void gqa_step_kernel(const StepArgs a, int G)
{
  extern __shared__ double dyn[];
  __shared__ double s_red[256];
  __shared__ Cand s_cand[256];
  const int u = (int)blockIdx.x, tid = threadIdx.x;
  const int C = a.C, R = a.R;
  const int rows_cap = C + 2;
  double *s_e = dyn;                       // [C+1] scores, then e^{s - m*}, then the new accumulated scores
  double *s_inc = dyn + rows_cap;          // [C+1] this step's probabilities per pair, summed over the heads
  double *s_q = s_inc + rows_cap;          // [D] the head's query
  double *s_f = s_q + D;                   // [R] the head's phi(q)

  const int n = a.n_seen[u];
  const int m = n < C ? n : C;             // live slots are 0..m-1 (slots fill in order)
  const int rows = m + 1;                  // + the appended pair (K', V' of Eq. 3)
  const bool full = (m == C);
  T *kc = reinterpret_cast<T *>(a.k_cache) + (size_t)u * C * D;
  T *vc = reinterpret_cast<T *>(a.v_cache) + (size_t)u * C * D;
  const T *kn = reinterpret_cast<const T *>(a.k) + (size_t)u * D;
  const T *vn = reinterpret_cast<const T *>(a.v) + (size_t)u * D;
  float *Hu = a.H + (size_t)u * R * D;
  double *zu = a.z + (size_t)u * R;
  const double sqrt_d = sqrt((double)D);

  for (int r = tid; r < rows; r += 256) s_inc[r] = 0.0;

  for (int g = 0; g < G; ++g) {
    const T *qg = reinterpret_cast<const T *>(a.q) + ((size_t)u * G + g) * D;
    __syncthreads();
    if (tid < D) s_q[tid] = (double)Store<T>::to_float(qg[tid]);
    if (tid < R) s_f[tid] = a.f_phi[((size_t)u * G + g) * R + tid];
    __syncthreads();
    // scores against the cached keys and the appended key
    double mx = -__builtin_inf();
    for (int r = tid; r < rows; r += 256) {
      const T *row = r < m ? kc + (size_t)r * D : kn;
      double acc = 0.0;
      for (int d = 0; d < D; ++d) acc = fma(s_q[d], (double)Store<T>::to_float(row[d]), acc);
      const double s = acc / sqrt_d;
      s_e[r] = s;
      mx = fmax(mx, s);
    }
    mx = block_max(mx, s_red, tid);
    // phi(q) z^T and the common shift m* = max(scores, ln(phi(q) z^T)) (Eq. 3 times e^{-m*})
    double fz = 0.0;
    for (int r = 0; r < R; ++r) fz = fma(s_f[r], zu[r], fz);
    const double lfz = fz > 0.0 ? log(fz) : -__builtin_inf();
    const double mstar = fmax(mx, lfz);
    const double wl = fz > 0.0 ? exp(lfz - mstar) : 0.0;
    double part = 0.0;
    for (int r = tid; r < rows; r += 256) {
      const double e = exp(s_e[r] - mstar);
      s_e[r] = e;
      part += e;
    }
    const double den = wl + block_sum(part, s_red, tid);   // the barriers inside publish s_e
    // output column d: (phi(q) H e^{-m*} + sum_j e_j V_j) / den
    if (tid < D) {
      double num = 0.0;
      if (fz > 0.0) {
        double fh = 0.0;
        for (int r = 0; r < R; ++r) fh = fma(s_f[r], (double)Hu[(size_t)r * D + tid], fh);
        num = fh * exp(-mstar);
      }
      for (int r = 0; r < m; ++r) num = fma(s_e[r], (double)Store<T>::to_float(vc[(size_t)r * D + tid]), num);
      num = fma(s_e[m], (double)Store<T>::to_float(vn[tid]), num);
      reinterpret_cast<T *>(a.out)[((size_t)u * G + g) * D + tid] = Store<T>::from_float((float)(num / den));
    }
    // this head's probabilities (H2O accumulates those of every head)
    const double dacc = (a.flags & LESSDEC_FLAG_SPARSE_DENOM) ? den - wl : den;
    for (int r = tid; r < rows; r += 256) s_inc[r] += s_e[r] / dacc;
  }
  __syncthreads();

  // accumulated scores; eviction candidate of this thread's rows
  const bool lambda = (a.flags & LESSDEC_FLAG_LAMBDA) != 0;
  Cand best = cand_none();
  for (int r = tid; r < rows; r += 256) {
    double na = s_inc[r];
    int pj = n;
    if (r < m) {
      na += a.acc[(size_t)u * C + r];
      pj = a.pos[(size_t)u * C + r];
    }
    s_e[r] = na;
    if (full) {
      const bool is_cand = (r < m) ? (pj <= n - a.Nr && (!lambda || pj >= a.Nh)) : (a.Nr == 0);
      const Cand cnd{lambda ? 0.0 : na, pj, r};
      if (is_cand && cand_less(cnd, best)) best = cnd;
    }
  }
  s_cand[tid] = best;
  __syncthreads();
  for (int o = 128; o > 0; o >>= 1) {
    if (tid < o && cand_less(s_cand[tid + o], s_cand[tid])) s_cand[tid] = s_cand[tid + o];
    __syncthreads();
  }
  const Cand win = s_cand[0];
  const int eslot = full ? win.slot : -1;                    // eslot == m: the new pair itself
  const bool evict = eslot >= 0;
  const int ins_slot = full ? ((evict && eslot < m) ? eslot : -1) : m;

  // fold of the discarded pair into H, z (Eq. 4, Eq. 5), before its row is overwritten
  if (evict) {
    const float *pe = eslot < m ? a.psi + ((size_t)u * C + eslot) * R : a.f_psi + (size_t)u * R;
    if (tid < D) {
      const double ve = (double)Store<T>::to_float(eslot < m ? vc[(size_t)eslot * D + tid] : vn[tid]);
      for (int r = 0; r < R; ++r)
        Hu[(size_t)r * D + tid] = (float)fma((double)pe[r], ve, (double)Hu[(size_t)r * D + tid]);
    } else if (tid - D < R) {
      zu[tid - D] += (double)pe[tid - D];
    }
  }
  __syncthreads();
  // scores of the pairs that stay, and the new pair into its slot (Sec. 3.2: in place)
  for (int r = tid; r < m; r += 256)
    if (r != ins_slot) a.acc[(size_t)u * C + r] = s_e[r];
  if (ins_slot >= 0) {
    if (tid < D) {
      kc[(size_t)ins_slot * D + tid] = kn[tid];
      vc[(size_t)ins_slot * D + tid] = vn[tid];
    }
    if (tid < R) a.psi[((size_t)u * C + ins_slot) * R + tid] = a.f_psi[(size_t)u * R + tid];
    if (tid == 0) {
      a.acc[(size_t)u * C + ins_slot] = s_e[m];
      a.pos[(size_t)u * C + ins_slot] = n;
    }
  }
  if (tid == 0) {
    a.n_seen[u] = n + 1;
    a.pend_slot[u] = -1;
    if (a.evicted_pos) a.evicted_pos[u] = evict ? win.pos : -1;
  }
}

hipError_t launch_step_gqa(const StepArgs &a, int G, int dtype, int D, hipStream_t st)
{
  const size_t lds = (size_t)(2 * (a.C + 2) + D + 64) * sizeof(double);
  if (dtype == LESSDEC_DTYPE_F16) {
    if (D == 128) gqa_step_kernel<__half, 128><<<a.U, 256, lds, st>>>(a, G);
    else gqa_step_kernel<__half, 64><<<a.U, 256, lds, st>>>(a, G);
  } else {
    if (D == 128) gqa_step_kernel<float, 128><<<a.U, 256, lds, st>>>(a, G);
    else gqa_step_kernel<float, 64><<<a.U, 256, lds, st>>>(a, G);
  }
  return hipGetLastError();
}

}  // namespace lessdec
