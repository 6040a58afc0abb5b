// Decode step (Algorithm 1) for several query heads per key/value head (multi-query and
// grouped-query attention; Sec. 3.2, "Inexpensive Training", extends H2O to the attention
// scores of all query heads).  The G query heads of a unit share its sparse cache and its state
// H, z (psi acts on keys); each has its own phi and its own Eq. 3; a pair's accumulated score
// grows by its probability under every head.
//
// First form of this path: one block of 256 threads per unit, the heads one after the other,
// all arithmetic fp64 in the order of the equations, cache rows read straight from memory.
// It folds the discarded pair into H, z within the step (nothing is left pending).
#include "lessdec_wave.h"

namespace lessdec {

namespace {

// all-reduce over the block's four waves: within a wave by lane exchange, across waves through
// four LDS words, combined in wave order
template <typename Op>
__device__ inline double block_allreduce(double v, double *s_red, int tid, Op op)
{
  v = wave_allreduce(v, op);
  if (tid % kWave == 0) s_red[tid / kWave] = v;
  __syncthreads();
  const double r = op(op(op(s_red[0], s_red[1]), s_red[2]), s_red[3]);
  __syncthreads();
  return r;
}

}  // namespace

// q, out: [U,G,D]; k, v: [U,D]; f_phi [U,G,R] fp64 or f_phi32 in fp32; f_psi: [U,R] fp32.
// grid = U, block = 256, dynamic LDS: see launch_step_gqa_t.
// After the last head: accumulated scores, eviction choice, fold of the discarded pair into
// H, z (Eq. 4, Eq. 5), in-place insert of the new pair (Sec. 3.2).  s_inc holds the step's
// probabilities per pair summed over the heads; s_e is scratch of the same size.
template <typename T, int D>
__device__ inline void gqa_finish_unit(const StepArgs &a, int u, int tid, double *s_e, const double *s_inc,
                                       Cand *s_cand)
{
  const int C = a.C, R = a.R;
  const int n = a.n_seen[u];
  const int m = n < C ? n : C;
  const int rows = m + 1;
  const bool full = (m == C);
  T *kc = reinterpret_cast<T *>(a.k_cache) + (size_t)u * C * D;
  T *vc = reinterpret_cast<T *>(a.v_cache) + (size_t)u * C * D;
  const T *kn = reinterpret_cast<const T *>(a.k) + (size_t)u * D;
  const T *vn = reinterpret_cast<const T *>(a.v) + (size_t)u * D;
  float *Hu = a.H + (size_t)u * R * D;
  double *zu = a.z + (size_t)u * R;
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

// STAGE: the unit's key and value rows (and H, z) are copied into the LDS once and every head
// works from there; without it each head reads them from memory again (any capacity).
template <typename T, int D, bool STAGE>
__global__ __launch_bounds__(256) void gqa_step_kernel(const StepArgs a, int G, int nhb)
{
  extern __shared__ double dyn[];
  __shared__ double s_red[4];
  __shared__ Cand s_cand[256];
  __shared__ double s_num[256];
  constexpr int EPL = Store<T>::kPerVec, LPR = D / EPL, RPB = 256 / LPR;   // lanes per row, rows per pass
  using Vec = typename Store<T>::Vec;
  // nhb blocks per unit, each with a contiguous share of the unit's heads
  const int u = (int)blockIdx.x / nhb, hb = (int)blockIdx.x % nhb, tid = threadIdx.x;
  const int g_begin = (int)((long)G * hb / nhb), g_end = (int)((long)G * (hb + 1) / nhb);
  const int lr = tid % LPR, rb = tid / LPR;
  const int C = a.C, R = a.R;
  const int rows_cap = C + 2;
  double *s_e = dyn;                       // [C+1] scores, then e^{s - m*}, then the new accumulated scores
  double *s_inc = dyn + rows_cap;          // [C+1] this step's probabilities per pair, summed over the heads
  double *s_q = s_inc + rows_cap;          // [D] the head's query
  double *s_f = s_q + D;                   // [R] the head's phi(q)
  double *s_z = s_f + 64;                  // [R] z
  float *s_H = reinterpret_cast<float *>(s_z + 64);                    // STAGE: [R,D]
  T *s_k = reinterpret_cast<T *>(s_H + (STAGE ? R * D : 0));          // STAGE: [C+1,D] keys, the appended one last
  T *s_v = s_k + (STAGE ? (size_t)(C + 1) * D : 0);                    // STAGE: [C+1,D] values

  const int n = a.n_seen[u];
  const int m = n < C ? n : C;             // live slots are 0..m-1 (slots fill in order)
  const int rows = m + 1;                  // + the appended pair (K', V' of Eq. 3)
  T *kc = reinterpret_cast<T *>(a.k_cache) + (size_t)u * C * D;
  T *vc = reinterpret_cast<T *>(a.v_cache) + (size_t)u * C * D;
  const T *kn = reinterpret_cast<const T *>(a.k) + (size_t)u * D;
  const T *vn = reinterpret_cast<const T *>(a.v) + (size_t)u * D;
  float *Hu = a.H + (size_t)u * R * D;
  double *zu = a.z + (size_t)u * R;
  const double sqrt_d = sqrt((double)D);

  for (int r = tid; r < rows; r += 256) s_inc[r] = 0.0;
  if (tid < R) s_z[tid] = zu[tid];
  if constexpr (STAGE) {
    constexpr int VPR = D / EPL;                             // 16-byte vectors per row
    for (int i = tid; i < rows * VPR; i += 256) {
      const int r = i / VPR, c = i % VPR;
      reinterpret_cast<Vec *>(s_k)[i] = load_vec<T>((r < m ? kc + (size_t)r * D : kn) + c * EPL);
      reinterpret_cast<Vec *>(s_v)[i] = load_vec<T>((r < m ? vc + (size_t)r * D : vn) + c * EPL);
    }
    for (int i = tid; i < R * D; i += 256) s_H[i] = Hu[i];
  }

  // a head's query element and phi entry of this thread, requested one head ahead
  auto fetch_q = [&](int g) -> double {
    return tid < D ? (double)Store<T>::to_float(reinterpret_cast<const T *>(a.q)[((size_t)u * G + g) * D + tid]) : 0.0;
  };
  auto fetch_f = [&](int g) -> double {
    if (tid >= R) return 0.0;
    const size_t i = ((size_t)u * G + g) * R + tid;
    return a.f_phi32 ? (double)a.f_phi32[i] : a.f_phi[i];
  };
  double q_next = fetch_q(g_begin), f_next = fetch_f(g_begin);
  const double inv_sqrt_d = 1.0 / sqrt_d;
  for (int g = g_begin; g < g_end; ++g) {
    __syncthreads();
    if (tid < D) s_q[tid] = q_next;
    if (tid < R) s_f[tid] = f_next;
    if (g + 1 < g_end) {
      q_next = fetch_q(g + 1);
      f_next = fetch_f(g + 1);
    }
    __syncthreads();
    double qreg[EPL];                                        // this lane's share of the query
#pragma unroll
    for (int i = 0; i < EPL; ++i) qreg[i] = s_q[lr * EPL + i];
    // scores against the cached keys and the appended key: LPR lanes of 16 bytes per row; the
    // rows of the first NP passes are requested together, further passes one at a time
    double mx = -__builtin_inf();
    auto row_ptr = [&](int r) -> const T * {
      const int rc = r < rows ? r : rows - 1;
      if constexpr (STAGE) return s_k + (size_t)rc * D + lr * EPL;
      return (rc < m ? kc + (size_t)rc * D : kn) + lr * EPL;
    };
    auto score = [&](int r, const Vec &kv) {
      double acc = 0.0;
#pragma unroll
      for (int i = 0; i < EPL; ++i) acc = fma(qreg[i], (double)Store<T>::get(kv, i), acc);
      acc = row_sum<LPR>(acc);
      const double s = acc * inv_sqrt_d;
      if (lr == 0 && r < rows) s_e[r] = s;
      if (r < rows) mx = fmax(mx, s);
    };
    constexpr int NP = 8;
    Vec kvs[NP];
#pragma unroll
    for (int p = 0; p < NP; ++p) kvs[p] = load_vec<T>(row_ptr(p * RPB + rb));   // clamped: always in range
#pragma unroll
    for (int p = 0; p < NP; ++p)
      if (p * RPB < rows) score(p * RPB + rb, kvs[p]);
    for (int r0 = NP * RPB; r0 < rows; r0 += RPB) score(r0 + rb, load_vec<T>(row_ptr(r0 + rb)));
    mx = block_allreduce(mx, s_red, tid, OpMax{});
    // phi(q) z^T and the common shift m* = max(scores, ln(phi(q) z^T)) (Eq. 3 times e^{-m*})
    double fz = 0.0;
    for (int r = 0; r < R; ++r) fz = fma(s_f[r], s_z[r], fz);
    const double lfz = fz > 0.0 ? log(fz) : -__builtin_inf();
    const double mstar = fmax(mx, lfz);
    const double wl = fz > 0.0 ? exp(lfz - mstar) : 0.0;
    double part = 0.0;
    for (int r = tid; r < rows; r += 256) {
      const double e = exp(s_e[r] - mstar);
      s_e[r] = e;
      part += e;
    }
    const double den = wl + block_allreduce(part, s_red, tid, OpAdd{});   // the barriers inside publish s_e
    // output column d: (phi(q) H e^{-m*} + sum_j e_j V_j) / den; the 256 / D thread groups
    // take the rows in turn and meet in the LDS
    {
      constexpr int NG = 256 / D;
      const int d = tid % D, grp = tid / D;
      double num = 0.0;
      if (grp == 0 && fz > 0.0) {
        double fh = 0.0;
        for (int r = 0; r < R; ++r) fh = fma(s_f[r], (double)(STAGE ? s_H[r * D + d] : Hu[(size_t)r * D + d]), fh);
        num = fh * exp(-mstar);
      }
      if constexpr (STAGE) {
#pragma unroll 8
        for (int r = grp; r < rows; r += NG) num = fma(s_e[r], (double)Store<T>::to_float(s_v[(size_t)r * D + d]), num);
      } else {
#pragma unroll 8
        for (int r = grp; r < m; r += NG) num = fma(s_e[r], (double)Store<T>::to_float(vc[(size_t)r * D + d]), num);
        if (grp == m % NG) num = fma(s_e[m], (double)Store<T>::to_float(vn[d]), num);
      }
      s_num[tid] = num;
      __syncthreads();
      if (tid < D) {
#pragma unroll
        for (int k = 1; k < NG; ++k) num += s_num[k * D + tid];
        reinterpret_cast<T *>(a.out)[((size_t)u * G + g) * D + tid] = Store<T>::from_float((float)(num / den));
      }
    }
    // this head's probabilities (H2O accumulates those of every head)
    const double dacc = (a.flags & LESSDEC_FLAG_SPARSE_DENOM) ? den - wl : den;
    for (int r = tid; r < rows; r += 256) s_inc[r] += s_e[r] / dacc;
  }
  __syncthreads();

  if (nhb > 1) {
    // the unit's heads are spread over nhb blocks: leave this block's sums for the finishing launch
    double *part = a.gqa_parts + ((size_t)u * nhb + hb) * rows_cap;
    for (int r = tid; r < rows; r += 256) part[r] = s_inc[r];
    return;
  }
  gqa_finish_unit<T, D>(a, u, tid, s_e, s_inc, s_cand);
}

// Finishing launch when a unit's heads were spread over several blocks: adds their sums in
// block order and finishes the unit.   grid = U, block = 256, dynamic LDS = 2 (C + 2) doubles.
template <typename T, int D>
__global__ __launch_bounds__(256) void gqa_finish_kernel(const StepArgs a, int nhb)
{
  extern __shared__ double dyn[];
  __shared__ Cand s_cand[256];
  const int u = (int)blockIdx.x, tid = threadIdx.x;
  const int rows_cap = a.C + 2;
  double *s_e = dyn, *s_inc = dyn + rows_cap;
  const int n = a.n_seen[u];
  const int rows = (n < a.C ? n : a.C) + 1;
  for (int r = tid; r < rows; r += 256) {
    double v = 0.0;
    for (int hb = 0; hb < nhb; ++hb) v += a.gqa_parts[((size_t)u * nhb + hb) * rows_cap + r];
    s_inc[r] = v;
  }
  __syncthreads();
  gqa_finish_unit<T, D>(a, u, tid, s_e, s_inc, s_cand);
}

// Blocks per unit: one when the units alone fill the chip, else the heads are spread over up
// to kGqaMaxHeadBlocks blocks (the cache rows are then staged once per block).
int gqa_head_blocks(long units, int G)
{
  int nhb = (int)((512 + units - 1) / units);          // measured: 512 units x 8 heads lose with a split
  if (nhb > kGqaMaxHeadBlocks) nhb = kGqaMaxHeadBlocks;
  if (nhb > G) nhb = G;
  return nhb < 1 ? 1 : nhb;
}

template <typename T, int D>
static hipError_t launch_step_gqa_t(const StepArgs &a, int G, hipStream_t st)
{
  const int nhb = gqa_head_blocks(a.U, G);
  const size_t base = (size_t)(2 * (a.C + 2) + D + 64 + 64) * sizeof(double);
  const size_t staged = base + (size_t)a.R * D * sizeof(float) + 2 * (size_t)(a.C + 1) * D * sizeof(T);
  if (staged <= 64 * 1024)
    gqa_step_kernel<T, D, true><<<a.U * nhb, 256, staged, st>>>(a, G, nhb);
  else
    gqa_step_kernel<T, D, false><<<a.U * nhb, 256, base, st>>>(a, G, nhb);
  if (nhb > 1) gqa_finish_kernel<T, D><<<a.U, 256, (size_t)2 * (a.C + 2) * sizeof(double), st>>>(a, nhb);
  return hipGetLastError();
}

hipError_t launch_step_gqa(const StepArgs &a, int G, int dtype, int D, hipStream_t st)
{
  if (dtype == LESSDEC_DTYPE_F16)
    return D == 128 ? launch_step_gqa_t<__half, 128>(a, G, st) : launch_step_gqa_t<__half, 64>(a, G, st);
  return D == 128 ? launch_step_gqa_t<float, 128>(a, G, st) : launch_step_gqa_t<float, 64>(a, G, st);
}

}  // namespace lessdec
