// Decode step (Algorithm 1) for several query heads per key/value head (multi-query and
// grouped-query attention; Sec. 3.2, "Inexpensive Training", extends H2O to the attention
// scores of all query heads).  The G query heads of a unit share its sparse cache and its state
// H, z (psi acts on keys); each has its own phi and its own Eq. 3; a pair's accumulated score
// grows by its probability under every head.
//
// One block of 256 threads per unit (or per share of a unit's heads), all arithmetic fp64 in the
// order of the equations, the heads four at a time; a block first copies its unit's rows into the
// LDS when they fit.  The discarded pair is folded into H, z within the step (nothing is left
// pending).
#include "lessdec_wave.h"

namespace lessdec {

namespace {

// four adjacent stored elements (8 or 16 bytes, aligned) as floats, and back
template <typename T> __device__ inline void load_four(const T *p, float (&v)[4]);
template <> __device__ inline void load_four<float>(const float *p, float (&v)[4])
{
  const float4 x = *reinterpret_cast<const float4 *>(p);
  v[0] = x.x; v[1] = x.y; v[2] = x.z; v[3] = x.w;
}
template <> __device__ inline void load_four<__half>(const __half *p, float (&v)[4])
{
  const uint2 x = *reinterpret_cast<const uint2 *>(p);
  const __half2 lo = *reinterpret_cast<const __half2 *>(&x.x), hi = *reinterpret_cast<const __half2 *>(&x.y);
  v[0] = __low2float(lo); v[1] = __high2float(lo); v[2] = __low2float(hi); v[3] = __high2float(hi);
}
template <typename T> __device__ inline void store_four(T *p, const float (&v)[4]);
template <> __device__ inline void store_four<float>(float *p, const float (&v)[4])
{
  *reinterpret_cast<float4 *>(p) = make_float4(v[0], v[1], v[2], v[3]);
}
template <> __device__ inline void store_four<__half>(__half *p, const float (&v)[4])
{
  const __half2 lo = __halves2half2(__float2half(v[0]), __float2half(v[1]));
  const __half2 hi = __halves2half2(__float2half(v[2]), __float2half(v[3]));
  uint2 x;
  x.x = *reinterpret_cast<const unsigned *>(&lo);
  x.y = *reinterpret_cast<const unsigned *>(&hi);
  *reinterpret_cast<uint2 *>(p) = x;
}

}  // namespace

// Layouts of this file's kernels: q, out [U,G,D]; k, v [U,D]; f_phi [U,G,R] fp64 or f_phi32 in
// fp32; f_psi [U,R] fp32.

// LDS copies of a unit's rows as they were before the step (H before the fold), for
// gqa_finish_unit; every null member is read from memory instead.
template <typename T>
struct LdsCopies {
  const T *k = nullptr, *v = nullptr;      // [m+1, D] rows in slot order, the appended pair last
  const float *H = nullptr;                // [R, D]
  const double *acc = nullptr;             // [m]
  const int *pos = nullptr;                // [m]
};

// After the unit's last head, by the whole block of 256 threads: accumulated scores, eviction
// choice, fold of the discarded pair into H, z (Eq. 4, Eq. 5), in-place insert of the new pair
// (Sec. 3.2).  s_inc holds the step's probabilities per pair summed over the heads; s_e is
// scratch of the same size; s_cand 256 entries.
template <typename T, int D>
__device__ inline void gqa_finish_unit(const StepArgs &a, int u, int tid, double *s_e, const double *s_inc,
                                       Cand *s_cand, const LdsCopies<T> lds = LdsCopies<T>())
{
  const int C = a.C, R = a.R;
  const int n = sane_n_seen(a.n_seen[u]);
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
      na += lds.acc ? lds.acc[r] : a.acc[(size_t)u * C + r];
      pj = lds.pos ? lds.pos[r] : a.pos[(size_t)u * C + r];
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

  // fold of the discarded pair into H, z (Eq. 4, Eq. 5), before its row is overwritten; the
  // pair's psi goes through the LDS and H's column is requested eight rows at a time
  if (evict) {
    const float *pe = eslot < m ? a.psi + ((size_t)u * C + eslot) * R : a.f_psi + (size_t)u * R;
    float *s_pe = reinterpret_cast<float *>(s_cand + 1);     // s_cand[0] has been read; [1..] is free
    double ve = 0.0;
    if (tid < D)
      ve = (double)Store<T>::to_float(lds.v ? lds.v[(size_t)eslot * D + tid]
                                            : (eslot < m ? vc[(size_t)eslot * D + tid] : vn[tid]));
    if (tid < R) s_pe[tid] = pe[tid];
    __syncthreads();
    if (tid < D) {
      for (int r0 = 0; r0 < R; r0 += 8) {
        float h[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) h[j] = (lds.H ? lds.H : Hu)[(size_t)(r0 + j < R ? r0 + j : R - 1) * D + tid];
#pragma unroll
        for (int j = 0; j < 8; ++j)
          if (r0 + j < R) Hu[(size_t)(r0 + j) * D + tid] = (float)fma((double)s_pe[r0 + j], ve, (double)h[j]);
      }
    } else if (tid - D < R) {
      zu[tid - D] += (double)s_pe[tid - D];
    }
  }
  __syncthreads();
  // scores of the pairs that stay, and the new pair into its slot (Sec. 3.2: in place)
  for (int r = tid; r < m; r += 256)
    if (r != ins_slot) a.acc[(size_t)u * C + r] = s_e[r];
  if (ins_slot >= 0) {
    if (tid < D) {
      kc[(size_t)ins_slot * D + tid] = lds.k ? lds.k[(size_t)m * D + tid] : kn[tid];
      vc[(size_t)ins_slot * D + tid] = lds.v ? lds.v[(size_t)m * D + tid] : vn[tid];
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

// The heads of a unit (or of a block's share of them) are taken four at a time (kGqaChunk = the
// block's four waves).  Per chunk: every thread scores its 16-byte share of a key row against
// the four queries; wave w then does the softmax of head w by itself (maximum, Eq. 3's low-rank
// denominator term, exponentials, their sum) with lane exchanges only, and the head's output the
// same way.  Four barriers per chunk.
// STAGE: the unit's key and value rows, H, the scores and positions are copied into the LDS
// once and every chunk works from there.  Without it (rows too many for the LDS) they are read
// from memory where they are used, the first passes of a sweep requested together.
// Dynamic LDS: see gqa_chunk_lds.
constexpr int kGqaChunk = 4;

template <typename T, int D, bool STAGE>
__global__ __launch_bounds__(256) void gqa_chunk_kernel(const StepArgs a, int G, int nhb)
{
  extern __shared__ double dyn[];
  constexpr int GC = kGqaChunk;
  constexpr int EPL = Store<T>::kPerVec, LPR = D / EPL, RPB = 256 / LPR;   // lanes per row, rows per pass
  constexpr int NQ = GC * D / 256;                                         // query elements per thread and chunk
  static_assert(NQ >= 1 && GC == 256 / kWave, "head_dim 64 or 128; one wave per head of a chunk");
  using Vec = typename Store<T>::Vec;
  const int u = (int)blockIdx.x / nhb, hb = (int)blockIdx.x % nhb, tid = threadIdx.x;
  const int g_begin = (int)((long)G * hb / nhb), g_end = (int)((long)G * (hb + 1) / nhb);
  const int lr = tid % LPR, rb = tid / LPR, lane = tid % kWave, w = tid / kWave;
  const int C = a.C, R = a.R;
  const int rows_cap = C + 2;                        // stride of the partial sums in the workspace
  const int ecap = (C + 3) & ~1;                     // LDS stride of a head's scores: even, so that all arrays stay 16-byte aligned
  double *s_e = dyn;                                 // [GC][ecap] scores, then e^{s - m*}
  double *s_inc = s_e + GC * ecap;               // [ecap] this step's probabilities per pair, summed over the heads
  double *s_q = s_inc + ecap;                    // [GC][D] queries of the chunk
  double *s_f = s_q + GC * D;                        // [GC][64] phi(q) of the chunk
  double *s_z = s_f + GC * 64;                       // [64] z
  double *s_hd = s_z + 64;                           // [GC][4] per head: e^{-m*} (0 without a state term), 1/den, 1/dacc
  double *s_acc = s_hd + GC * 4;                     // [C rounded up to 2] accumulated scores before the step
  int *s_pos = reinterpret_cast<int *>(s_acc + (C + 1) / 2 * 2);   // [C rounded up to 4] positions; 16-byte steps
  float *s_H = reinterpret_cast<float *>(s_pos + (C + 3) / 4 * 4);   // [R,D]
  T *s_k = reinterpret_cast<T *>(s_H + R * D);                  // [C+1,D] keys, the appended one last
  T *s_v = s_k + (size_t)(C + 1) * D;                           // [C+1,D] values
  Cand *s_cand = reinterpret_cast<Cand *>(s_q);                 // after the last chunk (256 entries fit in s_q, s_f)
  static_assert(sizeof(Cand) * 256 <= (GC * D + GC * 64) * sizeof(double), "candidates overlay the query area");

  const int n = sane_n_seen(a.n_seen[u]);
  const int m = n < C ? n : C;             // live slots are 0..m-1 (slots fill in order)
  const int rows = m + 1;                  // + the appended pair (K', V' of Eq. 3)
  const T *kc = reinterpret_cast<const T *>(a.k_cache) + (size_t)u * C * D;
  const T *vc = reinterpret_cast<const T *>(a.v_cache) + (size_t)u * C * D;
  const T *kn = reinterpret_cast<const T *>(a.k) + (size_t)u * D;
  const T *vn = reinterpret_cast<const T *>(a.v) + (size_t)u * D;
  const float *Hu = a.H + (size_t)u * R * D;

  // a chunk's query elements and phi entry of this thread, requested one chunk ahead; heads past
  // the block's share repeat its last one (computed, never stored)
  auto head_of = [&](int g0, int i) { return g0 + i < g_end ? g0 + i : g_end - 1; };
  auto fetch_q = [&](int g0, int j) -> double {
    const int e = j * 256 + tid, g = head_of(g0, e / D);
    return (double)Store<T>::to_float(reinterpret_cast<const T *>(a.q)[((size_t)u * G + g) * D + e % D]);
  };
  auto fetch_f = [&](int g0) -> double {
    if (tid >= GC * R) return 0.0;
    const size_t i = ((size_t)u * G + head_of(g0, tid / R)) * R + tid % R;
    return a.f_phi32 ? (double)a.f_phi32[i] : a.f_phi[i];
  };
  double q_next[NQ], f_next;
#pragma unroll
  for (int j = 0; j < NQ; ++j) q_next[j] = fetch_q(g_begin, j);
  f_next = fetch_f(g_begin);

  for (int r = tid; r < rows; r += 256) s_inc[r] = 0.0;
  if (tid < R) s_z[tid] = a.z[(size_t)u * R + tid];
  if constexpr (STAGE) {
    for (int r = tid; r < m; r += 256) {
      s_acc[r] = a.acc[(size_t)u * C + r];
      s_pos[r] = a.pos[(size_t)u * C + r];
    }
    // all requests of a batch first, then the LDS stores (the staged sizes fit one batch)
    constexpr int VPR = D / EPL, NB = 8;                     // 16-byte vectors per row; vectors per thread and batch
    const int nvec = rows * VPR;
    for (int b0 = 0; b0 < nvec; b0 += NB * 256) {
      Vec kb[NB], vb[NB];
#pragma unroll
      for (int j = 0; j < NB; ++j) {
        const int i = b0 + j * 256 + tid, ic = i < nvec ? i : nvec - 1;
        const int r = ic / VPR, c = ic % VPR;
        kb[j] = load_vec<T>((r < m ? kc + (size_t)r * D : kn) + c * EPL);
        vb[j] = load_vec<T>((r < m ? vc + (size_t)r * D : vn) + c * EPL);
      }
#pragma unroll
      for (int j = 0; j < NB; ++j) {
        const int i = b0 + j * 256 + tid;
        if (i < nvec) {
          reinterpret_cast<Vec *>(s_k)[i] = kb[j];
          reinterpret_cast<Vec *>(s_v)[i] = vb[j];
        }
      }
    }
    const int nh4 = R * D / 4;
    for (int b0 = 0; b0 < nh4; b0 += 4 * 256) {
      float4 hb4[4];
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int i = b0 + j * 256 + tid;
        hb4[j] = reinterpret_cast<const float4 *>(Hu)[i < nh4 ? i : nh4 - 1];
      }
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int i = b0 + j * 256 + tid;
        if (i < nh4) reinterpret_cast<float4 *>(s_H)[i] = hb4[j];
      }
    }
  }
  const double inv_sqrt_d = 1.0 / sqrt((double)D);
  const bool sparse_den = (a.flags & LESSDEC_FLAG_SPARSE_DENOM) != 0;

  for (int g0 = g_begin; g0 < g_end; g0 += GC) {
    __syncthreads();                                         // the previous chunk is done with s_q, s_f, s_e, s_hd
#pragma unroll
    for (int j = 0; j < NQ; ++j) s_q[j * 256 + tid] = q_next[j];
    if (tid < GC * R) s_f[(tid / R) * 64 + tid % R] = f_next;
    if (g0 + GC < g_end) {
#pragma unroll
      for (int j = 0; j < NQ; ++j) q_next[j] = fetch_q(g0 + GC, j);
      f_next = fetch_f(g0 + GC);
    }
    __syncthreads();
    // scores of the four heads against the cached keys and the appended key: LPR lanes of 16
    // bytes per row, RPB rows per pass
    {
      double qreg[GC][EPL];
#pragma unroll
      for (int g = 0; g < GC; ++g)
#pragma unroll
        for (int i = 0; i < EPL; ++i) qreg[g][i] = s_q[g * D + lr * EPL + i];
      auto row_vec = [&](int r) -> Vec {                     // this lane's 16 bytes of key row r (clamped: in range)
        const int rc = r < rows ? r : rows - 1;
        if constexpr (STAGE) return *reinterpret_cast<const Vec *>(s_k + (size_t)rc * D + lr * EPL);
        return load_vec<T>((rc < m ? kc + (size_t)rc * D : kn) + lr * EPL);
      };
      auto score = [&](int r, const Vec &kv) {
        double kd[EPL];
#pragma unroll
        for (int i = 0; i < EPL; ++i) kd[i] = (double)Store<T>::get(kv, i);
#pragma unroll
        for (int g = 0; g < GC; ++g) {
          double acc = 0.0;
#pragma unroll
          for (int i = 0; i < EPL; ++i) acc = fma(qreg[g][i], kd[i], acc);
          acc = row_sum<LPR>(acc);
          if (lr == 0 && r < rows) s_e[g * ecap + r] = acc * inv_sqrt_d;
        }
      };
      if constexpr (STAGE) {
        for (int r0 = 0; r0 < rows; r0 += RPB) score(r0 + rb, row_vec(r0 + rb));
      } else {
        // from memory: the rows of the first NP passes are requested together
        constexpr int NP = 8;
        Vec kvs[NP];
#pragma unroll
        for (int p = 0; p < NP; ++p) kvs[p] = row_vec(p * RPB + rb);
#pragma unroll
        for (int p = 0; p < NP; ++p)
          if (p * RPB < rows) score(p * RPB + rb, kvs[p]);
        for (int r0 = NP * RPB; r0 < rows; r0 += RPB) score(r0 + rb, row_vec(r0 + rb));
      }
    }
    __syncthreads();
    // wave w: softmax of head w.  m* = max(scores, ln(phi(q) z^T)) is the common shift (Eq. 3
    // times e^{-m*}); den = phi(q) z^T e^{-m*} + sum_j e^{s_j - m*}
    {
      double *e_w = s_e + w * ecap;
      double mx = -__builtin_inf();
      for (int r = lane; r < rows; r += kWave) mx = fmax(mx, e_w[r]);
      mx = wave_allreduce(mx, OpMax{});
      double fz = 0.0;
      for (int r = 0; r < R; ++r) fz = fma(s_f[w * 64 + r], s_z[r], fz);
      const double lfz = fz > 0.0 ? log(fz) : -__builtin_inf();
      const double mstar = fmax(mx, lfz);
      const double wl = fz > 0.0 ? exp(lfz - mstar) : 0.0;
      double part = 0.0;
      for (int r = lane; r < rows; r += kWave) {
        const double e = exp_softmax_f64(e_w[r] - mstar);
        e_w[r] = e;
        part += e;
      }
      const double sum = wave_allreduce(part, OpAdd{});
      const double den = wl + sum;
      if (lane == 0) {
        s_hd[w * 4 + 0] = fz > 0.0 ? exp(-mstar) : 0.0;
        s_hd[w * 4 + 1] = 1.0 / den;
        s_hd[w * 4 + 2] = g0 + w < g_end ? 1.0 / (sparse_den ? sum : den) : 0.0;   // heads past the share add nothing
      }
    }
    __syncthreads();
    // wave w: output of head w, (phi(q) H e^{-m*} + sum_j e_j V_j) / den.  A lane takes four
    // adjacent columns and every NRS-th row; the row shares then meet by lane exchange.
    {
      constexpr int NQD = D / 4, NRS = kWave / NQD;          // column quads; row shares per wave
      const int dq = lane % NQD, rs = lane / NQD;
      const double *e_w = s_e + w * ecap;
      const double hs = s_hd[w * 4 + 0];
      double num[4] = {0.0, 0.0, 0.0, 0.0};
      if (rs == 0 && hs > 0.0) {
#pragma unroll 8
        for (int r = 0; r < R; ++r) {
          const float4 h4 = *reinterpret_cast<const float4 *>((STAGE ? s_H : Hu) + r * D + 4 * dq);
          const double f = s_f[w * 64 + r];
          num[0] = fma(f, (double)h4.x, num[0]);
          num[1] = fma(f, (double)h4.y, num[1]);
          num[2] = fma(f, (double)h4.z, num[2]);
          num[3] = fma(f, (double)h4.w, num[3]);
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) num[i] *= hs;
      }
#pragma unroll 8
      for (int r = rs; r < rows; r += NRS) {
        const double e = e_w[r];
        float v4[4];
        if constexpr (STAGE) load_four<T>(s_v + (size_t)r * D + 4 * dq, v4);
        else load_four<T>((r < m ? vc + (size_t)r * D : vn) + 4 * dq, v4);
#pragma unroll
        for (int i = 0; i < 4; ++i) num[i] = fma(e, (double)v4[i], num[i]);
      }
#pragma unroll
      for (int o = NQD; o < kWave; o *= 2)
#pragma unroll
        for (int i = 0; i < 4; ++i) num[i] += __shfl_xor(num[i], o);
      if (rs == 0 && g0 + w < g_end) {
        const double inv_den = s_hd[w * 4 + 1];
        float o4[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          o4[i] = (float)(num[i] * inv_den);
          asm volatile("" : "+v"(o4[i]));                  // fp64 -> fp16 in one step would be a software sequence
        }
        store_four<T>(reinterpret_cast<T *>(a.out) + ((size_t)u * G + g0 + w) * D + 4 * dq, o4);
      }
    }
    // the chunk's probabilities (H2O accumulates those of every head), in head order
    for (int r = tid; r < rows; r += 256) {
      double inc = s_inc[r];
#pragma unroll
      for (int g = 0; g < GC; ++g) inc = fma(s_e[g * ecap + r], s_hd[g * 4 + 2], inc);
      s_inc[r] = inc;
    }
  }
  __syncthreads();

  if (nhb > 1) {
    // the unit's heads are spread over nhb blocks: leave this block's sums for the finishing launch
    double *part = a.gqa_parts + ((size_t)u * nhb + hb) * rows_cap;
    for (int r = tid; r < rows; r += 256) part[r] = s_inc[r];
    return;
  }
  LdsCopies<T> lds;
  if constexpr (STAGE) {
    lds.k = s_k; lds.v = s_v; lds.H = s_H; lds.acc = s_acc; lds.pos = s_pos;
  }
  gqa_finish_unit<T, D>(a, u, tid, s_e, s_inc, s_cand, lds);
}

// Dynamic LDS of gqa_chunk_kernel, in bytes.
template <typename T, int D>
static size_t gqa_chunk_lds(int C, int R, bool stage)
{
  const size_t work = (size_t)((kGqaChunk + 1) * ((C + 3) & ~1) + kGqaChunk * (D + 64) + 64 + kGqaChunk * 4) * sizeof(double);
  if (!stage) return work;
  return work + (size_t)((C + 1) / 2 * 2) * sizeof(double) + (size_t)((C + 3) / 4 * 4) * sizeof(int) +
         (size_t)R * D * sizeof(float) + 2 * (size_t)(C + 1) * D * sizeof(T);
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
  const int n = sane_n_seen(a.n_seen[u]);
  const int rows = (n < a.C ? n : a.C) + 1;
  for (int r = tid; r < rows; r += 256) {
    double p[kGqaMaxHeadBlocks];
#pragma unroll
    for (int hb = 0; hb < kGqaMaxHeadBlocks; ++hb)
      p[hb] = a.gqa_parts[((size_t)u * nhb + (hb < nhb ? hb : nhb - 1)) * rows_cap + r];
    double v = 0.0;
#pragma unroll
    for (int hb = 0; hb < kGqaMaxHeadBlocks; ++hb)
      if (hb < nhb) v += p[hb];
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

// Most dynamic LDS the staged form may take: two blocks of it share a compute unit's 160 KB.
constexpr size_t kGqaStagedLds = 76 * 1024;

// LDS one block may take on this device (queried once; the devices of a process are alike).
static size_t block_lds_limit()
{
  static const size_t limit = [] {
    int dev = 0, v = 0;
    if (hipGetDevice(&dev) != hipSuccess) return (size_t)0;
    if (hipDeviceGetAttribute(&v, hipDeviceAttributeMaxSharedMemoryPerBlock, dev) != hipSuccess) return (size_t)0;
    return (size_t)v;
  }();
  return limit;
}

template <typename T, int D>
static hipError_t launch_step_gqa_t(const StepArgs &a, int G, hipStream_t st)
{
  int nhb = gqa_head_blocks(a.U, G);
  const int nchunk = (G + kGqaChunk - 1) / kGqaChunk;
  if (nhb > nchunk) nhb = nchunk;                           // whole chunks per block
  // the rows are staged whenever they fit: with a single chunk per block they are read once either
  // way, but the copy has all its requests in flight at once (measured: 25.6 against 26.5 us)
  const size_t staged = gqa_chunk_lds<T, D>(a.C, a.R, true), plain = gqa_chunk_lds<T, D>(a.C, a.R, false);
  const bool stage = staged <= kGqaStagedLds && staged <= block_lds_limit();
  if (!stage && plain > block_lds_limit()) return hipErrorInvalidValue;
  if (stage)
    gqa_chunk_kernel<T, D, true><<<a.U * nhb, 256, staged, st>>>(a, G, nhb);
  else
    gqa_chunk_kernel<T, D, false><<<a.U * nhb, 256, plain, st>>>(a, G, nhb);
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
