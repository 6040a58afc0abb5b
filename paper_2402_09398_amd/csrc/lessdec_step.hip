// Decode step (Algorithm 1): the fused attention / score-accumulate / evict / state-update
// kernel (Eq. 3-5) and the write-behind state fold.
#include "lessdec_common.h"
#include "lessdec_internal.h"

namespace lessdec {

typedef unsigned int u4v __attribute__((ext_vector_type(4)));

// =====================================================================================
// Fused step kernel: one block of 256 threads per unit.
//
// A cache row is D * sizeof(T) bytes = LPR lanes of 16 bytes; the block covers RPB =
// 256 / LPR rows (4096 bytes) per iteration with fully coalesced 16-byte loads.  With
// NIT > 0 every K and V row of the unit is requested at kernel entry (NIT buffer loads of
// each per thread, sharing one offset register; rows past the capacity read as zero;
// non-temporal, since a row is not touched again before the same layer's next token), so
// the memory system sees the whole unit at once and nothing after that waits on a load
// whose address depends on the step's decisions.  NIT = 0 is the looped form for any
// capacity.
//
// Head     while K and V are in flight: fold the pair discarded by the previous step into
//          H, z (Eq. 4, Eq. 5) and put the previous key's psi into its slot.  That fold is
//          written behind by one step because its inputs (psi of the discarded slot) are
//          only addressable once the eviction is known; doing it here keeps every such
//          dependent load off the tail of the kernel.  Eq. 3 of this step sees the folded
//          H, z, exactly as if the fold had happened at the end of the previous step.
// Phase 1  all waves: scores s_j = q . K_j / sqrt(D) of the live slots and of the appended
//          key, fp64, reduced over the LPR lanes of a row.
// Phase 2  wave 0, one lane per row: shift, exponentials, the denominator of Eq. 3 with
//          phi(q) z^T, probabilities, H2O score accumulation, eviction argmin (Sec. 2.1),
//          all by DPP / readlane reductions.
// Phase 3  all waves: p . V in fp32 with the row mapping of phase 1; the discarded value
//          row is picked out of the registers that already hold it.
// Phase 4  one thread per column: out = p V + phi(q) H / den (Eq. 3); the new pair goes
//          into the freed slot (Sec. 3.2); the discarded value row is left pending.
// =====================================================================================
template <int CTRL>
__device__ inline int dpp_mov(int x)
{
  return __builtin_amdgcn_update_dpp(0, x, CTRL, 0xf, 0xf, true);
}
template <int CTRL>
__device__ inline double dpp_mov(double x)
{
  return __hiloint2double(dpp_mov<CTRL>(__double2hiint(x)), dpp_mov<CTRL>(__double2loint(x)));
}
// All-reduce over the 16 lanes of a DPP row: quad_perm [1,0,3,2], quad_perm [2,3,0,1],
// row_ror 4, row_ror 8.  Every lane ends with the row's result.
template <typename V, typename Op>
__device__ inline V row16_allreduce(V v, Op op)
{
  v = op(v, dpp_mov<0xB1>(v));
  v = op(v, dpp_mov<0x4E>(v));
  v = op(v, dpp_mov<0x124>(v));
  v = op(v, dpp_mov<0x128>(v));
  return v;
}
__device__ inline int readlane_v(int x, int l) { return __builtin_amdgcn_readlane(x, l); }
__device__ inline double readlane_v(double x, int l)
{
  return __hiloint2double(__builtin_amdgcn_readlane(__double2hiint(x), l),
                          __builtin_amdgcn_readlane(__double2loint(x), l));
}
// All-reduce over the wave, combined in the fixed order ((row0, row1), row2), row3.
template <typename V, typename Op>
__device__ inline V wave_allreduce(V v, Op op)
{
  v = row16_allreduce(v, op);
  return op(op(op(readlane_v(v, 0), readlane_v(v, 16)), readlane_v(v, 32)), readlane_v(v, 48));
}
struct OpAdd { __device__ double operator()(double a, double b) const { return a + b; } };
struct OpMax { __device__ double operator()(double a, double b) const { return fmax(a, b); } };
struct OpMin { __device__ double operator()(double a, double b) const { return fmin(a, b); } };
struct OpMinI { __device__ int operator()(int a, int b) const { return a < b ? a : b; } };

template <int LPR>
__device__ inline double row_sum(double v)
{
  if constexpr (LPR == 16) {
    return row16_allreduce(v, OpAdd{});
  } else {
#pragma unroll
    for (int o = LPR / 2; o > 0; o >>= 1) v += __shfl_xor(v, o);
    return v;
  }
}

template <typename T>
__device__ inline typename Store<T>::Vec load_vec_nt(const T *p)
{
  typename Store<T>::Vec v;
  const u4v t = __builtin_nontemporal_load(reinterpret_cast<const u4v *>(p));
  __builtin_memcpy(&v.raw, &t, 16);
  return v;
}
template <typename T>
__device__ inline typename Store<T>::Vec buffer_load_nt(__amdgpu_buffer_rsrc_t rsrc, int voffset, int soffset)
{
  typename Store<T>::Vec v;
  const u4v t = __builtin_amdgcn_raw_buffer_load_b128(rsrc, voffset, soffset, 2 /* nt */);
  __builtin_memcpy(&v.raw, &t, 16);
  return v;
}

// pend_slot values: -1 nothing pending; s in [0, C): the pair that sat in slot s was
// discarded (its psi is still in psi[s], its value row in pend_v) and psi[s] is to become
// pend_psi; C: the last step's own pair was discarded (its psi is pend_psi).
template <typename T>
__device__ inline float pending_psi(const StepArgs &a, int u, int C, int R, int ps, int r)
{
  return ps < C ? a.psi[((size_t)u * C + ps) * R + r] : a.pend_psi[(size_t)u * R + r];
}

// Waves per SIMD the register allocation aims for (the K and V rows held in registers
// take 8 VGPRs per iteration).
constexpr int step_waves_per_simd(int nit) { return nit == 0 ? 6 : nit <= 2 ? 6 : nit <= 7 ? 5 : nit <= 11 ? 3 : 2; }

#ifdef LESSDEC_TRACE
__device__ unsigned long long *g_trace = nullptr;   // [blocks][8], set by the tracing harness
#define LESSDEC_STAMP(i)                                                                  \
  do {                                                                                    \
    if (g_trace && (threadIdx.x & 63) == 0)                                               \
      g_trace[(size_t)blockIdx.x * 8 + (i)] = __builtin_amdgcn_s_memrealtime();           \
  } while (0)
#else
#define LESSDEC_STAMP(i) do { } while (0)
#endif

template <typename T, int D, int NIT>
__global__ __launch_bounds__(256, step_waves_per_simd(NIT)) void step_unit_kernel(const StepArgs a)
{
  LESSDEC_STAMP(0);
  constexpr int kThreads = 256;
  constexpr int EPL = Store<T>::kPerVec;   // elements per lane
  constexpr int LPR = D / EPL;             // lanes per row
  constexpr int RPB = kThreads / LPR;      // rows per block iteration
  constexpr int NBUF = NIT > 0 ? NIT : 1;
  constexpr int kIterBytes = kThreads * 16;
  static_assert(LPR >= 8 && LPR <= 32, "row must span 8..32 lanes");
  using Vec = typename Store<T>::Vec;

  extern __shared__ double dyn[];
  const int C = a.C;
  double *s_sc = dyn;                                        // [C+1] scores
  float *s_p = reinterpret_cast<float *>(dyn + (C + 1));     // [C+1] probabilities (fp32)
  __shared__ __attribute__((aligned(16))) float s_o[RPB * D];   // per row-group partial outputs
  __shared__ float s_psie[LESSDEC_MAX_RANK];                 // psi of the pending discarded pair
  __shared__ float s_f[LESSDEC_MAX_RANK];                    // phi(q) for the column threads
  __shared__ Vec s_ve[LPR];                                  // value row discarded by this step
  __shared__ double s_lscale;
  __shared__ int s_eslot;

  const int u = blockIdx.x;
  const int tid = threadIdx.x, lane = tid % kWave;
  const int lr = tid % LPR, rb = tid / LPR;
  // Roles rotate with the block index: the blocks that share a CU differ in blockIdx / 256
  // (blocks go round-robin over 8 XCDs x 32 CUs), so their serial phase 2 lands on different
  // SIMDs instead of queueing on one.  "wave" is the role index, not the hardware wave.
  const int wave = (tid / kWave + (int)(blockIdx.x >> 8)) & 3;
  const int col = wave * kWave + lane - (kThreads - D);   // role waves 4 - D/64 .. 3 own one column each
  const int R = a.R;

  T *kc = reinterpret_cast<T *>(a.k_cache) + (size_t)u * C * D;
  T *vc = reinterpret_cast<T *>(a.v_cache) + (size_t)u * C * D;
  const T *qn = reinterpret_cast<const T *>(a.q) + (size_t)u * D;
  const T *kn = reinterpret_cast<const T *>(a.k) + (size_t)u * D;
  const T *vn = reinterpret_cast<const T *>(a.v) + (size_t)u * D;

  // ---- requests, small ones first -----------------------------------------------------------
  // Loads return to a wave in issue order, so everything the head of the kernel works on
  // while the keys are in flight (counters, feature-map partial sums, scores, H, the pending
  // pair) is requested before the keys.
  const int n = a.n_seen[u];
  const int ps = a.pend_slot[u];
  const Vec qv = load_vec<T>(qn + lr * EPL);
  const Vec knv = load_vec<T>(kn + lr * EPL);
  const Vec vnv = load_vec<T>(vn + lr * EPL);
  // wave 0 owns one row per lane in phase 2: its accumulated score and position; and z
  constexpr int NR2 = NIT > 0 ? (NIT * RPB + kWave - 1) / kWave : 1;
  constexpr int kPre = 4;                 // feature-map parts fetched ahead (R' <= 512)
  double acc_pre[NR2];
  int pos_pre[NR2];
  float pphi[kPre];
  double f_lane = 0.0, z_lane = 0.0;
  float ppsi_lane = 0.f;
  if (wave == 0) {
    if constexpr (NIT > 0) {
#pragma unroll
      for (int i = 0; i < NR2; ++i) {
        const int j = lane + i * kWave;
        acc_pre[i] = (j < C) ? a.acc[(size_t)u * C + j] : 0.0;
        pos_pre[i] = (j < C) ? a.pos[(size_t)u * C + j] : -1;
      }
    }
    if (lane < R) {
      z_lane = a.z[(size_t)u * R + lane];
      ppsi_lane = a.pend_psi[(size_t)u * R + lane];
      if (a.nparts > 0) {
#pragma unroll
        for (int p = 0; p < kPre; ++p)
          pphi[p] = p < a.nparts ? a.part_phi[((size_t)p * a.U + u) * kMlpPartStride + lane] : 0.f;
      } else {
        f_lane = a.f_phi[(size_t)u * R + lane];
      }
    }
  }
  // column threads: their column of H and of the pending value row
  float hreg[16];
  float pend_v_c = 0.f, psin_c = 0.f;     // psin_c: psi of this step's key, threads col < R
  if (col >= 0) {
    if (R <= 16) {
#pragma unroll
      for (int r = 0; r < 16; ++r) hreg[r] = (r < R) ? a.H[((size_t)u * R + r) * D + col] : 0.f;
    }
    pend_v_c = Store<T>::to_float(reinterpret_cast<const T *>(a.pend_v)[(size_t)u * D + col]);
    if (col < R) psin_c = a.psi_new[(size_t)u * R + col];
  }
  __builtin_amdgcn_sched_barrier(0);
  Vec kbuf[NBUF], vbuf[NBUF];
  if constexpr (NIT > 0) {
    const int cache_bytes = C * D * (int)sizeof(T);
    const __amdgpu_buffer_rsrc_t rk = __builtin_amdgcn_make_buffer_rsrc(kc, 0, cache_bytes, 0x00020000);
#pragma unroll
    for (int it = 0; it < NIT; ++it) kbuf[it] = buffer_load_nt<T>(rk, tid * 16, it * kIterBytes);
  }
  __builtin_amdgcn_sched_barrier(0);
  const bool fold = ps >= 0;

  // ---- head work of wave 0 while the keys are in flight ---------------------------------------
  if (wave == 0) {
    if (a.nparts > 0) {
      // matrix-core path: add the partial sums of layer 2, then the last activation of Eq. 1
      double sp = 0.0;
      if (lane < R) {
#pragma unroll
        for (int p = 0; p < kPre; ++p) sp += (double)pphi[p];
        for (int p = kPre; p < a.nparts; ++p)
          sp += (double)a.part_phi[((size_t)p * a.U + u) * kMlpPartStride + lane];
      }
      f_lane = lane < R ? fabs(gelu_f64(sp)) : 0.0;
    }
    if (lane < R) {
      s_f[lane] = (float)f_lane;
      if (fold) s_psie[lane] = pending_psi<T>(a, u, C, R, ps, lane);
    }
  }
  const int m = n < C ? n : C;          // live slots are 0..m-1 (slots fill in order)
  const int rows = m + 1;               // + the appended pair (K', V' of Eq. 3)
  const bool full = (m == C);
  if constexpr (NIT > 0) {
    // row m of K', V' is the appended pair: it takes the place of the (empty or
    // out-of-range) cache row in the registers of the threads that cover it
#pragma unroll
    for (int it = 0; it < NIT; ++it) {
      if (it * RPB + rb == m) kbuf[it] = knv;
    }
  }

  // ---- phase 1: scores ---------------------------------------------------------------
  {
    double qd[EPL];
#pragma unroll
    for (int i = 0; i < EPL; ++i) qd[i] = (double)Store<T>::get(qv, i);
    const double inv_sqrt_d = 1.0 / sqrt((double)D);      // folded at compile time
    auto score_row = [&](int r, const Vec kv) {
      double part = 0.0;
#pragma unroll
      for (int i = 0; i < EPL; ++i) part = fma(qd[i], (double)Store<T>::get(kv, i), part);
      part = row_sum<LPR>(part);
      if (lr == 0 && r < rows) s_sc[r] = part * inv_sqrt_d;
    };
    if constexpr (NIT > 0) {
      // Each value row is requested as soon as the key row of the same iteration has been
      // consumed, into the registers it leaves.  Requested at kernel entry the values would
      // share the memory queues with every block's keys and delay all scores; requested
      // here they keep the memory system busy while the scores are computed and are in
      // flight while wave 0 works through phase 2.
      const __amdgpu_buffer_rsrc_t rv =
          __builtin_amdgcn_make_buffer_rsrc(vc, 0, C * D * (int)sizeof(T), 0x00020000);
#pragma unroll
      for (int it = 0; it < NIT; ++it) {
        score_row(it * RPB + rb, kbuf[it]);       // rows past m are computed but not stored
        __builtin_amdgcn_sched_barrier(0);        // one row at a time: keeps the fp64 temporaries few
        vbuf[it] = buffer_load_nt<T>(rv, tid * 16, it * kIterBytes);
        __builtin_amdgcn_sched_barrier(0);
      }
    } else {
      for (int r0 = 0; r0 < rows; r0 += RPB) {
        const int r = r0 + rb;
        Vec kv = knv;
        if (r < m) kv = load_vec_nt<T>(kc + (size_t)r * D + lr * EPL);
        score_row(r, kv);
      }
    }
  }
  LESSDEC_STAMP(1);
  __syncthreads();
  LESSDEC_STAMP(2);


  // ---- head work of the column threads: fold the pending pair into H (Eq. 4) --------------
  if (col >= 0 && fold) {
    float *Hu = a.H + (size_t)u * R * D;
    if (R <= 16) {
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        if (r < R) {
          hreg[r] = fmaf(s_psie[r], pend_v_c, hreg[r]);
          Hu[(size_t)r * D + col] = hreg[r];
        }
      }
    } else {
      for (int r = 0; r < R; ++r) Hu[(size_t)r * D + col] = fmaf(s_psie[r], pend_v_c, Hu[(size_t)r * D + col]);
    }
  }

  // ---- phase 2 (wave 0): softmax pieces, H2O accumulation, eviction choice --------------
  if (wave == 0) {
    // pending fold of z (Eq. 5) and the slot write of the previous key's psi
    if (fold && lane < R) {
      z_lane += (double)s_psie[lane];
      a.z[(size_t)u * R + lane] = z_lane;
      if (ps < C) a.psi[((size_t)u * C + ps) * R + lane] = ppsi_lane;
    }
    const double fz = wave_allreduce(f_lane * z_lane, OpAdd{});      // phi(q) z^T

    double M = -__builtin_inf();
    for (int j = lane; j < rows; j += kWave) M = fmax(M, s_sc[j]);
    M = wave_allreduce(M, OpMax{});
    double S = 0.0;
    for (int j = lane; j < rows; j += kWave) {
      const double e = exp(s_sc[j] - M);
      s_sc[j] = e;
      S += e;
    }
    S = wave_allreduce(S, OpAdd{});                       // sparse part of the denominator, shifted
    // den = phi(q) z^T + sum_j e^{s_j}, in whichever scaling cannot overflow:
    //   M > 0 (or no low-rank term): everything times e^{-M};  M <= 0: unscaled, e^{M} <= 1
    double pscale, lscale;
    if (fz > 0.0 && M <= 0.0) {
      const double w = exp(M);
      const double inv = 1.0 / (fz + w * S);
      pscale = w * inv;
      lscale = inv;
    } else {
      const double eM = (fz > 0.0) ? exp(-M) : 0.0;
      const double inv = 1.0 / (fz * eM + S);
      pscale = inv;
      lscale = eM * inv;
    }
    double ascale = pscale;
    if (a.flags & LESSDEC_FLAG_SPARSE_DENOM) ascale = 1.0 / S;

    Cand best = cand_none();
    for (int j = lane, i = 0; j < rows; j += kWave, ++i) {
      const double e = s_sc[j];
      s_p[j] = (float)(e * pscale);
      double na = e * ascale;
      int pj = n;
      if (j < m) {
        if constexpr (NIT > 0) {
          na += acc_pre[i];
          pj = pos_pre[i];
        } else {
          na += a.acc[(size_t)u * C + j];
          pj = a.pos[(size_t)u * C + j];
        }
      }
      s_sc[j] = na;
      if (full) {
        const bool is_cand = (j < m) ? (pj <= n - a.Nr) : (a.Nr == 0);
        const Cand cnd{na, pj, j};
        if (is_cand && cand_less(cnd, best)) best = cnd;
      }
    }
    // argmin over (score, position): smallest score, then the oldest among equals
    int eslot = -1, epos = -1;
    if (full) {
      const double amin = wave_allreduce(best.acc, OpMin{});
      const int pmin = wave_allreduce(best.acc == amin ? best.pos : INT_MAX, OpMinI{});
      const unsigned long long win = __ballot(best.acc == amin && best.pos == pmin && best.slot >= 0);
      if (win != 0ull) {
        eslot = __builtin_amdgcn_readlane(best.slot, __ffsll((long long)win) - 1);
        epos = pmin;
      }
    }
    const bool evict = eslot >= 0;                         // eslot == m: the new pair itself
    const int ins_slot = full ? ((evict && eslot < m) ? eslot : -1) : m;
    // accumulated scores and positions (each lane reads back only what it wrote to s_sc)
    for (int j = lane; j < rows; j += kWave) {
      if (j < m) {
        if (j != ins_slot) a.acc[(size_t)u * C + j] = s_sc[j];
      } else if (ins_slot >= 0) {
        a.acc[(size_t)u * C + ins_slot] = s_sc[m];
        a.pos[(size_t)u * C + ins_slot] = n;
      }
    }
    if (lane == 0) {
      s_lscale = lscale;
      s_eslot = eslot;
      a.pend_slot[u] = evict ? (eslot < m ? eslot : C) : -1;
      if (a.evicted_pos) a.evicted_pos[u] = evict ? epos : -1;
      a.n_seen[u] = n + 1;
    }
    LESSDEC_STAMP(3);
  }
  __syncthreads();
  LESSDEC_STAMP(4);

  // ---- phase 3: p . V -----------------------------------------------------------------------
  {
    const int eslot = s_eslot;
    float o[EPL];
#pragma unroll
    for (int i = 0; i < EPL; ++i) o[i] = 0.f;
    auto pv_row = [&](int r, const Vec vv) {
      if (r < rows) {                                    // rows past m may hold anything
        const float p = s_p[r];
#pragma unroll
        for (int i = 0; i < EPL; ++i) o[i] = fmaf(p, Store<T>::get(vv, i), o[i]);
      }
      if (r == eslot) s_ve[lr] = vv;                     // the discarded pair's value row
    };
    if constexpr (NIT > 0) {
#pragma unroll
      for (int it = 0; it < NIT; ++it) {
        Vec vv = vbuf[it];
        if (it * RPB + rb == m) vv = vnv;         // the appended pair's value row
        pv_row(it * RPB + rb, vv);
        __builtin_amdgcn_sched_barrier(0);
      }
    } else {
      for (int r0 = 0; r0 < rows; r0 += RPB) {
        const int r = r0 + rb;
        Vec vv = vnv;
        if (r < m) vv = load_vec_nt<T>(vc + (size_t)r * D + lr * EPL);
        pv_row(r, vv);
      }
    }
    float4 *so4 = reinterpret_cast<float4 *>(s_o + rb * D + lr * EPL);
#pragma unroll
    for (int i = 0; i < EPL / 4; ++i) so4[i] = float4{o[4 * i], o[4 * i + 1], o[4 * i + 2], o[4 * i + 3]};
  }
  LESSDEC_STAMP(5);
  __syncthreads();

  // ---- phase 4: output, in-place insert, pending value row -----------------------------------
  if (col >= 0) {
    const int eslot = s_eslot;
    const bool evict = eslot >= 0;
    const int ins_slot = full ? ((evict && eslot < m) ? eslot : -1) : m;
    float pv = 0.f;
#pragma unroll
    for (int gidx = 0; gidx < RPB; ++gidx) pv += s_o[gidx * D + col];
    float fh = 0.f;
    if (R <= 16) {
#pragma unroll
      for (int r = 0; r < 16; ++r)
        if (r < R) fh = fmaf(s_f[r], hreg[r], fh);
    } else {
      const float *Hu = a.H + (size_t)u * R * D;
      for (int r = 0; r < R; ++r) fh = fmaf(s_f[r], Hu[(size_t)r * D + col], fh);
    }
    const double o = (double)pv + s_lscale * (double)fh;
    reinterpret_cast<T *>(a.out)[(size_t)u * D + col] = Store<T>::from_float((float)o);
    if (evict)
      reinterpret_cast<T *>(a.pend_v)[(size_t)u * D + col] = reinterpret_cast<const T *>(s_ve)[col];
    if (ins_slot >= 0) {
      kc[(size_t)ins_slot * D + col] = kn[col];
      vc[(size_t)ins_slot * D + col] = vn[col];
    }
    // psi of this step's key: straight into its slot while the cache fills, else pending
    if (col < R) {
      if (evict) a.pend_psi[(size_t)u * R + col] = psin_c;
      else a.psi[((size_t)u * C + m) * R + col] = psin_c;
    }
  }
  LESSDEC_STAMP(6);
#ifdef LESSDEC_TRACE
  if (g_trace && threadIdx.x == 0) {
    unsigned hwid;
    asm volatile("s_getreg_b32 %0, hwreg(HW_REG_HW_ID)" : "=s"(hwid));
    unsigned xcc;
    asm volatile("s_getreg_b32 %0, hwreg(HW_REG_XCC_ID)" : "=s"(xcc));
    g_trace[(size_t)blockIdx.x * 8 + 7] = ((unsigned long long)xcc << 32) | hwid;
  }
#endif
}

#ifdef LESSDEC_TRACE
extern "C" int lessdec_trace_set(unsigned long long *buf)
{
  return (int)hipMemcpyToSymbol(HIP_SYMBOL(g_trace), &buf, sizeof(buf));
}
#endif

// Folds whatever the last step left pending, so that H, z and psi are current (Eq. 4, 5).
template <typename T>
__global__ __launch_bounds__(256) void state_sync_kernel(const StepArgs a, int D)
{
  const int u = blockIdx.x, tid = threadIdx.x, C = a.C, R = a.R;
  __shared__ float s_psie[LESSDEC_MAX_RANK];
  const int ps = a.pend_slot[u];
  if (ps < 0) return;                                    // uniform per block
  if (tid < R) s_psie[tid] = pending_psi<T>(a, u, C, R, ps, tid);
  __syncthreads();
  if (tid < D) {
    const float v = Store<T>::to_float(reinterpret_cast<const T *>(a.pend_v)[(size_t)u * D + tid]);
    for (int r = 0; r < R; ++r) {
      float *h = a.H + ((size_t)u * R + r) * D + tid;
      *h = fmaf(s_psie[r], v, *h);
    }
  }
  if (tid < R) {
    a.z[(size_t)u * R + tid] += (double)s_psie[tid];
    if (ps < C) a.psi[((size_t)u * C + ps) * R + tid] = a.pend_psi[(size_t)u * R + tid];
  }
  if (tid == 0) a.pend_slot[u] = -1;
}

template <typename T, int D>
static hipError_t launch_step_t(const StepArgs &a, int units, hipStream_t st)
{
  constexpr int RPB = 256 / (D / Store<T>::kPerVec);
  const size_t lds = (size_t)(a.C + 1) * (sizeof(double) + sizeof(float));
  const int need = (a.C + 1 + RPB - 1) / RPB;            // row iterations to cover C + 1 rows
  if (need <= 2) step_unit_kernel<T, D, 2><<<units, 256, lds, st>>>(a);
  else if (need <= 7) step_unit_kernel<T, D, 7><<<units, 256, lds, st>>>(a);
  else if (need <= 11) step_unit_kernel<T, D, 11><<<units, 256, lds, st>>>(a);
  else if (need <= 21) step_unit_kernel<T, D, 21><<<units, 256, lds, st>>>(a);
  else step_unit_kernel<T, D, 0><<<units, 256, lds, st>>>(a);
  return hipGetLastError();
}

hipError_t launch_step(const StepArgs &a, int units, int dtype, int D, hipStream_t st)
{
  if (dtype == LESSDEC_DTYPE_F16) {
    return D == 128 ? launch_step_t<__half, 128>(a, units, st) : launch_step_t<__half, 64>(a, units, st);
  }
  return D == 128 ? launch_step_t<float, 128>(a, units, st) : launch_step_t<float, 64>(a, units, st);
}

hipError_t launch_state_sync(const StepArgs &a, int units, int dtype, int D, hipStream_t st)
{
  if (dtype == LESSDEC_DTYPE_F16) state_sync_kernel<__half><<<units, 256, 0, st>>>(a, D);
  else state_sync_kernel<float><<<units, 256, 0, st>>>(a, D);
  return hipGetLastError();
}

}  // namespace lessdec
