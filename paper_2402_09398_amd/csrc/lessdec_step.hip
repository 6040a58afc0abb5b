// Decode step (Algorithm 1): the fused attention / score-accumulate / evict / state-update
// kernel (Eq. 3-5) and the write-behind state fold.
#include "lessdec_wave.h"

namespace lessdec {

// Waves per SIMD the register allocation aims for (the K and V rows held in registers
// take 4 VGPRs per iteration, the values reusing the keys' registers).
constexpr int step_waves_per_simd(int nit) { return nit == 0 ? 6 : nit <= 2 ? 6 : nit <= 7 ? 5 : nit <= 11 ? 3 : 2; }

// =====================================================================================
// General form of the step: one block of four waves per unit, any capacity, rank and storage
// type.  The feature maps phi(q), psi(k) of the step come from the launches before it.
//
// A cache row is D * sizeof(T) bytes = LPR lanes of 16 bytes; the block covers RPB =
// 256 / LPR rows (4096 bytes) per iteration with fully coalesced 16-byte loads.  With
// NIT > 0 every key row of the unit is requested at kernel entry (NIT buffer loads per
// thread sharing one offset register; rows past the capacity read as zero; non-temporal,
// a row is not touched again before the same layer's next token) and every value row right
// after the scores, into the same registers.  Loads come back to a wave in issue order, so
// anything the head of the kernel wants early is requested before the keys, and nothing
// after the decisions waits on a load whose address depends on them.  NIT = 0 is the
// looped form for any capacity.
//
// Roles: wave 0 owns the scores (phase 2); wave 1 owns the low-rank side (phi(q), the
// pending fold of z, phi(q) z^T); the last D / 64 waves own one output column per thread
// (H, out, insert).
//
// Head     wave 1 / column threads: fold the pair discarded by the previous step into H, z
//          (Eq. 4, Eq. 5) and put the previous key's psi into its slot.  That fold is
//          written behind by one step because psi of the discarded slot is only addressable
//          once the eviction is known; here it costs no latency.  Eq. 3 of this step sees
//          the folded H, z, exactly as if the fold had happened at the end of the previous
//          step.
// Phase 1  all waves: scores s_j = q . K_j / sqrt(D) of the live slots and of the appended
//          key, fp64, reduced over the LPR lanes of a row by DPP.
// Phase 2a wave 0, one lane per row: shift and exponentials.  Meanwhile wave 1 forms
//          phi(q) z^T.
// Phase 2b wave 0: denominator of Eq. 3, probabilities, H2O score accumulation, eviction
//          argmin (Sec. 2.1).
// Phase 3  all waves: p . V in fp32 with the row mapping of phase 1; the discarded value
//          row is picked out of the registers that already hold it.
// Phase 4  column threads: out = p V + phi(q) H / den (Eq. 3); the new pair goes into the
//          freed slot (Sec. 3.2); the discarded value row is left pending.
// =====================================================================================
template <typename T, int D, int NIT>
__global__ __launch_bounds__(256, step_waves_per_simd(NIT)) void step_kernel(const StepArgs a)
{
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
  __shared__ double s_fz, s_lscale;
  __shared__ int s_eslot;

  const int u = (int)blockIdx.x;
  const int tid = threadIdx.x, wave = tid / kWave, lane = tid % kWave;
  const int lr = tid % LPR, rb = tid / LPR;
  const int col = tid - (kThreads - D);    // threads of the last D / 64 waves own one column each
  const int R = a.R;

  T *kc = reinterpret_cast<T *>(a.k_cache) + (size_t)u * C * D;
  T *vc = reinterpret_cast<T *>(a.v_cache) + (size_t)u * C * D;
  const T *qn = reinterpret_cast<const T *>(a.q) + (size_t)u * D;
  const T *kn = reinterpret_cast<const T *>(a.k) + (size_t)u * D;
  const T *vn = reinterpret_cast<const T *>(a.v) + (size_t)u * D;

  // ---- requests, small ones first -----------------------------------------------------------
  const int n = sane_n_seen(a.n_seen[u]);
  const Pending pend = decode_pending(a.pend_slot[u], C);
  const Vec qv = load_vec<T>(qn + lr * EPL);
  const Vec knv = load_vec<T>(kn + lr * EPL);
  const Vec vnv = load_vec<T>(vn + lr * EPL);
  constexpr int NR2 = NIT > 0 ? (NIT * RPB + kWave - 1) / kWave : 1;
  double acc_pre[NR2];                    // wave 0: accumulated score and position of its rows
  int pos_pre[NR2];
  double f_lane = 0.0, z_lane = 0.0;      // wave 1, lane r < R
  float ppsi_lane = 0.f, npsi_lane = 0.f; // psi of the previous step's key and of this step's
  if (wave == 0) {
    if constexpr (NIT > 0) {
#pragma unroll
      for (int i = 0; i < NR2; ++i) {
        const int j = lane + i * kWave;
        acc_pre[i] = (j < C) ? a.acc[(size_t)u * C + j] : 0.0;
        pos_pre[i] = (j < C) ? a.pos[(size_t)u * C + j] : -1;
      }
    }
  } else if (wave == 1 && lane < R) {
    z_lane = a.z[(size_t)u * R + lane];
    ppsi_lane = a.pend_psi[(size_t)u * R + lane];
    npsi_lane = a.f_psi[(size_t)u * R + lane];
    f_lane = a.f_phi[(size_t)u * R + lane];
  }
  float hreg[16];                          // column threads: their column of H
  float pend_v_c = 0.f;
  if (col >= 0) {
    if (R <= 16) {
#pragma unroll
      for (int r = 0; r < 16; ++r) hreg[r] = (r < R) ? a.H[((size_t)u * R + r) * D + col] : 0.f;
    }
    pend_v_c = Store<T>::to_float(reinterpret_cast<const T *>(a.pend_v)[(size_t)u * D + col]);
  }
  __builtin_amdgcn_sched_barrier(0);
  Vec kbuf[NBUF], vbuf[NBUF];
  if constexpr (NIT > 0) {
    const __amdgpu_buffer_rsrc_t rk =
        __builtin_amdgcn_make_buffer_rsrc(kc, 0, C * D * (int)sizeof(T), 0x00020000);
#pragma unroll
    for (int it = 0; it < NIT; ++it) kbuf[it] = buffer_load_nt<T>(rk, tid * 16, it * kIterBytes);
  }
  __builtin_amdgcn_sched_barrier(0);
  // psi of the pending discarded pair (address known only now; it returns behind the keys)
  float psie_lane = 0.f;
  if (wave == 1 && lane < R && pend.fold)
    psie_lane = pend.slot < C ? a.psi[((size_t)u * C + pend.slot) * R + lane] : ppsi_lane;

  const int m = n < C ? n : C;          // live slots are 0..m-1 (slots fill in order)
  const int rows = m + 1;               // + the appended pair (K', V' of Eq. 3)
  const bool full = (m == C);
  if constexpr (NIT > 0) {
    // row m of K' is the appended key: it takes the place of the (empty or out-of-range)
    // cache row in the registers of the threads that cover it
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
#pragma unroll
      for (int it = 0; it < NIT; ++it) {
        score_row(it * RPB + rb, kbuf[it]);       // rows past m are computed but not stored
        __builtin_amdgcn_sched_barrier(0);        // one row at a time: keeps the fp64 temporaries few
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
  if constexpr (NIT > 0) {
    // The value rows are requested now, into the registers the keys just left: at kernel
    // entry they would share the memory queues with every block's keys and delay all scores.
    __builtin_amdgcn_sched_barrier(0);
    const __amdgpu_buffer_rsrc_t rv =
        __builtin_amdgcn_make_buffer_rsrc(vc, 0, C * D * (int)sizeof(T), 0x00020000);
#pragma unroll
    for (int it = 0; it < NIT; ++it) vbuf[it] = buffer_load_nt<T>(rv, tid * 16, it * kIterBytes);
    __builtin_amdgcn_sched_barrier(0);
  }
  if (wave == 1 && lane < R && pend.fold) s_psie[lane] = psie_lane;
  __syncthreads();

  double M = 0.0, S = 0.0;
  if (wave == 0) {
    // ---- phase 2a: shift and exponentials ------------------------------------------------
    M = -__builtin_inf();
    for (int j = lane; j < rows; j += kWave) M = fmax(M, s_sc[j]);
    M = wave_allreduce(M, OpMax{});
    for (int j = lane; j < rows; j += kWave) {
      const double e = exp(s_sc[j] - M);
      s_sc[j] = e;
      S += e;
    }
    S = wave_allreduce(S, OpAdd{});                       // sparse part of the denominator, shifted
  } else if (wave == 1) {
    // ---- low-rank side: phi(q), pending fold of z (Eq. 5), phi(q) z^T ---------------------
    if (lane < R) {
      if (pend.fold) {
        z_lane += (double)psie_lane;
        a.z[(size_t)u * R + lane] = z_lane;
      }
      if (pend.slot >= 0 && pend.slot < C) a.psi[((size_t)u * C + pend.slot) * R + lane] = ppsi_lane;
      a.pend_psi[(size_t)u * R + lane] = npsi_lane;
      s_f[lane] = (float)f_lane;
    }
    const double fz = wave_allreduce(f_lane * z_lane, OpAdd{});      // phi(q) z^T
    if (lane == 0) s_fz = fz;
  } else if (col >= 0 && pend.fold) {
    // ---- column threads: fold the pending pair into H (Eq. 4) ---------------------------------
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
  __syncthreads();

  // ---- phase 2b (wave 0): denominator, H2O accumulation, eviction choice -------------------
  if (wave == 0) {
    const double fz = s_fz;
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

    const bool lambda = (a.flags & LESSDEC_FLAG_LAMBDA) != 0;
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
        // H2O: every pair that is not among the Nr most recent competes on its score;
        // Lambda-masking: the first Nh tokens never leave and the oldest of the others does
        const bool is_cand = (j < m) ? (pj <= n - a.Nr && (!lambda || pj >= a.Nh)) : (a.Nr == 0);
        const Cand cnd{lambda ? 0.0 : na, pj, j};
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
      // what the next step has to finish: fold of the discarded pair and / or the slot write
      a.pend_slot[u] = evict ? (eslot < m ? eslot : C) : (m | kPendNoFold);
      if (a.evicted_pos) a.evicted_pos[u] = evict ? epos : -1;
      a.n_seen[u] = n + 1;
    }
  }
  __syncthreads();

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
        if (it * RPB + rb == m) vv = vnv;                // the appended pair's value row
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
    float of = (float)o;
    asm volatile("" : "+v"(of));                             // fp64 -> fp16 in one step would be a software sequence
    reinterpret_cast<T *>(a.out)[(size_t)u * D + col] = Store<T>::from_float(of);
    if (evict)
      reinterpret_cast<T *>(a.pend_v)[(size_t)u * D + col] = reinterpret_cast<const T *>(s_ve)[col];
    if (ins_slot >= 0) {
      kc[(size_t)ins_slot * D + col] = kn[col];
      vc[(size_t)ins_slot * D + col] = vn[col];
    }
  }
}

// Finishes whatever the last step left pending, so that H, z and psi are current (Eq. 4, 5).
template <typename T>
__global__ __launch_bounds__(256) void state_sync_kernel(const StepArgs a, int D)
{
  const int u = blockIdx.x, tid = threadIdx.x, C = a.C, R = a.R;
  __shared__ float s_psie[LESSDEC_MAX_RANK];
  const Pending pend = decode_pending(a.pend_slot[u], C);
  if (pend.slot < 0) return;                             // uniform per block
  const float *ppsi = a.pend_psi + (size_t)u * R;
  if (pend.fold) {
    if (tid < R) s_psie[tid] = pend.slot < C ? a.psi[((size_t)u * C + pend.slot) * R + tid] : ppsi[tid];
    __syncthreads();
    if (tid < D) {
      const float v = Store<T>::to_float(reinterpret_cast<const T *>(a.pend_v)[(size_t)u * D + tid]);
      for (int r = 0; r < R; ++r) {
        float *h = a.H + ((size_t)u * R + r) * D + tid;
        *h = fmaf(s_psie[r], v, *h);
      }
    }
    if (tid < R) a.z[(size_t)u * R + tid] += (double)s_psie[tid];
  }
  if (tid < R && pend.slot < C) a.psi[((size_t)u * C + pend.slot) * R + tid] = ppsi[tid];
  if (tid == 0) a.pend_slot[u] = -1;
}

template <typename T, int D>
static hipError_t launch_step_t(const StepArgs &a, hipStream_t st)
{
  constexpr int RPB = 256 / (D / Store<T>::kPerVec);
  const size_t lds = (size_t)(a.C + 1) * (sizeof(double) + sizeof(float));
  const int need = (a.C + 1 + RPB - 1) / RPB;            // row iterations to cover C + 1 rows
  const unsigned grid = (unsigned)a.U;
  if (need <= 2) step_kernel<T, D, 2><<<grid, 256, lds, st>>>(a);
  else if (need <= 7) step_kernel<T, D, 7><<<grid, 256, lds, st>>>(a);
  else if (need <= 11) step_kernel<T, D, 11><<<grid, 256, lds, st>>>(a);
  else if (need <= 21) step_kernel<T, D, 21><<<grid, 256, lds, st>>>(a);
  else step_kernel<T, D, 0><<<grid, 256, lds, st>>>(a);
  return hipGetLastError();
}

hipError_t launch_step(const StepArgs &a, int dtype, int D, hipStream_t st)
{
  if (dtype == LESSDEC_DTYPE_F16) {
    return D == 128 ? launch_step_t<__half, 128>(a, st) : launch_step_t<__half, 64>(a, st);
  }
  return D == 128 ? launch_step_t<float, 128>(a, st) : launch_step_t<float, 64>(a, st);
}

hipError_t launch_state_sync(const StepArgs &a, int dtype, int D, hipStream_t st)
{
  if (dtype == LESSDEC_DTYPE_F16) state_sync_kernel<__half><<<a.U, 256, 0, st>>>(a, D);
  else state_sync_kernel<float><<<a.U, 256, 0, st>>>(a, D);
  return hipGetLastError();
}

}  // namespace lessdec
