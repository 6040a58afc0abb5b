// Decode step (Algorithm 1) with several query heads per key/value head (Sec. 3.2: H2O aggregates
// the scores of all query heads), streaming form: one block per unit, one wave per query head.
//
// Every wave streams the unit's K rows and then its V rows through its own register ring, as the
// single-head streaming kernel does (lessdec_wpu.hip): the G waves of a block ask for the same
// lines at nearly the same time, so each line comes from memory once and from the compute unit's
// cache for the other heads.  A wave has its own query, phi(q), scores, softmax (Eq. 3 with the
// shared state H, z) and output row.  What the heads share goes through the LDS:
//   barrier 1  every wave has the unit's state in registers (the lead wave may now store);
//   phase 2a   per head: shift and exponentials, which weight the value rows as they are (the
//              sum is scaled by 1 / den at the output), so that the value stream starts here and
//              everything below up to phase 3 is worked off between its first passes; Eq. 3's
//              denominator; the head's share of every pair's score increment goes to s_inc[head];
//   barrier 2  all increments visible;
//   phase 2b   every wave adds the increments in head order to the accumulated scores and works
//              out the eviction for itself (same data, same result);
//   phase 3/4  per head p . V, phi(q) H, output; then, behind its last load, the lead wave stores
//              the unit's new state and parks the discarded pair (no store stands in mid-stream:
//              a wave's memory counter runs in order; all stores go through the L2 to memory);
//   barrier 3  every wave is through with the cache rows; the lead wave writes the new pair
//              into its slot (Sec. 3.2).
// The fold of the discarded pair into H, z is left to the next step (pend_slot, as on the
// single-head path).  phi(q) per head and psi(k) come from the feature-map launch before it,
// complete or as the parts of their layer-2 sums, or (FUSED) from jobs inside this launch.
#include "lessdec_mlp.h"
#include "lessdec_wave.h"

namespace lessdec {

constexpr int kGqsMaxHeads = 8;     // waves per block
constexpr int kGqsMaxRows = 512;    // C + 1 at most
constexpr int kGqsParts = 8;        // feature maps taken as parts up to this many (R' <= 512)

// FUSED: the step's feature-map jobs (mlp_parts_gq_job) are the first n_mlp workgroups of the launch
// and hand their results to the attention waves through the exchange array, as in the one-wave-
// per-unit kernel (wpu_step_kernel): an entry no job has written yet holds kMlpEmpty, jobs write
// through with device-scope stores, waves read with device-scope loads, ask again while any entry
// is empty (bounded by kGqsSpinLimit polls, then the NaNs of the empty entries show in the unit's
// outputs), and hand the entries back empty with their other stores.  Workgroups are dispatched in
// index order and a job waits for nothing, so no cycle of waits exists.  A job is four waves: a
// block of four query heads runs one job, a block of eight two.
constexpr int kGqsSpinLimit = 1 << 14;
template <int D, int NR2, int RM, int DEPTH, bool FUSED>
__global__ __launch_bounds__(kGqsMaxHeads * kWave, FUSED ? 2 : 1) void gqs_step_kernel(
    void *k_cache_, const void *q_, const void *k_, int C_, int G_, int n_mlp, const void *Wq1_, const void *Wk1_,
    const void *Wq2_, const StepArgs a)
{
  using T = __half;
  constexpr int EPL = 8;                   // elements per lane
  constexpr int LPR = D / EPL;             // lanes per row
  constexpr int RPI = kWave / LPR;         // rows per load instruction
  using Vec = typename Store<T>::Vec;

  extern __shared__ __attribute__((aligned(16))) double dyn[];

  const int C = C_, R = a.R, G = G_;
  const int g = __builtin_amdgcn_readfirstlane((int)threadIdx.x >> 6);    // this wave's query head
  const int lane = threadIdx.x & 63;
  if constexpr (FUSED) {
    if ((int)blockIdx.x < n_mlp) {
      mlp_parts_gq_job<D, true>(reinterpret_cast<const __half *>(q_), reinterpret_cast<const __half *>(k_),
                                reinterpret_cast<const __half *>(Wq1_), reinterpret_cast<const __half *>(Wk1_),
                                reinterpret_cast<const __half *>(Wq2_), reinterpret_cast<const __half *>(a.Wk2), a.Hh, G,
                                a.Rp, R, a.B, a.mlp_out, (int)blockIdx.x * (G / 4) + g / 4,
                                reinterpret_cast<unsigned char *>(dyn) + (g / 4) * mlp_slab_bytes(D), g % 4, lane);
      return;
    }
  }
  const int lr = lane % LPR, rb = lane / LPR;
  const int u = FUSED ? (int)blockIdx.x - n_mlp : (int)blockIdx.x;
  const bool lead = g == 0;                                  // the wave that writes the unit's state
  const int rows_cap = (C + 2) & ~1;
  double *s_sc = dyn + (size_t)g * rows_cap;                 // [G][C+1] scores
  double *s_inc = dyn + (size_t)G * rows_cap;                // [G][C+1] a head's share of the score increments
  float *s_p = reinterpret_cast<float *>(dyn + 2 * (size_t)G * rows_cap) + (size_t)g * rows_cap;   // [G][C+1]

  T *kc = reinterpret_cast<T *>(k_cache_) + (size_t)u * C * D;
  T *vc = reinterpret_cast<T *>(a.v_cache) + (size_t)u * C * D;
  const T *qn = reinterpret_cast<const T *>(q_) + ((size_t)u * G + g) * D;
  const T *kn = reinterpret_cast<const T *>(k_) + (size_t)u * D;
  const T *vn = reinterpret_cast<const T *>(a.v) + (size_t)u * D;

  // ---- requests, in the order they are wanted back (all unconditional, clamped addresses) ----------
  const Vec qv = load_vec<T>(qn + lr * EPL);
  const Vec knv = load_vec<T>(kn + lr * EPL);
  u4v buf[DEPTH];
  {
    const __amdgpu_buffer_rsrc_t rk =
        __builtin_amdgcn_make_buffer_rsrc(kc, 0, C * D * (int)sizeof(T), 0x00020000);
#pragma unroll
    for (int j = 0; j < DEPTH; ++j)
      buf[j] = __builtin_amdgcn_raw_buffer_load_b128(rk, lane * 16, j * (kWave * 16), 2 /* nt */);
  }
  __builtin_amdgcn_sched_barrier(0);
  const int rl = (lane & 15) < R ? (lane & 15) : R - 1;
  // phi(q) of this head and psi(k) of the step's key (lane r < R): complete from the feature-map
  // launch, or (a.mlp_parts) as the parts of their layer-2 sums, which this wave adds up and
  // finishes after the first pass of the key stream (Eq. 1, Eq. 2), where nothing waits for anything
  constexpr int NP = kGqsParts;
  const bool parts = a.mlp_parts != nullptr;
  const int nparts = mlp_nparts(a.Rp), rp = mlp_entry_stride(R);
  const size_t fi = ((size_t)u * G + g) * R + rl;
  double f_lane = 0.0;
  float npsi_lane = 0.f;
  float pq[NP], pk[NP];
  __half w3[RM];
  const float *eq = a.mlp_parts + ((size_t)u * G + g) * nparts * rp + rl;
  const float *ek = a.mlp_parts + ((size_t)a.U * G + u) * nparts * rp + rl;
  auto request_parts = [&]() __attribute__((always_inline)) {
#pragma unroll
    for (int p = 0; p < NP; ++p) {
      const int pc = p < nparts ? p : nparts - 1;
      if constexpr (FUSED) {
        pq[p] = __hip_atomic_load(eq + (size_t)pc * rp, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        pk[p] = __hip_atomic_load(ek + (size_t)pc * rp, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      } else {
        pq[p] = eq[(size_t)pc * rp];
        pk[p] = ek[(size_t)pc * rp];
      }
    }
  };
  auto finish_maps = [&]() __attribute__((always_inline)) {
    double sq = 0.0, sk = 0.0;
#pragma unroll
    for (int p = 0; p < NP; ++p) {
      if (p < nparts) {
        sq += (double)pq[p];
        sk += (double)pk[p];
      }
    }
    f_lane = lane < R ? fabs(gelu_poly_f64(sq)) : 0.0;   // last activation of Eq. 1
    const double h2 = gelu_poly_f64(sk);                 // lane r < R; Eq. 2: |W3 gelu(.)|
    double acc3 = 0.0;
#pragma unroll
    for (int j = 0; j < RM; ++j)
      if (j < R) acc3 = fma(readlane_v(h2, j), (double)__half2float(w3[j]), acc3);
    npsi_lane = (float)fabs(acc3);
  };
  if (parts) {
    if constexpr (!FUSED) request_parts();
    const __half *w3row = reinterpret_cast<const __half *>(a.Wk3) + ((size_t)(u % a.Hh) * R + rl) * R;
#pragma unroll
    for (int j = 0; j < RM; ++j) w3[j] = w3row[j < R ? j : R - 1];
  } else {
    f_lane = a.f_phi32 ? (double)a.f_phi32[fi] : a.f_phi[fi];
    npsi_lane = a.f_psi[(size_t)u * R + rl];
  }
  // unit state (wanted from phase 2 on)
  const int n = sane_n_seen(a.n_seen[u]);
  const Pending pend = decode_pending(a.pend_slot[u], C);
  const int m = n < C ? n : C;          // live slots are 0..m-1 (slots fill in order)
  const int rows = m + 1;               // + the appended pair (K', V' of Eq. 3)
  const bool full = (m == C);
  // (FUSED: the accumulated scores are asked for behind the keys, with the rows of H: the kernel
  // has to stay within the registers of four resident waves per SIMD)
  double acc_pre[NR2];
  int pos_pre[NR2];
  auto request_scores = [&]() __attribute__((always_inline)) {
#pragma unroll
    for (int i = 0; i < NR2; ++i) {
      const int j = lane + i * kWave;
      const size_t idx = (size_t)u * C + (j < C ? j : C - 1);
      acc_pre[i] = a.acc[idx];
      pos_pre[i] = a.pos[idx];
    }
  };
  if constexpr (!FUSED) request_scores();
  double z_lane = a.z[(size_t)u * R + rl];                   // lane r < R
  const float ppsi_lane = a.pend_psi[(size_t)u * R + rl];
  float psie_lane = a.psi[((size_t)u * C + (pend.slot >= 0 && pend.slot < C ? pend.slot : 0)) * R + rl];
  __builtin_amdgcn_sched_barrier(0);

  // The stream: position s < nitp is load s of K, position nitp + t is load t of V.
  const int nit = (rows + RPI - 1) / RPI;                    // load instructions per stream (>= 1)
  const int nitp = (nit + DEPTH - 1) / DEPTH * DEPTH;        // K part of the stream, padded
  const int live_bytes = m * D * (int)sizeof(T);
  auto issue = [&](int s) -> u4v {                           // s is wave-uniform
    const bool isk = s < nitp;
    const __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc(isk ? kc : vc, 0, live_bytes, 0x00020000);
    return __builtin_amdgcn_raw_buffer_load_b128(rs, lane * 16, (isk ? s : s - nitp) * (kWave * 16), 2 /* nt */);
  };

  // ---- phase 1: this head's scores as the key rows arrive -------------------------------------------
  {
    const double inv_sqrt_d = 1.0 / sqrt((double)D);
    u4v knu;                                               // (as a value: a choice between addresses would put the ring into scratch memory)
    __builtin_memcpy(&knu, &knv.raw, 16);
    auto key_pass = [&](int base) __attribute__((always_inline)) {
#pragma unroll
      for (int j = 0; j < DEPTH; ++j) {
        const int s = base + j;
        if (s < nit) {
          const int r = s * RPI + rb;
          const u4v kraw = (r == m) ? knu : buf[j];          // r == m: the appended key
          Vec kv;
          __builtin_memcpy(&kv.raw, &kraw, 16);
          // a product of two halves is exact in fp32, so fp32 multiply, widen, fp64 add
          double part = 0.0;
#pragma unroll
          for (int i = 0; i < EPL; ++i) part += (double)(Store<T>::get(qv, i) * Store<T>::get(kv, i));
          part = row_sum<LPR>(part);
          if (lr == 0 && r < rows) s_sc[r] = part * inv_sqrt_d;
        }
        buf[j] = issue(s + DEPTH);
        __builtin_amdgcn_sched_barrier(0);
      }
    };
    if constexpr (FUSED) {
      // the entries are asked for before the last pass of the key stream
      int base = 0;
      for (; base + DEPTH < nitp; base += DEPTH) key_pass(base);
      request_parts();
      key_pass(base);
      // (looked at here, before the requests behind the keys: the entries give their sixteen
      // registers back before the rows of H take theirs)
      // The first look stands outside the loop and looks at every entry: a look at the loop's head,
      // or one that leaves after the first empty entry, would make whoever uses the entries next
      // wait for everything in flight.
      auto have_all = [&]() {
        unsigned missing = 0;
#pragma unroll
        for (int p = 0; p < NP; ++p)
          missing |= (unsigned)(__float_as_uint(pq[p]) == kMlpEmpty) | (unsigned)(__float_as_uint(pk[p]) == kMlpEmpty);
        return __all(missing == 0u) != 0;
      };
      bool have = have_all();
      for (int spin = 0; !have && spin < kGqsSpinLimit; ++spin) {
        __builtin_amdgcn_s_sleep(32);
        request_parts();
        have = have_all();
      }
      finish_maps();
    } else {
      int base = 0;
      do {                                                   // nitp >= DEPTH
        key_pass(base);
        if (base == 0 && parts) finish_maps();
      } while ((base += DEPTH) < nitp);
    }
  }

  // ---- requests behind the keys: what the value stream and the output want --------------------------
  const Vec vnv = load_vec<T>(vn + lr * EPL);
  constexpr int NHB = RPI / 2, HR = RM / NHB;
  const int col0 = lr * EPL + ((lane & LPR) ? 4 : 0);
  const int hb = lane / (2 * LPR);                           // which rows of H: r = NHB * i + hb
  float4 hreg[HR];
#pragma unroll
  for (int i = 0; i < HR; ++i) {
    const int r = NHB * i + hb;
    hreg[i] = *reinterpret_cast<const float4 *>(a.H + ((size_t)u * R + (r < R ? r : R - 1)) * D + col0);
  }
  const uint2 pend_v_h = *reinterpret_cast<const uint2 *>(reinterpret_cast<const T *>(a.pend_v) + (size_t)u * D + col0);
  if constexpr (FUSED) request_scores();
  // barrier 1: the lead wave's stores must not overtake another wave's loads of the same state:
  // have those loads back before the waves meet (the value rows requested after them stay in flight)
#pragma unroll
  for (int i = 0; i < NR2; ++i) asm volatile("" ::"v"(acc_pre[i]), "v"(pos_pre[i]));
#pragma unroll
  for (int i = 0; i < HR; ++i) asm volatile("" ::"v"(hreg[i].x), "v"(hreg[i].y), "v"(hreg[i].z), "v"(hreg[i].w));
  asm volatile("" ::"v"(z_lane), "v"(ppsi_lane), "v"(psie_lane), "v"(pend_v_h.x), "v"(pend_v_h.y));
  if constexpr (!FUSED) asm volatile("" ::"v"(npsi_lane), "v"(f_lane));
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
  __builtin_amdgcn_s_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");

  // ---- phase 2a, first part: what the value stream needs, the exponentials e^{s_j - M} -------------
  // As on the single-head path the value rows are weighted with the exponentials as they are, the
  // sum is scaled by 1 / den at the output, and the rest of phase 2 (denominator, the heads'
  // increments and barrier 2, accumulated scores and eviction, the fold into H) is worked off
  // between the first passes of the value stream, while the rows requested by the pass before
  // are on their way.  Every wave runs the same sequence of passes and barriers.
  double lscale = 0.0, pscale = 0.0;
  if (lane >= R) f_lane = 0.0;
  double sc[NR2];
  double M = -__builtin_inf();
#pragma unroll
  for (int i = 0; i < NR2; ++i) {
    const int j = lane + i * kWave;
    sc[i] = j < rows ? s_sc[j] : -__builtin_inf();
    M = fmax(M, sc[i]);
  }
  M = wave_allreduce(M, OpMax{});
#pragma unroll
  for (int i = 0; i < NR2; ++i) {
    const int j = lane + i * kWave;
    sc[i] = j < rows ? exp_softmax_f64(sc[i] - M) : 0.0;
    if (j < rows) s_p[j] = (float)sc[i];
  }
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");

  // ---- phase 3: e^{s - M} . V as the value rows arrive ----------------------------------------------
  float o[EPL];
#pragma unroll
  for (int i = 0; i < EPL; ++i) o[i] = 0.f;
  float fh[4] = {0.f, 0.f, 0.f, 0.f};                        // phi(q) H, this lane's columns and rows
  auto value_pass = [&](int base) __attribute__((always_inline)) {
#pragma unroll
    for (int j = 0; j < DEPTH; ++j) {
      const int s = base + j;
      if (s < nit) {
        const int r = s * RPI + rb;
        Vec vv;
        __builtin_memcpy(&vv.raw, &buf[j], 16);
        if (r < m) {
          const float p = s_p[r];
#pragma unroll
          for (int i = 0; i < EPL; ++i) o[i] = fmaf(p, Store<T>::get(vv, i), o[i]);
        }
      }
      buf[j] = issue(nitp + s + DEPTH);
      __builtin_amdgcn_sched_barrier(0);
    }
  };
  // Passes past the end of the stream consume nothing and request rows outside the buffer's
  // range, which fetches nothing: the three passes always run, so that no load sits under a
  // condition.
  value_pass(0);

  // ---- phase 2a, second part: Eq. 3's denominator, the head's share of the score increments ---------
  {
    double S = 0.0;
#pragma unroll
    for (int i = 0; i < NR2; ++i) S += sc[i];
    S = wave_allreduce(S, OpAdd{});                          // sparse part of the denominator, shifted
    // pending fold of z (Eq. 5), then phi(q) z^T
    if (lane >= R) z_lane = 0.0;
    if (!pend.fold) psie_lane = 0.f;
    else if (pend.slot >= C) psie_lane = ppsi_lane;          // the previous step discarded its own pair
    if (lane < R && pend.fold) z_lane += (double)psie_lane;
    const double fz = wave_allreduce(f_lane * z_lane, OpAdd{});
    if (fz > 0.0 && M <= 0.0) {
      const double w = exp_softmax_f64(M);
      const double inv = 1.0 / (fz + w * S);
      pscale = w * inv;
      lscale = inv;
    } else {
      const double eM = (fz > 0.0) ? exp_softmax_f64(-M) : 0.0;
      const double inv = 1.0 / (fz * eM + S);
      pscale = inv;
      lscale = eM * inv;
    }
    double ascale = pscale;
    if (a.flags & LESSDEC_FLAG_SPARSE_DENOM) ascale = 1.0 / S;
#pragma unroll
    for (int i = 0; i < NR2; ++i) {
      const int j = lane + i * kWave;
      if (j < rows) s_inc[(size_t)g * rows_cap + j] = sc[i] * ascale;
    }
  }
  // barrier 2: every head's increments are in the LDS
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
  __builtin_amdgcn_s_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
  value_pass(DEPTH);

  // ---- phase 2b: accumulated scores and the eviction, by every wave for itself ----------------------
  int eslot = -1, ins_slot = -1, epos = -1;
  double na_[NR2];
  u4v pv_row = {0u, 0u, 0u, 0u};                            // the discarded pair's value row
  {
    const bool lambda = (a.flags & LESSDEC_FLAG_LAMBDA) != 0;
    Cand best = cand_none();
#pragma unroll
    for (int i = 0; i < NR2; ++i) {
      const int j = lane + i * kWave;
      na_[i] = 0.0;
      if (j < rows) {
        double inc = 0.0;
        for (int h = 0; h < G; ++h) inc += s_inc[(size_t)h * rows_cap + j];     // in head order
        double na = inc;
        int pj = n;
        if (j < m) {
          na += acc_pre[i];
          pj = pos_pre[i];
        }
        na_[i] = na;
        if (full) {
          const bool is_cand = (j < m) ? (pj <= n - a.Nr && (!lambda || pj >= a.Nh)) : (a.Nr == 0);
          const Cand cnd{lambda ? 0.0 : na, pj, j};
          if (is_cand && cand_less(cnd, best)) best = cnd;
        }
      }
    }
    if (full) {
      const double amin = wave_allreduce(best.acc, OpMin{});
      const int pmin = wave_allreduce(best.acc == amin ? best.pos : INT_MAX, OpMinI{});
      const unsigned long long win = __ballot(best.acc == amin && best.pos == pmin && best.slot >= 0);
      if (win != 0ull) {
        eslot = __builtin_amdgcn_readlane(best.slot, __ffsll((long long)win) - 1);
        epos = pmin;
      }
    }
    const bool evict = eslot >= 0;                           // eslot == m: the new pair itself
    ins_slot = full ? ((evict && eslot < m) ? eslot : -1) : m;
    // its value row once more (the stream may have passed it): unconditional, from row 0 where no
    // cached pair leaves
    const __amdgpu_buffer_rsrc_t rv = __builtin_amdgcn_make_buffer_rsrc(vc, 0, C * D * (int)sizeof(T), 0x00020000);
    const int er = (evict && eslot < m) ? eslot : 0;
    pv_row = __builtin_amdgcn_raw_buffer_load_b128(rv, lr * 16, er * (D * (int)sizeof(T)), 0);
  }
  value_pass(2 * DEPTH);
  {
    // fold the pending pair into H (Eq. 4; stored by the lead wave), then this head's phi(q) H
    const float f32 = (float)f_lane;
    const __half2 *pvh = reinterpret_cast<const __half2 *>(&pend_v_h);
    const float2 pv01 = __half22float2(pvh[0]), pv23 = __half22float2(pvh[1]);
#pragma unroll
    for (int i = 0; i < HR; ++i) {
      const int r = NHB * i + hb;
      const int rc = r < R ? r : R - 1;
      const float fr = r < R ? __shfl(f32, rc) : 0.f;
      const float pe = __shfl(psie_lane, rc);
      if (pend.fold) {
        hreg[i].x = fmaf(pe, pv01.x, hreg[i].x);
        hreg[i].y = fmaf(pe, pv01.y, hreg[i].y);
        hreg[i].z = fmaf(pe, pv23.x, hreg[i].z);
        hreg[i].w = fmaf(pe, pv23.y, hreg[i].w);
      }
      fh[0] = fmaf(fr, hreg[i].x, fh[0]);
      fh[1] = fmaf(fr, hreg[i].y, fh[1]);
      fh[2] = fmaf(fr, hreg[i].z, fh[2]);
      fh[3] = fmaf(fr, hreg[i].w, fh[3]);
    }
  }
  // The unit's new state, by the lead wave.  No store stands in mid-stream (a wave's memory
  // counter runs in order: a store holds up the rows requested after it): these go out before the
  // last pass, whose rows are requested ahead of them, and through the L2 to memory (a line left
  // dirty there is written back when the kernel ends, before the next launch can start).
  auto state_stores = [&]() __attribute__((always_inline)) {
    if (pend.fold) {                                         // H with the pending pair folded in (Eq. 4)
#pragma unroll
      for (int i = 0; i < HR; ++i) {
        const int r = NHB * i + hb;
        if (r < R) store_wt16(a.H + (size_t)u * R * D, (r * D + col0) * (int)sizeof(float), hreg[i]);
      }
    }
    if (lane < R) {
      if (pend.fold) store_wt(a.z + (size_t)u * R + lane, z_lane);
      if (pend.slot >= 0 && pend.slot < C) store_wt(a.psi + ((size_t)u * C + pend.slot) * R + lane, ppsi_lane);
      store_wt(a.pend_psi + (size_t)u * R + lane, npsi_lane);
    }
#pragma unroll
    for (int i = 0; i < NR2; ++i) {
      const int j = lane + i * kWave;
      if (j < m) {
        if (j != ins_slot) store_wt(a.acc + (size_t)u * C + j, na_[i]);
      } else if (j == m && ins_slot >= 0) {
        store_wt(a.acc + (size_t)u * C + ins_slot, na_[i]);
        store_wt(a.pos + (size_t)u * C + ins_slot, n);
      }
    }
    if (lane == 0) {
      store_wt(a.pend_slot + u, eslot >= 0 ? (eslot < m ? eslot : C) : (m | kPendNoFold));
      if (a.evicted_pos) store_wt(a.evicted_pos + u, eslot >= 0 ? epos : -1);
      store_wt(a.n_seen + u, n + 1);
    }
    if (eslot >= 0 && rb == 0) {
      uint4 row = vnv.raw;
      if (eslot < m) __builtin_memcpy(&row, &pv_row, 16);
      store_wt16(reinterpret_cast<T *>(a.pend_v) + (size_t)u * D, lr * EPL * (int)sizeof(T), row);
    }
  };
  {
    int base = 3 * DEPTH;
    for (; base + DEPTH < nit; base += DEPTH) value_pass(base);
    if (lead) state_stores();
    if (base < nit) value_pass(base);                        // the last pass requests nothing real
  }
  // the appended pair's value row
  if (rb == 0) {
    const float p = s_p[m];
#pragma unroll
    for (int i = 0; i < EPL; ++i) o[i] = fmaf(p, Store<T>::get(vnv, i), o[i]);
  }
  // The RPI row groups hold partial sums of the same 8 columns: reduce-scatter over the first
  // stage (a lane keeps the four columns selected by its bit LPR), all-reduce over the rest,
  // together with the partial phi(q) H of the row subsets.
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const bool hi = lane & LPR;
    const float send = hi ? o[i] : o[i + 4], keep = hi ? o[i + 4] : o[i];
    o[i] = keep + __shfl_xor(send, LPR);
  }
#pragma unroll
  for (int x = 2 * LPR; x < kWave; x *= 2) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      o[i] += __shfl_xor(o[i], x);
      fh[i] += __shfl_xor(fh[i], x);
    }
  }
  // ---- phase 4: this head's output; the new pair goes into its slot once every head is through ------
  if (hb == 0) {
    __half2 res[2];
    res[0] = __floats2half2_rn((float)(pscale * (double)o[0] + lscale * (double)fh[0]), (float)(pscale * (double)o[1] + lscale * (double)fh[1]));
    res[1] = __floats2half2_rn((float)(pscale * (double)o[2] + lscale * (double)fh[2]), (float)(pscale * (double)o[3] + lscale * (double)fh[3]));
    store_wt8(reinterpret_cast<T *>(a.out) + ((size_t)u * G + g) * D + col0, *reinterpret_cast<const uint2 *>(res));
  }
  // the feature-map entries go back empty: this head's, and (lead wave) the key's
  if (parts) {
    for (int e = lane; e < nparts * (rp / 4); e += kWave) {
      store_wt16(a.mlp_out + ((size_t)u * G + g) * nparts * rp, e * 16, uint4{kMlpEmpty, kMlpEmpty, kMlpEmpty, kMlpEmpty});
      if (lead)
        store_wt16(a.mlp_out + ((size_t)a.U * G + u) * nparts * rp, e * 16, uint4{kMlpEmpty, kMlpEmpty, kMlpEmpty, kMlpEmpty});
    }
  }
  // barrier 3: the rows still in a ring are requests past the value stream (out of range, zeros),
  // so every wave that arrives here has all the cache rows it will ever read
#pragma unroll
  for (int j = 0; j < DEPTH; ++j) asm volatile("" ::"v"(buf[j]));
  __builtin_amdgcn_s_barrier();
  if (lead && ins_slot >= 0 && rb == 0) {
    store_wt16(kc + (size_t)ins_slot * D, lr * EPL * (int)sizeof(T), knv.raw);
    store_wt16(vc + (size_t)ins_slot * D, lr * EPL * (int)sizeof(T), vnv.raw);
  }
}

bool gqs_supported(int dtype, int D, int C, int R, int G)
{
  return dtype == LESSDEC_DTYPE_F16 && (D == 64 || D == 128) && R <= 16 && C + 1 <= kGqsMaxRows && G >= 2 &&
         G <= kGqsMaxHeads;
}

bool gqs_takes_parts(int Rp) { return mlp_nparts(Rp) <= kGqsParts; }

// One launch for the whole step: four or eight query heads per unit (the block is then one or two
// feature-map jobs of four waves), parts that fit the registers kept for them, and the kernel form
// that stays within the 128 registers four resident waves per SIMD leave each.
bool gqs_fusable(int D, int C, int Rp, int R, int G)
{
  return (G == 4 || G == 8) && D == 128 && C + 1 <= 2 * kWave && R <= 8 && mlp_nparts(Rp) <= kGqsParts;
}

template <int D, int RM>
static hipError_t launch_step_gqs_t(const StepArgs &a, int G, hipStream_t st, const MlpPartsArgs *fm)
{
  constexpr int kDepth = 7;
  const int rows_cap = (a.C + 2) & ~1;
  const size_t lds = (size_t)G * rows_cap * (2 * sizeof(double) + sizeof(float));
  const unsigned block = (unsigned)(G * kWave);
  const int rows = a.C + 1;
  if (fm) {
    if constexpr (D == 128 && RM == 8) {
      const int per = G / 4;                               // jobs per block
      const unsigned n_mlp = (unsigned)((mlp_parts_gq_jobs(a.Hh, G, a.Rp, a.B) + per - 1) / per);
      const size_t slabs = (size_t)per * mlp_slab_bytes(D), lds_f = lds < slabs ? slabs : lds;
      gqs_step_kernel<D, 2, RM, 6, true><<<n_mlp + (unsigned)a.U, block, lds_f, st>>>(a.k_cache, a.q, a.k, a.C, G, (int)n_mlp,
                                                                                   fm->Wq1, fm->Wk1, fm->Wq2, a);
      return hipGetLastError();
    } else {
      return hipErrorInvalidValue;
    }
  }
  const unsigned grid = (unsigned)a.U;
#define LESSDEC_GQS_LAUNCH(NR2)                                                                                   \
  gqs_step_kernel<D, NR2, RM, kDepth, false><<<grid, block, lds, st>>>(a.k_cache, a.q, a.k, a.C, G, 0, nullptr, nullptr, \
                                                                       nullptr, a)
  if (rows <= 2 * kWave) LESSDEC_GQS_LAUNCH(2);
  else if (rows <= 4 * kWave) LESSDEC_GQS_LAUNCH(4);
  else LESSDEC_GQS_LAUNCH(kGqsMaxRows / kWave);
#undef LESSDEC_GQS_LAUNCH
  return hipGetLastError();
}

hipError_t launch_step_gqs(const StepArgs &a, int G, int D, hipStream_t st, const MlpPartsArgs *fm)
{
  if (fm && !gqs_fusable(D, a.C, a.Rp, a.R, G)) return hipErrorInvalidValue;
  if (D == 64) return launch_step_gqs_t<64, 16>(a, G, st, fm);
  return a.R <= 8 ? launch_step_gqs_t<128, 8>(a, G, st, fm) : launch_step_gqs_t<128, 16>(a, G, st, fm);
}

}  // namespace lessdec
