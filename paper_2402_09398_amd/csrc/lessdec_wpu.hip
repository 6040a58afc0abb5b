// Decode step (Algorithm 1), streaming form: one wave per unit.  The layer-2 sums of the step's
// feature maps come from the feature-map jobs (lessdec_mlp.h): the first workgroups of this very
// launch (FUSED) or the launch before it (lessdec_mlp.hip).
#include "lessdec_mlp.h"
#include "lessdec_wave.h"

namespace lessdec {

constexpr int kWpuUnits = 8;        // units (waves) per block, at most
constexpr int kWpuMaxRows = 512;    // C + 1 at most
constexpr int kWpuSplitWaves = 3072; // a unit's rows are split over more waves while the launch stays below this many
constexpr int kWpuFusedUnits = 4;   // FUSED: units (waves) per block, the size of a feature-map job
constexpr int kWpuSpinLimit = 1 << 14;   // FUSED: polls of the feature-map entries before a wave gives up

// =====================================================================================
// A block is up to 8 waves = 8 units that share a head (4 when FUSED): consecutive batch rows of
// head h (head fastest in blockIdx, so with Hh a multiple of 8 the units of a head run on
// the XCD whose L2 holds the feature-map sums written for them).  The waves of a block share
// nothing and never meet at a barrier; each is on its own from the first instruction.
// (SPLIT, for launches with few units: the block is one unit and its waves take every nw-th
// load of each stream.  They meet twice: when the scores are complete, after which each wave
// works out phase 2 for itself and only the lead wave stores; and when the partial outputs
// are complete, which the lead wave adds in wave order and finishes.)
//
// A cache row is LPR = D / 8 lanes of 16 bytes, one load instruction covers RPI = 64 / LPR
// rows.  The rows of K and then of V pass through a ring of DEPTH registers per lane: each
// load is consumed in issue order and its register re-used for the load DEPTH places
// ahead, so the number of bytes in flight is constant (DEPTH KiB per wave) from the first
// key row to the last value row.  The K part of the stream is padded to a multiple of DEPTH so
// that ring positions are compile-time constants; loads past the live rows are requested out of
// the buffer's range, which returns zeros and moves no data.
//
// Phase 1  scores s_j = q . K_j / sqrt(D) of the live slots and the appended key as they
//          arrive: exact fp32 products added in fp64, reduced over the LPR lanes of a row by
//          DPP, parked in the LDS.  (!FUSED: after the first pass over the ring, phi(q) and
//          psi(k) are finished from their layer-2 sums: last activations of Eq. 1 and Eq. 2, W3,
//          in fp64.)
// Phase 2  in parts.  First what the value stream needs: lane j owns rows j, j + 64, ..: the
//          maximum M and the exponentials e^{s_j - M}, which weight the value rows as they are
//          (the sum is scaled by 1 / den at the output).  The rest is one dependent chain of fp64
//          reductions and is worked off between the first three passes of the value stream, each
//          part while the rows requested by the pass before it are on their way:
//          (a) FUSED: the feature maps from their entries; the fold of the pair the previous step
//          discarded into z (Eq. 5), which Eq. 3 of this step must already see; phi(q) z^T and
//          the denominator of Eq. 3; (b) H2O score accumulation and the eviction argmin
//          (Sec. 2.1); the value row of the discarded slot is asked for once more (the stream
//          may have passed it); (c) the fold of the pending pair into H (Eq. 4) and phi(q) H.
// Phase 3  e^{s - M} . V in fp32 as the value rows arrive; the RPI partial rows are combined by a
//          reduce-scatter that leaves each lane with the four output columns it also holds of H.
// Stores   none in mid-stream: a wave's memory counter runs in order, so a store would hold up
//          every row requested after it until it is acknowledged.  The unit's new state (H, z,
//          psi, accumulated scores, positions, counters, the parked pair, the feature-map entries
//          handed back empty) goes out before the last pass of the value stream, whose rows are
//          requested ahead of it; the output out = (sum / den) + phi(q) H / den (Eq. 3) and the
//          new pair into the freed slot (Sec. 3.2) at the very end.  All of them go through the
//          L2 to memory (system scope): a line left dirty in an L2 is written back when the
//          kernel ends, before the next launch can start.
//
// FUSED: the whole step in one launch.  The first n_mlp blocks are the step's feature-map jobs
// (mlp_parts_block: four waves a job, or two for batches of up to 32 rows), the blocks behind them
// the attention waves, four units per block (SPLIT: a unit over four or eight waves).  Workgroups
// are dispatched in index order, so every job is on a compute unit before any attention wave that
// may wait for it, and the jobs wait for nothing: no cycle of waits exists.
// The layer-2 sums travel through the exchange array as 32-bit entries, written through by the
// jobs and read with device-scope loads.  An entry that no job has written yet holds kMlpEmpty:
// an attention wave requests its entries before the last pass of the key stream (by then the jobs
// are normally long done), looks at them after the first pass of the value stream, asks again
// while any is still empty, and puts kMlpEmpty back with its other stores, so that the array is
// all empty again when the step ends.  (The form that gets its entries from a launch before it,
// !FUSED, empties them as well: either form can follow the other on one workspace.)  A wave that
// has polled kWpuSpinLimit times gives up and computes with the empty entries, which are NaN: the
// outputs of its unit then show it.
// =====================================================================================
template <int D, int NR2, int RM, int DEPTH, bool SPLIT, bool FUSED>
__global__ __launch_bounds__((FUSED && !(SPLIT && NR2 > 2) ? kWpuFusedUnits : kWpuUnits) * kWave,
                             FUSED && !(SPLIT && NR2 > 2) ? ((SPLIT || NR2 > 2 || RM > 8) ? 3 : 4) : 1) void wpu_step_kernel(
    void *k_cache_, const void *q_, const void *k_, int crp_, int hb_, int xs_, int n_mlp_, const void *Wq1_,
    const void *Wk1_, const void *Wq2_, const StepArgs a)
{
  // The first arguments repeat what the head of the kernel needs to request the first rows:
  // scalar arguments can be preloaded into registers by the launch (the compile flag asks for
  // it), the struct has to be fetched.  crp_ = C | R << 12 | R' << 19, hb_ = Hh | B << 16, xs_ = the
  // distance in elements between the q / k / v / out rows of consecutive units.
  using T = __half;
  constexpr int EPL = 8;                   // elements per lane
  constexpr int LPR = D / EPL;             // lanes per row
  constexpr int RPI = kWave / LPR;         // rows per load instruction
  constexpr int NP = 8;                    // feature-map parts requested up front (R' <= 512)
  using Vec = typename Store<T>::Vec;

  extern __shared__ __attribute__((aligned(16))) double dyn[];

  const int C = crp_ & 0xfff, R = (crp_ >> 12) & 0x7f, Rp = crp_ >> 19, Hh = hb_ & 0xffff, B_ = (int)((unsigned)hb_ >> 16);
  const int wave = __builtin_amdgcn_readfirstlane((int)threadIdx.x >> 6);
  const int lane = threadIdx.x & 63;
  // bits 0..23: feature-map blocks; 24..29: waves per block (the block size itself would have to be
  // fetched from memory before anything else could be asked for); 30..: groups of four waves in a
  // feature-map block, minus one
  const int n_mlp = n_mlp_ & 0xffffff;
  if constexpr (FUSED) {
    if ((int)blockIdx.x < n_mlp) {
      // a block of eight waves (a unit's rows over eight waves) is two groups of four; the count
      // comes with the (preloaded) arguments: the block size would have to be fetched first, a
      // round trip to memory ahead of a job that is a chain of them
      const int groups = 1 + (int)((unsigned)n_mlp_ >> 30), grp4 = wave >> 2;
      mlp_parts_block<D, true>(reinterpret_cast<const __half *>(q_), reinterpret_cast<const __half *>(k_),
                               reinterpret_cast<const __half *>(Wq1_), reinterpret_cast<const __half *>(Wk1_),
                               reinterpret_cast<const __half *>(Wq2_), reinterpret_cast<const __half *>(a.Wk2), Hh, Rp, R,
                               B_, xs_, a.mlp_out, (int)blockIdx.x * groups + grp4,
                               reinterpret_cast<unsigned char *>(dyn) + grp4 * (4 / mlp_parts_nwj(B_)) * mlp_slab_bytes(D),
                               wave & 3, lane);
      return;
    }
  }
  const int bid = FUSED ? (int)blockIdx.x - n_mlp : (int)blockIdx.x;
  const int lr = lane % LPR, rb = lane / LPR;
  const int h = bid % Hh, chunk = bid / Hh;
  const int upb = (n_mlp_ >> 24) & 0x3f;                     // waves in this block
  // SPLIT: the waves of the block share one unit, wave w taking every nw-th load of each
  // stream; otherwise a wave is a unit.
  const int nw = SPLIT ? upb : 1, wv = SPLIT ? wave : 0;
  const bool lead = !SPLIT || wave == 0;                     // the wave that writes the unit's state
  const int bb = SPLIT ? chunk : chunk * upb + wave;
  if (bb >= B_) return;                                      // uniform over the unit's waves
  const int u = bb * Hh + h;
  const int rows_cap = (C + 2) & ~1;
  double *s_sc = dyn + (SPLIT ? 0 : (size_t)wave * rows_cap);                      // [C+1] scores
  float *s_p = reinterpret_cast<float *>(dyn + (SPLIT ? 1 : (size_t)upb) * rows_cap) + (size_t)wave * rows_cap;
  float *s_o = reinterpret_cast<float *>(dyn + rows_cap) + (size_t)upb * rows_cap;  // SPLIT: [nw][D] partial outputs

  T *kc = reinterpret_cast<T *>(k_cache_) + (size_t)u * C * D;
  T *vc = reinterpret_cast<T *>(a.v_cache) + (size_t)u * C * D;
  const T *qn = reinterpret_cast<const T *>(q_) + (size_t)u * xs_;
  const T *kn = reinterpret_cast<const T *>(k_) + (size_t)u * xs_;
  const T *vn = reinterpret_cast<const T *>(a.v) + (size_t)u * xs_;

  // ---- requests, in the order they are wanted back ------------------------------------------------
  // Every load here is unconditional, from a clamped address where the wanted one may not
  // exist: a load under a condition makes the first use of anything requested before it
  // wait for it as well, and a wait in mid-stream drains the ring.
  // 1. the step's rows and the head of the key stream (bounded by the capacity: the number of
  //    live rows is not known yet; rows past them are fetched only while the cache fills)
  const Vec qv = load_vec<T>(qn + lr * EPL);
  const Vec knv = load_vec<T>(kn + lr * EPL);
  u4v buf[DEPTH];
  {
    const __amdgpu_buffer_rsrc_t rk =
        __builtin_amdgcn_make_buffer_rsrc(kc, 0, C * D * (int)sizeof(T), 0x00020000);
#pragma unroll
    for (int j = 0; j < DEPTH; ++j)
      buf[j] = __builtin_amdgcn_raw_buffer_load_b128(rk, lane * 16, (j * nw + wv) * (kWave * 16), 2 /* nt */);
  }
  __builtin_amdgcn_sched_barrier(0);
  // 2. layer-2 sums of the two feature maps by parts (lane r + 16 i reads what lane r reads),
  //    row r of W3
  const int nparts = mlp_nparts(Rp), rp = mlp_entry_stride(R);
  const int rl = (lane & 15) < R ? (lane & 15) : R - 1;
  float pq[NP], pk[NP];
  // FUSED: device-scope loads, the entries may come from another XCD in this very launch
  auto request_parts = [&]() {
#pragma unroll
    for (int p = 0; p < NP; ++p) {
      const int pc = p < nparts ? p : nparts - 1;
      const float *eq = a.mlp_parts + ((size_t)u * 2 * nparts + pc) * rp + rl;
      const float *ek = a.mlp_parts + (((size_t)u * 2 + 1) * nparts + pc) * rp + rl;
      if constexpr (FUSED) {
        pq[p] = __hip_atomic_load(eq, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        pk[p] = __hip_atomic_load(ek, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      } else {
        pq[p] = *eq;
        pk[p] = *ek;
      }
    }
  };
  if constexpr (!FUSED) request_parts();
  __half w3[RM];
  {
    const __half *w3row = reinterpret_cast<const __half *>(a.Wk3) + ((size_t)h * R + rl) * R;
    if (RM == 8 && R == 8) {                                 // a row is one aligned 16-byte load
      const uint4 raw = *reinterpret_cast<const uint4 *>(w3row);
      __builtin_memcpy(w3, &raw, 16);
    } else {
#pragma unroll
      for (int j = 0; j < RM; ++j) w3[j] = w3row[j < R ? j : R - 1];
    }
  }
  // 3. unit state (wanted from phase 2 on)
  const int n = sane_n_seen(a.n_seen[u]);
  const Pending pend = decode_pending(a.pend_slot[u], C);
  const int m = n < C ? n : C;          // live slots are 0..m-1 (slots fill in order)
  const int rows = m + 1;               // + the appended pair (K', V' of Eq. 3)
  const bool full = (m == C);
  // (accumulated scores and positions: a single wave asks for them in phase 2, two passes of the
  // value stream before it needs them; waves that share a unit must have them before they meet,
  // since the lead wave stores the new ones after that)
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
  if constexpr (SPLIT) request_scores();
  double z_lane = a.z[(size_t)u * R + rl];                   // lane r < R
  const float ppsi_lane = a.pend_psi[(size_t)u * R + rl];
  float psie_lane = a.psi[((size_t)u * C + (pend.slot >= 0 && pend.slot < C ? pend.slot : 0)) * R + rl];
  __builtin_amdgcn_sched_barrier(0);

  // The stream: position s < nitp is load s of K, position nitp + t is load t of V.
  const int nl = (rows + RPI - 1) / RPI;                     // load instructions per stream
  const int nit = SPLIT ? (nl > wv ? (nl - wv + nw - 1) / nw : 1) : nl;   // this wave's share (>= 1)
  const int nitp = (nit + DEPTH - 1) / DEPTH * DEPTH;        // K part of the stream, padded
  const int live_bytes = m * D * (int)sizeof(T);
  auto issue = [&](int s) -> u4v {                           // s is wave-uniform
    const bool isk = s < nitp;
    const __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc(isk ? kc : vc, 0, live_bytes, 0x00020000);
    return __builtin_amdgcn_raw_buffer_load_b128(rs, lane * 16, ((isk ? s : s - nitp) * nw + wv) * (kWave * 16), 2 /* nt */);
  };

  // ---- phase 1: scores as the key rows arrive; the feature maps after the first pass ------------
  double f_lane = 0.0;                   // phi(q), lane r < R
  float npsi_lane = 0.f;                 // psi(k) of this step's key, lane r < R
  const double inv_sqrt_d = 1.0 / sqrt((double)D);        // folded at compile time
  u4v knu;
  __builtin_memcpy(&knu, &knv.raw, 16);
  auto key_pass = [&](int base) {
#pragma unroll
      for (int j = 0; j < DEPTH; ++j) {
        const int s = base + j;
        if (s < nit) {
          const int r = (s * nw + wv) * RPI + rb;
          const u4v kraw = (r == m) ? knu : buf[j];       // r == m: the appended key
          Vec kv;
          __builtin_memcpy(&kv.raw, &kraw, 16);
          // a product of two halves is exact in fp32 (22 bits), so fp32 multiply, widen, fp64 add
          // gives the bits of an fp64 multiply-add with two conversions fewer per element
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
    // Both feature maps from their layer-2 sums, and the entries handed back empty.
    auto finish_maps = [&]() {
      double sq = 0.0, sk = 0.0;
#pragma unroll
      for (int p = 0; p < NP; ++p) {
        if (p < nparts) {
          sq += (double)pq[p];
          sk += (double)pk[p];
        }
      }
      for (int p = NP; p < nparts; ++p) {                  // hidden widths above 512 (never FUSED)
        sq += (double)a.mlp_parts[((size_t)u * 2 * nparts + p) * rp + rl];
        sk += (double)a.mlp_parts[(((size_t)u * 2 + 1) * nparts + p) * rp + rl];
      }
      f_lane = lane < R ? fabs(gelu_poly_f64(sq)) : 0.0;   // last activation of Eq. 1
      const double h2 = gelu_poly_f64(sk);                 // lane r < R; Eq. 2: |W3 gelu(.)|
      double acc3 = 0.0;
#pragma unroll
      for (int j = 0; j < RM; ++j)
        if (j < R) acc3 = fma(readlane_v(h2, j), (double)__half2float(w3[j]), acc3);
      npsi_lane = (float)fabs(acc3);
    };
    if constexpr (FUSED) {
      // The entries are requested before the last pass of the key stream and first looked at after
      // the sparse part of phase 2: that hides their way from memory.  (Asking a pass earlier
      // still keeps their sixteen registers live through two passes and makes the kernel spill.)
      int base = 0;
      for (; base + DEPTH < nitp; base += DEPTH) key_pass(base);
      request_parts();
      key_pass(base);
    } else {
      int base = 0;
      do {                                                 // nitp >= DEPTH
        key_pass(base);
        // The parts have been back for a while (they were requested before the loads this pass
        // re-issued): finish both feature maps here, where nothing is waiting for anything.
        if (base == 0) finish_maps();
      } while ((base += DEPTH) < nitp);
    }

  // ---- requests behind the keys: what the value stream and the output want --------------------------
  // This lane's share of H and of the pending value row, wanted after the value stream: four
  // consecutive columns (those the reduce-scatter of phase 3 leaves it with) of every NHB-th
  // row, so that one 16-byte load per lane covers NHB whole rows of H per instruction.
  // (FUSED: requested inside phase 2, once the feature-map entries have given their registers back.)
  constexpr int NHB = RPI / 2, HR = RM / NHB;
  const int col0 = lr * EPL + ((lane & LPR) ? 4 : 0);
  const int hb = lane / (2 * LPR);                           // which rows: r = NHB * i + hb
  Vec vnv;
  float4 hreg[HR];
  uint2 pend_v_h;
  auto request_tail = [&]() {
    vnv = load_vec<T>(vn + lr * EPL);
#pragma unroll
    for (int i = 0; i < HR; ++i) {
      const int r = NHB * i + hb;
      hreg[i] = *reinterpret_cast<const float4 *>(a.H + ((size_t)u * R + (r < R ? r : R - 1)) * D + col0);
    }
    pend_v_h = *reinterpret_cast<const uint2 *>(reinterpret_cast<const T *>(a.pend_v) + (size_t)u * D + col0);
  };
  if constexpr (!FUSED) request_tail();
  if constexpr (SPLIT) {
    // Every wave works out phase 2 for itself from the shared scores; only the lead wave
    // stores.  Its stores must not overtake another wave's loads of the same state: have
    // those loads back before the waves meet (the value rows requested after them stay in
    // flight), then meet with the scores visible.
#pragma unroll
    for (int i = 0; i < NR2; ++i) asm volatile("" ::"v"(acc_pre[i]), "v"(pos_pre[i]));
    asm volatile("" ::"v"(z_lane), "v"(ppsi_lane), "v"(psie_lane));
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
  } else {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
  }

  int eslot = -1, ins_slot = -1;
  double lscale = 0.0, pscale = 0.0, ascale = 0.0;
  // ---- phase 2, first part: what the value stream needs, the exponentials e^{s_j - M} ------------
  // The value rows are weighted with the exponentials as they are and the sum is scaled by
  // 1 / den at the end, so the stream goes on while the rest of phase 2 (the low-rank term, the
  // denominator, the H2O bookkeeping and the choice of the discarded pair: one dependent chain of
  // fp64 reductions) is worked through in three parts between its first passes, each while the
  // rows requested by the pass before it are on their way.
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

  // second part: low-rank term and denominator
  auto denominators = [&]() __attribute__((always_inline)) {
    double S = 0.0;
#pragma unroll
    for (int i = 0; i < NR2; ++i) S += sc[i];
    S = wave_allreduce(S, OpAdd{});                         // sparse part of the denominator, shifted
    if constexpr (FUSED) {
      // the feature-map entries, requested during the key stream: all there?
      // (every entry is looked at, without a way out after the first empty one: a way out would
      // leave the later requests unaccounted for, and whoever uses them next would wait for
      // everything in flight)
      auto have_all = [&]() {
        unsigned missing = 0;
#pragma unroll
        for (int p = 0; p < NP; ++p)
          missing |= (unsigned)(__float_as_uint(pq[p]) == kMlpEmpty) | (unsigned)(__float_as_uint(pk[p]) == kMlpEmpty);
        return __all(missing == 0u) != 0;
      };
      // (the first look stands outside the loop: a look at the loop's head would have to wait
      // for whatever the loop body may have requested, which is everything in flight)
      bool have = have_all();
      for (int spin = 0; !have && spin < kWpuSpinLimit; ++spin) {
        __builtin_amdgcn_s_sleep(32);
        request_parts();
        have = have_all();
      }
      finish_maps();
      request_tail();
    }
    // pending fold of z (Eq. 5), then phi(q) z^T
    if (lane >= R) z_lane = 0.0;
    if (!pend.fold) psie_lane = 0.f;
    else if (pend.slot >= C) psie_lane = ppsi_lane;        // the previous step discarded its own pair
    if (lane < R && pend.fold) z_lane += (double)psie_lane;
    const double fz = wave_allreduce(f_lane * z_lane, OpAdd{});
    // den = phi(q) z^T + sum_j e^{s_j}, in whichever scaling cannot overflow:
    //   M > 0 (or no low-rank term): everything times e^{-M};  M <= 0: unscaled, e^{M} <= 1
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
    ascale = pscale;
    if (a.flags & LESSDEC_FLAG_SPARSE_DENOM) ascale = 1.0 / S;
    if constexpr (!SPLIT) request_scores();
  };

  // third part: H2O bookkeeping and the choice of the discarded pair; its value row is asked for
  // again (the stream may have passed it already) and parked in phase 4
  u4v pv_row = {0u, 0u, 0u, 0u};
  int epos = -1;
  auto bookkeeping = [&]() __attribute__((always_inline)) {
    const bool lambda = (a.flags & LESSDEC_FLAG_LAMBDA) != 0;
    Cand best = cand_none();
#pragma unroll
    for (int i = 0; i < NR2; ++i) {
      const int j = lane + i * kWave;
      if (j < rows) {
        double na = sc[i] * ascale;
        int pj = n;
        if (j < m) {
          na += acc_pre[i];
          pj = pos_pre[i];
        }
        sc[i] = na;
        if (full) {
          // H2O: every pair that is not among the Nr most recent competes on its score;
          // Lambda-masking: the first Nh tokens never leave and the oldest of the others does
          const bool is_cand = (j < m) ? (pj <= n - a.Nr && (!lambda || pj >= a.Nh)) : (a.Nr == 0);
          const Cand cnd{lambda ? 0.0 : na, pj, j};
          if (is_cand && cand_less(cnd, best)) best = cnd;
        }
      }
    }
    // argmin over (score, position): smallest score, then the oldest among equals
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
    ins_slot = full ? ((evict && eslot < m) ? eslot : -1) : m;
    {
      // unconditional, from row 0 where no cached pair leaves
      const __amdgpu_buffer_rsrc_t rv = __builtin_amdgcn_make_buffer_rsrc(vc, 0, C * D * (int)sizeof(T), 0x00020000);
      const int er = (evict && eslot < m) ? eslot : 0;
      pv_row = __builtin_amdgcn_raw_buffer_load_b128(rv, lr * 16, er * (D * (int)sizeof(T)), 0);
    }
  };

  // ---- phase 3: e^{s - M} . V as the value rows arrive ------------------------------------------------
  float o[EPL];
#pragma unroll
  for (int i = 0; i < EPL; ++i) o[i] = 0.f;
  float fh[4] = {0.f, 0.f, 0.f, 0.f};                        // phi(q) H, this lane's columns and rows
  auto value_pass = [&](int base) __attribute__((always_inline)) {
#pragma unroll
    for (int j = 0; j < DEPTH; ++j) {
      const int s = base + j;
      if (s < nit) {
        const int r = (s * nw + wv) * RPI + rb;
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
  // fourth part: H and the pending value row are back (requested before the loads of the pass
  // before this): fold the pending pair into H (Eq. 4) and send H on its way while the value rows
  // still stream, then phi(q) H for this lane's columns and rows.
  auto fold_state = [&]() __attribute__((always_inline)) {
    const float f32 = (float)f_lane;
    const __half2 *pvh = reinterpret_cast<const __half2 *>(&pend_v_h);
    const float2 pv01 = __half22float2(pvh[0]), pv23 = __half22float2(pvh[1]);
#pragma unroll
    for (int i = 0; i < HR; ++i) {
      const int r = NHB * i + hb;                            // differs between the halves of the wave
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
  };
  // Passes past the end of the stream consume nothing and request rows outside the buffer's
  // range, which fetches nothing: the three passes always run, so that no load sits under a
  // condition.
  value_pass(0);
  denominators();
  value_pass(DEPTH);
  bookkeeping();
  value_pass(2 * DEPTH);
  fold_state();
  // The unit's new state.  Its stores stand behind the last load that fetches anything: the memory
  // counter of a wave runs in order, so a store in mid-stream holds up every row requested after
  // it until the store has been acknowledged.  The rows of the last pass are requested before
  // these stores and do not wait for them.  (SPLIT: the lead wave's.)
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
        if (j != ins_slot) store_wt(a.acc + (size_t)u * C + j, sc[i]);
      } else if (j == m && ins_slot >= 0) {
        store_wt(a.acc + (size_t)u * C + ins_slot, sc[i]);
        store_wt(a.pos + (size_t)u * C + ins_slot, n);
      }
    }
    if (lane == 0) {
      // what the next step has to finish: fold of the discarded pair and / or the slot write
      store_wt(a.pend_slot + u, eslot >= 0 ? (eslot < m ? eslot : C) : (m | kPendNoFold));
      if (a.evicted_pos) store_wt(a.evicted_pos + u, eslot >= 0 ? epos : -1);
      store_wt(a.n_seen + u, n + 1);
    }
    if constexpr (!SPLIT) {
      // the feature-map entries go back empty (the unit's 2 * nparts entries lie together)
      for (int e = lane; e < 2 * nparts * (rp / 4); e += kWave)
        store_wt16(a.mlp_out + (size_t)u * 2 * nparts * rp, e * 16, uint4{kMlpEmpty, kMlpEmpty, kMlpEmpty, kMlpEmpty});
    }
    // the discarded pair's value row, parked for the next step's fold (before the insert below
    // overwrites the row it was read from)
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
  if (lead && rb == 0) {
    const float p = s_p[m];
#pragma unroll
    for (int i = 0; i < EPL; ++i) o[i] = fmaf(p, Store<T>::get(vnv, i), o[i]);
  }
  {
    // The RPI row groups hold partial sums of the same 8 columns.  First stage (partner at
    // distance LPR): reduce-scatter, a lane keeps the four columns selected by its bit LPR;
    // remaining stages: all-reduce, together with the partial phi(q) H of the row subsets.
    {
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
    }

    if constexpr (SPLIT) {
      // the waves' partial p . V meet in the LDS and the lead wave adds them in wave order
      if (hb == 0) *reinterpret_cast<float4 *>(s_o + (size_t)wave * D + col0) = float4{o[0], o[1], o[2], o[3]};
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
      __builtin_amdgcn_s_barrier();
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
      if (!lead) return;
      const float4 first = *reinterpret_cast<const float4 *>(s_o + col0);
      o[0] = first.x; o[1] = first.y; o[2] = first.z; o[3] = first.w;
      for (int w = 1; w < nw; ++w) {
        const float4 part = *reinterpret_cast<const float4 *>(s_o + (size_t)w * D + col0);
        o[0] += part.x; o[1] += part.y; o[2] += part.z; o[3] += part.w;
      }
    }

    // ---- phase 4: output and the in-place insert (SPLIT: only the lead wave gets here) -------------
    if constexpr (SPLIT) {
      // the feature-map entries go back empty, now that every wave of the unit has read them
      for (int e = lane; e < 2 * nparts * (rp / 4); e += kWave)
        store_wt16(a.mlp_out + (size_t)u * 2 * nparts * rp, e * 16, uint4{kMlpEmpty, kMlpEmpty, kMlpEmpty, kMlpEmpty});
    }
    if (hb == 0) {
      __half2 res[2];
      res[0] = __floats2half2_rn((float)(pscale * (double)o[0] + lscale * (double)fh[0]), (float)(pscale * (double)o[1] + lscale * (double)fh[1]));
      res[1] = __floats2half2_rn((float)(pscale * (double)o[2] + lscale * (double)fh[2]), (float)(pscale * (double)o[3] + lscale * (double)fh[3]));
      store_wt8(reinterpret_cast<T *>(a.out) + (size_t)u * xs_ + col0, *reinterpret_cast<const uint2 *>(res));
    }
    if (ins_slot >= 0 && rb == 0) {
      store_wt16(kc + (size_t)ins_slot * D, lr * EPL * (int)sizeof(T), knv.raw);
      store_wt16(vc + (size_t)ins_slot * D, lr * EPL * (int)sizeof(T), vnv.raw);
    }
  }
}

// (batch and heads below 65536 each: the kernel takes them packed in one preloaded argument)
bool wpu_supported(int dtype, int D, int C, int Rp, int R)
{
  return dtype == LESSDEC_DTYPE_F16 && (D == 64 || D == 128) && R <= 16 && Rp % 32 == 0 && Rp >= 32 &&
         C + 1 <= kWpuMaxRows;
}

__global__ void fill_empty_kernel(unsigned *p, size_t count)
{
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < count; i += (size_t)gridDim.x * blockDim.x)
    p[i] = kMlpEmpty;
}

hipError_t launch_fill_empty(float *parts, size_t count, hipStream_t st)
{
  if (count == 0) return hipSuccess;
  const unsigned grid = (unsigned)((count + 255) / 256 < 2048 ? (count + 255) / 256 : 2048);
  fill_empty_kernel<<<grid, 256, 0, st>>>(reinterpret_cast<unsigned *>(parts), count);
  return hipGetLastError();
}

static inline int pack_crp(const StepArgs &a) { return a.C | (a.R << 12) | (a.Rp << 19); }

template <int D, int RM, bool SPLIT, bool FUSED>
static hipError_t launch_step_wpu_s(const StepArgs &a, int upb, hipStream_t st, const MlpPartsArgs *fm)
{
  constexpr int kDepth = FUSED ? 6 : 7;
  const int rows_cap = (a.C + 2) & ~1;
  size_t lds = (size_t)(SPLIT ? 1 : upb) * rows_cap * sizeof(double) + (size_t)upb * rows_cap * sizeof(float);
  if (SPLIT) lds += (size_t)upb * D * sizeof(float);
  const int groups = FUSED && upb > 4 ? upb / 4 : 1;       // groups of four waves a feature-map block has
  const unsigned n_mlp = FUSED ? (unsigned)((mlp_parts_blocks(a.Hh, a.Rp, a.B) + groups - 1) / groups) : 0u;
  if (FUSED) {                                             // the feature-map blocks stage their weights there
    const size_t slabs = (size_t)groups * (4 / mlp_parts_nwj(a.B)) * mlp_slab_bytes(D);
    if (lds < slabs) lds = slabs;
  }
  const unsigned grid = n_mlp + (unsigned)(a.Hh * (SPLIT ? a.B : (a.B + upb - 1) / upb));
  const unsigned block = (unsigned)(upb * kWave);
  const int rows = a.C + 1;
  const int crp = pack_crp(a), hb = a.Hh | (a.B << 16), xs = a.x_stride ? a.x_stride : D;
  const void *wq1 = fm ? fm->Wq1 : nullptr, *wk1 = fm ? fm->Wk1 : nullptr, *wq2 = fm ? fm->Wq2 : nullptr;
  // (more than 64 KiB of LDS per block has to be asked for: a setting of the kernel, no allocation)
#define LESSDEC_WPU_LAUNCH(NR2)                                                                                  \
  do {                                                                                                           \
    static size_t asked[64];                               /* per kernel form and device: granted so far */      \
    int dev = 0;                                                                                                 \
    if (lds > (size_t)64 * 1024 && (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64))                   \
      return hipErrorInvalidDevice;                                                                              \
    if (lds > (size_t)64 * 1024 && lds > asked[dev]) {                                                           \
      if (hipFuncSetAttribute(reinterpret_cast<const void *>(&wpu_step_kernel<D, NR2, RM, kDepth, SPLIT, FUSED>),    \
                              hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess)               \
        return hipErrorInvalidValue;                                                                             \
      asked[dev] = lds;                                                                                          \
    }                                                                                                            \
    wpu_step_kernel<D, NR2, RM, kDepth, SPLIT, FUSED><<<grid, block, lds, st>>>(a.k_cache, a.q, a.k, crp, hb, xs,  \
                                                                                (int)(n_mlp | (unsigned)upb << 24 | (unsigned)(groups - 1) << 30), wq1, wk1, wq2, a); \
  } while (0)
  if (rows <= 2 * kWave) LESSDEC_WPU_LAUNCH(2);
  else if (rows <= 4 * kWave) LESSDEC_WPU_LAUNCH(4);
  else LESSDEC_WPU_LAUNCH(kWpuMaxRows / kWave);
#undef LESSDEC_WPU_LAUNCH
  return hipGetLastError();
}

// Number of waves a unit's rows are split over (1: a wave per unit).
static int wpu_split_waves(long units, int D, int C)
{
  const int nl = (C + 1 + (kWave / (D / 8)) - 1) / (kWave / (D / 8));   // loads per stream
  int nw = 1;
  while (nw < kWpuUnits && units * nw * 2 <= kWpuSplitWaves && nl >= 8 * nw) nw *= 2;
  return nw;
}

// One launch for the whole step: either a wave per unit and enough units that the feature-map
// jobs and the attention waves fill the chip together, or a unit's rows split over four or eight
// waves (the block is then one or two groups of a job's four waves; few units, where a launch of its
// own for the feature maps is a third of the step); parts that fit the registers kept for them, and a shape whose
// kernel stays within the registers that four (split: three) resident waves per SIMD leave each
// (at most 128 rows and rank 8: the larger forms spill).
bool wpu_fusable(int B, int Hh, int D, int C, int Rp, int R)
{
  const long units = (long)B * Hh;
  const int nw = wpu_split_waves(units, D, C);
  if (mlp_nparts(Rp) > 8 || Rp >= 4096 || D != 128) return false;
  if ((long)Hh * 2 * mlp_nparts(Rp) * ((B + 31) / 32) >= (1L << 24)) return false;   // the block count travels in 24 bits
  if (nw == 4) return C + 1 <= 2 * kWave && R <= 8;
  if (nw == 8) return C + 1 > 2 * kWave && R <= 8;       // (the form for blocks of eight waves is that of more than 128 rows)
  return units >= 1024 && C + 1 <= 4 * kWave;
}

// Launch shape.  With thousands of units a wave per unit saturates the memory system; with
// few, a step is bounded by how fast one wave can work through its rows, so the rows of a
// unit are split over 2, 4 or 8 waves, while each keeps at least four loads per stream and
// the launch stays below kWpuSplitWaves waves (measured: 1280 units gain from two waves
// each, 2048 units lose).  Without a split, 8 units share a block when that still gives
// every compute unit a block, fewer for small batches.
template <int D, int RM>
static hipError_t launch_step_wpu_t(const StepArgs &a, hipStream_t st, const MlpPartsArgs *fm)
{
  const long units = (long)a.B * a.Hh;
  const int nw = wpu_split_waves(units, D, a.C);
  if (fm) {
    if constexpr (D == 128) {
      if constexpr (RM == 8)
        if (nw == 4 || nw == 8) return launch_step_wpu_s<D, RM, true, true>(a, nw, st, fm);
      return launch_step_wpu_s<D, RM, false, true>(a, kWpuFusedUnits, st, fm);
    } else {
      return hipErrorInvalidValue;
    }
  }
  if (nw > 1) return launch_step_wpu_s<D, RM, true, false>(a, nw, st, nullptr);
  int upb = kWpuUnits;
  while (upb > 1 && a.Hh * ((a.B + upb - 1) / upb) < 256) upb >>= 1;
  return launch_step_wpu_s<D, RM, false, false>(a, upb, st, nullptr);
}

hipError_t launch_step_wpu(const StepArgs &a, int D, hipStream_t st, const MlpPartsArgs *fm)
{
  if (fm && !wpu_fusable(a.B, a.Hh, D, a.C, a.Rp, a.R)) return hipErrorInvalidValue;
  if (D == 64) return launch_step_wpu_t<64, 16>(a, st, fm);
  return a.R <= 8 ? launch_step_wpu_t<128, 8>(a, st, fm) : launch_step_wpu_t<128, 16>(a, st, fm);
}

}  // namespace lessdec
