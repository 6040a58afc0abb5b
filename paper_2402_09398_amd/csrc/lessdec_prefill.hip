// Prompt phase: regular causal attention (remark after Eq. 3), H2O scores of the prompt
// tokens (column sums of the attention matrix), one-shot cut to the budget, and the
// low-rank state of everything cut away (Eq. 6).
//
// The scores decide which tokens are kept, so Q K^T runs in fp64 on the matrix cores
// (v_mfma_f64_16x16x4_f64).  Operand layout of that instruction, wave64, lane = 16 * g + c:
//   A[i][k] is taken from lane i + 16 k, B[k][j] from lane j + 16 k,
//   result register v of lane (g, c) holds D[g + 4 v][c].
// Both passes compute transposed tiles S^T[key][query] = K Q^T, so a lane always owns one
// query column (c) and four keys (g + 4 v); a head row of D values is split into four
// contiguous chunks of D / 4, chunk g supplying the k index of the instruction.
#include "lessdec_common.h"
#include "lessdec_internal.h"

namespace lessdec {

typedef double v4d __attribute__((ext_vector_type(4)));
typedef float v4f __attribute__((ext_vector_type(4)));
typedef _Float16 v4h __attribute__((ext_vector_type(4)));

template <typename T, int D>
struct Chunk {
  static constexpr int CH = D / 4;                       // values per lane group
  static constexpr int EPV = Store<T>::kPerVec;
  static constexpr int NV = CH / EPV;                    // 16-byte loads per lane
  typename Store<T>::Vec v[NV];
  __device__ inline void load(const T *row, int g)
  {
#pragma unroll
    for (int i = 0; i < NV; ++i) v[i] = load_vec<T>(row + g * CH + i * EPV);
  }
  __device__ inline double get(int s) const { return (double)Store<T>::get(v[s / EPV], s % EPV); }
};

// S^T tile: acc[v] = sum_d K[key g+4v][d] * Q[query c][d]; `a` holds the lane's key chunk,
// `b` the lane's query chunk (one of them already widened to fp64 by the caller).
template <typename T, int D>
__device__ inline v4d tile_kq(const Chunk<T, D> &kraw, const double (&qd)[D / 4])
{
  v4d acc = {0.0, 0.0, 0.0, 0.0};
#pragma unroll
  for (int s = 0; s < D / 4; ++s)
    acc = __builtin_amdgcn_mfma_f64_16x16x4f64(kraw.get(s), qd[s], acc, 0, 0, 0);
  return acc;
}
template <typename T, int D>
__device__ inline v4d tile_kq(const double (&kd)[D / 4], const Chunk<T, D> &qraw)
{
  v4d acc = {0.0, 0.0, 0.0, 0.0};
#pragma unroll
  for (int s = 0; s < D / 4; ++s)
    acc = __builtin_amdgcn_mfma_f64_16x16x4f64(kd[s], qraw.get(s), acc, 0, 0, 0);
  return acc;
}

constexpr int kPrefillWaves = 4;   // independent waves (16 queries or 16 keys each) per block
constexpr int kXcds = 8;           // workgroups go to the chip's 8 dies round-robin by index

// Workgroup -> (unit, group of kPrefillWaves tiles).  Causal sweeps have very different
// lengths, so every die gets the same sequence of groups: die x works through units x, x + 8,
// ..., each unit's groups in order.  The dies stay balanced and a unit's rows stay in one L2.
// grid = ceil(U / 8) * 8 * ngrp.
struct PrefillBlock { unsigned u; int grp; };
__device__ inline PrefillBlock prefill_block(unsigned b, int ngrp)
{
  const unsigned xcd = b % kXcds, r = b / kXcds;
  return PrefillBlock{(r / (unsigned)ngrp) * kXcds + xcd, (int)(r % (unsigned)ngrp)};
}

// p V^T for one tile of 16 keys, fp32 storage: v_mfma_f32_16x16x4_f32, one key group per
// instruction (result register w of lane (g, c) holds D[4 g + w][c]); O[b][w] is output
// element d = 16 b + 4 g + w of query c.
template <int D>
__device__ inline void tile_pv(const float *Vu, int P, int j0, int g, int c, const double (&e)[4],
                               v4f (&O)[D / 16])
{
#pragma unroll
  for (int v = 0; v < 4; ++v) {
    const int kj = j0 + g + 4 * v;
    const float *vrow = Vu + (size_t)(kj < P ? kj : P - 1) * D;
    const float pf = (float)e[v];
#pragma unroll
    for (int b = 0; b < D / 16; ++b)
      O[b] = __builtin_amdgcn_mfma_f32_16x16x4f32(vrow[b * 16 + c], pf, O[b], 0, 0, 0);
  }
}
template <int D>
__device__ inline void store_out(float *orow, int g, const v4f (&O)[D / 16], float inv)
{
#pragma unroll
  for (int b = 0; b < D / 16; ++b)
#pragma unroll
    for (int w = 0; w < 4; ++w) orow[b * 16 + 4 * g + w] = O[b][w] * inv;
}

// The same for fp16 storage on v_mfma_f32_16x16x16_f16: all 16 keys in one instruction.
// Lane (g, c) supplies k index 4 g + w, which stands for key g + 4 w (the keys whose
// probabilities the lane holds), and row i = c of the V^T operand stands for output element
// d = (D / 16) c + b in block b, so that a lane's operand values for all blocks are one
// contiguous run of each key row.  The probabilities go in as an fp16 pair hi + lo (22
// bits), accumulation is fp32.  O[b][w] is output element d = (D / 16)(4 g + w) + b.
template <int D>
struct VTile {
  static constexpr int NB = D / 16;                      // blocks = halves per lane per key row
  unsigned d[4][NB / 2];                                 // key row w: NB halves in NB / 2 dwords
  __device__ inline void load(const __half *Vu, int P, int j0, int g, int c)
  {
#pragma unroll
    for (int w = 0; w < 4; ++w) {
      const int kj = j0 + g + 4 * w;
      const __half *src = Vu + (size_t)(kj < P ? kj : P - 1) * D + NB * c;
      if constexpr (NB == 8) {
        const uint4 t = *reinterpret_cast<const uint4 *>(src);
        d[w][0] = t.x; d[w][1] = t.y; d[w][2] = t.z; d[w][3] = t.w;
      } else {
        const uint2 t = *reinterpret_cast<const uint2 *>(src);
        d[w][0] = t.x; d[w][1] = t.y;
      }
    }
  }
  // the operand of block b: element b of the four key rows, picked out of the dwords with byte
  // permutes (an array indexed per element would make a round trip through scratch memory)
  __device__ inline v4h operand(int b) const
  {
    typedef unsigned u2v __attribute__((ext_vector_type(2)));
    const unsigned sel = (b & 1) ? 0x07060302u : 0x05040100u;
    const u2v r = {__builtin_amdgcn_perm(d[1][b / 2], d[0][b / 2], sel),
                   __builtin_amdgcn_perm(d[3][b / 2], d[2][b / 2], sel)};
    return __builtin_bit_cast(v4h, r);
  }
};
template <int D>
__device__ inline void tile_pv(const VTile<D> &vt, const double (&e)[4], v4f (&O)[D / 16])
{
  v4h ph, pl;
#pragma unroll
  for (int v = 0; v < 4; ++v) {
    float ef = (float)e[v];
    // keep the fp32 value: folded into one fp64 -> fp16 conversion this becomes a long software
    // sequence (there is no such instruction)
    asm volatile("" : "+v"(ef));
    const _Float16 hi = (_Float16)ef;
    ph[v] = hi;
    pl[v] = (_Float16)(ef - (float)hi);
  }
#pragma unroll
  for (int b = 0; b < D / 16; ++b) {
    const v4h a = vt.operand(b);
    O[b] = __builtin_amdgcn_mfma_f32_16x16x16f16(a, ph, O[b], 0, 0, 0);
    O[b] = __builtin_amdgcn_mfma_f32_16x16x16f16(a, pl, O[b], 0, 0, 0);
  }
}
template <int D>
__device__ inline void store_out(__half *orow, int g, const v4f (&O)[D / 16], float inv)
{
  constexpr int NB = D / 16;
  // the lane owns elements NB (4 g + w) + b: one contiguous run of 4 NB halves
  __half run[4 * NB];
#pragma unroll
  for (int w = 0; w < 4; ++w)
#pragma unroll
    for (int b = 0; b < NB; ++b) run[NB * w + b] = __float2half_rn(O[b][w] * inv);
#pragma unroll
  for (int i = 0; i < 4 * NB / 8; ++i)
    *reinterpret_cast<uint4 *>(orow + 4 * NB * g + 8 * i) = *reinterpret_cast<const uint4 *>(run + 8 * i);
}

// -------------------------------------------------------------------------------------
// Row pass: one wave per block of 16 queries, kPrefillWaves consecutive query blocks per
// workgroup.  The workgroup sweeps the key tiles up to its last diagonal; every key tile is
// fetched and widened to fp64 once, by all 256 threads, into the LDS (two buffers, one
// barrier per tile) in the order the matrix instruction wants its operand, and each wave
// whose diagonal is not yet passed multiplies it with its own queries (kept in registers).
// A wave keeps the running row maximum m_i and sum L_i = sum_j e^{s_ij - m_i} (fp64) and, if
// an output is wanted, the flash-style running numerator in fp32, rescaled only in tiles
// where some row's maximum moved.  Leaves lse_i = m_i + ln L_i.
// LDS layout of a tile: lane (g, c) reads its operand values s = 2 i, 2 i + 1 (key row c,
// element g D/4 + s) as one 16-byte piece at index (4 i + g) 16 + c: conflict-free.
// -------------------------------------------------------------------------------------
template <typename T, int D>
__global__ __launch_bounds__(64 * kPrefillWaves) __attribute__((amdgpu_waves_per_eu(2, 2))) void prefill_rowpass_kernel(
    const T *__restrict__ Q, const T *__restrict__ K, const T *__restrict__ V, unsigned U, int G, int P,
    double *__restrict__ lse, T *__restrict__ out)
{
  // U counts query rows here: unit u's G query heads are rows u G .. u G + G - 1 of Q, out and
  // lse, and attend over unit u's keys and values
  constexpr int CH = D / 4, DB = D / 16;
  constexpr bool kHalf = sizeof(T) == 2;
  constexpr int EPT = 16 * D / (64 * kPrefillWaves);      // tile elements widened per thread
  static_assert(EPT % 2 == 0 && CH % EPT == 0, "a thread's elements stay within one lane group");
  __shared__ double2 s_k[2][16 * D / 2];
  const int nblk = (P + 15) / 16;
  const int ngrp = (nblk + kPrefillWaves - 1) / kPrefillWaves;
  const PrefillBlock pb = prefill_block(blockIdx.x, ngrp);
  if (pb.u >= U) return;                                  // uniform over the workgroup
  const int grp = ngrp - 1 - pb.grp;                      // long rows first
  const size_t u = pb.u;
  const int l = threadIdx.x % 64, g = l / 16, c = l % 16;
  const int it = grp * kPrefillWaves + (int)(threadIdx.x / 64);
  const bool active = it < nblk;                          // wave-uniform
  const int it_last = (grp + 1) * kPrefillWaves - 1 < nblk - 1 ? (grp + 1) * kPrefillWaves - 1 : nblk - 1;
  const int qi = it * 16 + c;
  const int qrow = qi < P ? qi : P - 1;
  const size_t ukv = u / (unsigned)G;
  const T *Qu = Q + u * (size_t)P * D, *Ku = K + ukv * (size_t)P * D, *Vu = V + ukv * (size_t)P * D;
  const double scale = 1.0 / sqrt((double)D);

  double qd[CH];
  {
    Chunk<T, D> qraw;
    qraw.load(Qu + (size_t)qrow * D, g);
#pragma unroll
    for (int s = 0; s < CH; ++s) qd[s] = qraw.get(s);
  }
  double m_run = -__builtin_inf(), L = 0.0;
  v4f O[DB];
#pragma unroll
  for (int b = 0; b < DB; ++b) O[b] = v4f{0.f, 0.f, 0.f, 0.f};

  // this thread's share of a key tile: EPT consecutive elements of row wc
  const int wc = threadIdx.x % 16, we = EPT * (int)(threadIdx.x / 16);
  const int wg = we / CH, wi = (we % CH) / 2;             // lane group and first piece of those elements
  T raw[EPT];
  auto fetch = [&](int jt) {
    const int kr = jt * 16 + wc;
    const T *src = Ku + (size_t)(kr < P ? kr : P - 1) * D + we;
    if constexpr (EPT * sizeof(T) == 32) {
      reinterpret_cast<uint4 *>(raw)[0] = reinterpret_cast<const uint4 *>(src)[0];
      reinterpret_cast<uint4 *>(raw)[1] = reinterpret_cast<const uint4 *>(src)[1];
    } else if constexpr (EPT * sizeof(T) == 16) {
      reinterpret_cast<uint4 *>(raw)[0] = reinterpret_cast<const uint4 *>(src)[0];
    } else {
      reinterpret_cast<uint2 *>(raw)[0] = reinterpret_cast<const uint2 *>(src)[0];
    }
  };
  fetch(0);
  for (int jt = 0; jt <= it_last; ++jt) {
    const int j0 = jt * 16;
    double2 *buf = s_k[jt & 1];
#pragma unroll
    for (int p = 0; p < EPT / 2; ++p)
      buf[((wi + p) * 4 + wg) * 16 + wc] =
          double2{(double)Store<T>::to_float(raw[2 * p]), (double)Store<T>::to_float(raw[2 * p + 1])};
    fetch(jt < it_last ? jt + 1 : jt);
    VTile<D> vt;
    if constexpr (kHalf) {
      if (out != nullptr) vt.load(reinterpret_cast<const __half *>(Vu), P, j0, g, c);
    }
    // tile jt is complete, and nobody still reads the buffer that tile jt + 1 will go into
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
    if (!active || jt > it) continue;                     // wave-uniform
    v4d acc = {0.0, 0.0, 0.0, 0.0};
#pragma unroll
    for (int i = 0; i < CH / 2; ++i) {
      const double2 kk = buf[(i * 4 + g) * 16 + c];
      acc = __builtin_amdgcn_mfma_f64_16x16x4f64(kk.x, qd[2 * i], acc, 0, 0, 0);
      acc = __builtin_amdgcn_mfma_f64_16x16x4f64(kk.y, qd[2 * i + 1], acc, 0, 0, 0);
    }
    double s[4], tmax = -__builtin_inf();
#pragma unroll
    for (int v = 0; v < 4; ++v) {
      const int kj = j0 + g + 4 * v;
      s[v] = (kj <= qi && kj < P) ? acc[v] * scale : -__builtin_inf();
      tmax = fmax(tmax, s[v]);
    }
    tmax = fmax(tmax, __shfl_xor(tmax, 16));
    tmax = fmax(tmax, __shfl_xor(tmax, 32));
    // key j0 <= qi always holds for jt <= it, so tmax is finite for every query with qi >= j0;
    // queries past the prompt end (qi >= P) still see key j0 < P.
    if (__any(tmax > m_run)) {
      const double m_new = fmax(m_run, tmax);
      const double alpha = exp(m_run - m_new);            // 1 where the maximum stayed
      L *= alpha;
      m_run = m_new;
      if (out != nullptr) {
        const float af = (float)alpha;
#pragma unroll
        for (int b = 0; b < DB; ++b) O[b] *= af;
      }
    }
    double e[4], esum = 0.0;
#pragma unroll
    for (int v = 0; v < 4; ++v) {
      e[v] = exp_softmax_f64(s[v] - m_run);
      esum += e[v];
    }
    L += esum;
    if (out != nullptr) {
      if constexpr (kHalf) tile_pv<D>(vt, e, O);
      else tile_pv<D>(reinterpret_cast<const float *>(Vu), P, j0, g, c, e, O);
    }
  }
  L += __shfl_xor(L, 16);
  L += __shfl_xor(L, 32);
  if (active && qi < P) {
    if (g == 0) lse[u * (size_t)P + qi] = m_run + log(L);
    if (out != nullptr) store_out<D>(out + (u * (size_t)P + qi) * D, g, O, (float)(1.0 / L));
  }
}

// -------------------------------------------------------------------------------------
// Feature-wise maximum of psi over a unit's prompt keys: psimax[u][r] = max_j psi_all[u][j][r].
// The values are >= 0 (Eq. 2 ends in an absolute value), so they order like their bit patterns
// and an integer LDS maximum does.   grid = U, block = 256.
// -------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void prefill_psimax_kernel(const float *__restrict__ psi_all, int P, int R,
                                                             float *__restrict__ psimax)
{
  __shared__ int s_max[LESSDEC_MAX_RANK];
  const size_t u = blockIdx.x;
  const int tid = threadIdx.x;
  if (tid < R) s_max[tid] = 0;
  __syncthreads();
  const float *pa = psi_all + u * (size_t)P * R;
  const int n = P * R;
  for (int i = tid; i < n; i += 256) atomicMax(&s_max[i % R], __float_as_int(pa[i]));
  __syncthreads();
  if (tid < R) psimax[u * R + tid] = __int_as_float(s_max[tid]);
}

// -------------------------------------------------------------------------------------
// Prefix states for the masked row pass: hpre[u][kb] = sum of psi(k_j)^T v_j and zpre[u][kb] =
// sum of psi(k_j) over the pairs Nh <= j < 64 kb (Eq. 6 restricted to a prefix), kb = 0 ..
// P / 64: what the low-rank part of Eq. 3 needs for a query whose discarded pairs reach at least
// to 64 kb.  fp32 sums (they only enter attention outputs and their normalisation, never a
// score; the state itself is built in fp64 by the finalize kernel).
// One workgroup per unit walks the keys in order, 64 at a time through the LDS; thread (d, rg)
// owns column d of rows rg, rg + 256 / D, ... of H, RC of them.   grid = U, block = 256.
// -------------------------------------------------------------------------------------
constexpr int kPrefixKeys = 64;
template <typename T, int D, int RC>
__global__ __launch_bounds__(256) void prefill_prefix_kernel(const T *__restrict__ V,
                                                             const float *__restrict__ psi_all, int P, int R,
                                                             int Nh, float *__restrict__ hpre,
                                                             float *__restrict__ zpre)
{
  constexpr int NG = 256 / D;                               // row groups
  __shared__ float s_psi[kPrefixKeys][LESSDEC_MAX_RANK + 1];
  const size_t u = blockIdx.x;
  const int tid = threadIdx.x, d = tid % D, rg = tid / D;
  const int nkb = P / kPrefixKeys + 1;
  const T *Vu = V + u * (size_t)P * D;
  const float *pa = psi_all + u * (size_t)P * R;
  float *hu = hpre + u * (size_t)nkb * R * D;
  float *zu = zpre + u * (size_t)nkb * R;
  float acc[RC];
#pragma unroll
  for (int i = 0; i < RC; ++i) acc[i] = 0.f;
  float zacc = 0.f;                                         // thread r < R: z's entry r
  for (int kb = 0; kb < nkb; ++kb) {
    // the state before this block of keys
#pragma unroll
    for (int i = 0; i < RC; ++i) {
      const int r = rg + NG * i;
      if (r < R) hu[((size_t)kb * R + r) * D + d] = acc[i];
    }
    if (tid < R) zu[(size_t)kb * R + tid] = zacc;
    const int j0 = kb * kPrefixKeys;
    if (j0 >= P) break;                                     // uniform
    const int nj = P - j0 < kPrefixKeys ? P - j0 : kPrefixKeys;
    __syncthreads();                                        // the previous block's readers are done
    for (int i = tid; i < nj * R; i += 256) {
      const int jj = i / R, r = i % R;
      s_psi[jj][r] = j0 + jj >= Nh ? pa[(size_t)j0 * R + i] : 0.f;   // the first Nh pairs are never discarded
    }
    __syncthreads();
#pragma unroll 8
    for (int jj = 0; jj < nj; ++jj) {
      const float v = Store<T>::to_float(Vu[(size_t)(j0 + jj) * D + d]);
#pragma unroll
      for (int i = 0; i < RC; ++i) acc[i] = fmaf(s_psi[jj][(rg + NG * i) % (LESSDEC_MAX_RANK + 1)], v, acc[i]);
    }
    if (tid < R)
      for (int jj = 0; jj < nj; ++jj) zacc += s_psi[jj][tid];
  }
}

// -------------------------------------------------------------------------------------
// Masked row pass: Lambda-masking taken through the prompt token by token (Sec. 4, "Setup";
// Sec. 3.2 builds the same matrix for training), all rows at once.  Under that policy the cache
// that token t meets is known beforehand: the first Nh tokens and the Nr tokens before it, the
// pairs discarded by then are Nh .. t - Nr - 1.  Row t of the attention matrix therefore has
// e^{q_t k_j / sqrt(D)} where pair j is cached (or is t itself) and phi(q_t) psi(k_j)^T where
// it was discarded, and out_t = (row t) V / (row t) 1 is Eq. 3 with H, z of Eq. 6.
// Same tiling as the row pass.  A workgroup first sweeps the key tiles that can hold cached
// pairs of any of its queries (the first ceil(Nh / 16) tiles and those from the window of its
// first query on), staged through the LDS as there, all other entries masked out.  Then every
// wave sweeps, on its own, the tiles that hold pairs discarded before its queries: the 16 x 16
// tile psi(K) phi(Q)^T is R / 4 matrix instructions instead of D / 4, nothing is staged.
// Online normalisation as in the row pass, the low-rank entries entering as w e^{-m}; before the
// second sweep m rises to ln of an upper bound of the query's weights (phi(q) . max_j psi(k_j),
// psimax [U, R] from prefill_psimax_kernel), so every weight handed to p V stays in [0, 1].
// Leaves lse_t = m_t + ln(sum of the entries that H2O's scores are normalised by): all of them,
// or with the sparse-denominator flag the exponentials only.
// -------------------------------------------------------------------------------------
template <typename T, int D>
__global__ __launch_bounds__(64 * kPrefillWaves) __attribute__((amdgpu_waves_per_eu(2, 2))) void prefill_maskedrows_kernel(
    const T *__restrict__ Q, const T *__restrict__ K, const T *__restrict__ V, unsigned U, int G, int P,
    const float *__restrict__ phi, const float *__restrict__ psi, const float *__restrict__ psimax,
    const float *__restrict__ hpre, const float *__restrict__ zpre, int R, int Nh, int Nr, int sparse_den,
    double *__restrict__ lse, T *__restrict__ out)
{
  constexpr int CH = D / 4, DB = D / 16;
  constexpr bool kHalf = sizeof(T) == 2;
  constexpr int EPT = 16 * D / (64 * kPrefillWaves);
  static_assert(EPT % 2 == 0 && CH % EPT == 0, "a thread's elements stay within one lane group");
  __shared__ double2 s_k[2][16 * D / 2];
  const int nblk = (P + 15) / 16;
  const int ngrp = (nblk + kPrefillWaves - 1) / kPrefillWaves;
  const PrefillBlock pb = prefill_block(blockIdx.x, ngrp);
  if (pb.u >= U) return;                                  // uniform over the workgroup
  const int grp = ngrp - 1 - pb.grp;                      // long rows first
  const size_t u = pb.u;
  const int l = threadIdx.x % 64, g = l / 16, c = l % 16;
  const int it = grp * kPrefillWaves + (int)(threadIdx.x / 64);
  const bool active = it < nblk;                          // wave-uniform
  const int it_last = (grp + 1) * kPrefillWaves - 1 < nblk - 1 ? (grp + 1) * kPrefillWaves - 1 : nblk - 1;
  const int qi = it * 16 + c;
  const int qrow = qi < P ? qi : P - 1;
  const size_t ukv = u / (unsigned)G;
  const T *Qu = Q + u * (size_t)P * D, *Ku = K + ukv * (size_t)P * D, *Vu = V + ukv * (size_t)P * D;
  const float *psi_u = psi + ukv * (size_t)P * R;
  const float *phi_q = phi + (u * (size_t)P + qrow) * R;
  const double scale = 1.0 / sqrt((double)D);

  // key tiles [0, nfirst) and [band0, it_last] can hold cached pairs of the workgroup's queries
  const int q0b = grp * kPrefillWaves * 16;
  int nfirst = (Nh + 15) / 16;
  if (nfirst > it_last + 1) nfirst = it_last + 1;
  int band0 = q0b - Nr >= 0 ? (q0b - Nr) / 16 : 0;
  if (band0 < nfirst) band0 = nfirst;
  if (band0 > it_last + 1) band0 = it_last + 1;
  const int ndense = nfirst + (it_last + 1 - band0);
  auto tile_of = [&](int idx) { return idx < nfirst ? idx : band0 + (idx - nfirst); };

  double qd[CH];
  {
    Chunk<T, D> qraw;
    qraw.load(Qu + (size_t)qrow * D, g);
#pragma unroll
    for (int s = 0; s < CH; ++s) qd[s] = qraw.get(s);
  }
  double m_run = -__builtin_inf(), L = 0.0;               // L: sum of the exponentials
  v4f O[DB];
#pragma unroll
  for (int b = 0; b < DB; ++b) O[b] = v4f{0.f, 0.f, 0.f, 0.f};

  // this thread's share of a key tile: EPT consecutive elements of row wc
  const int wc = threadIdx.x % 16, we = EPT * (int)(threadIdx.x / 16);
  const int wg = we / CH, wi = (we % CH) / 2;
  T raw[EPT];
  auto fetch = [&](int jt) {
    const int kr = jt * 16 + wc;
    const T *src = Ku + (size_t)(kr < P ? kr : P - 1) * D + we;
    if constexpr (EPT * sizeof(T) == 32) {
      reinterpret_cast<uint4 *>(raw)[0] = reinterpret_cast<const uint4 *>(src)[0];
      reinterpret_cast<uint4 *>(raw)[1] = reinterpret_cast<const uint4 *>(src)[1];
    } else if constexpr (EPT * sizeof(T) == 16) {
      reinterpret_cast<uint4 *>(raw)[0] = reinterpret_cast<const uint4 *>(src)[0];
    } else {
      reinterpret_cast<uint2 *>(raw)[0] = reinterpret_cast<const uint2 *>(src)[0];
    }
  };
  // 1) the cached pairs: the row pass over the tiles that can hold any, other entries masked out
  if (ndense > 0) fetch(tile_of(0));
  for (int idx = 0; idx < ndense; ++idx) {
    const int jt = tile_of(idx), j0 = jt * 16;
    double2 *buf = s_k[idx & 1];
#pragma unroll
    for (int p = 0; p < EPT / 2; ++p)
      buf[((wi + p) * 4 + wg) * 16 + wc] =
          double2{(double)Store<T>::to_float(raw[2 * p]), (double)Store<T>::to_float(raw[2 * p + 1])};
    fetch(tile_of(idx + 1 < ndense ? idx + 1 : idx));
    VTile<D> vt;
    if constexpr (kHalf) {
      if (out != nullptr) vt.load(reinterpret_cast<const __half *>(Vu), P, j0, g, c);
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
    // no cached pair of this wave's queries in the tile? (wave-uniform)
    if (!active || jt > it || (j0 >= Nh && j0 + 15 < it * 16 - Nr)) continue;
    v4d acc = {0.0, 0.0, 0.0, 0.0};
#pragma unroll
    for (int i = 0; i < CH / 2; ++i) {
      const double2 kk = buf[(i * 4 + g) * 16 + c];
      acc = __builtin_amdgcn_mfma_f64_16x16x4f64(kk.x, qd[2 * i], acc, 0, 0, 0);
      acc = __builtin_amdgcn_mfma_f64_16x16x4f64(kk.y, qd[2 * i + 1], acc, 0, 0, 0);
    }
    double sc[4], tmax = -__builtin_inf();
#pragma unroll
    for (int v = 0; v < 4; ++v) {
      const int kj = j0 + g + 4 * v;
      const bool cached = kj <= qi && kj < P && (kj < Nh || kj >= qi - Nr);
      sc[v] = cached ? acc[v] * scale : -__builtin_inf();
      tmax = fmax(tmax, sc[v]);
    }
    tmax = fmax(tmax, __shfl_xor(tmax, 16));
    tmax = fmax(tmax, __shfl_xor(tmax, 32));
    if (__any(tmax > m_run)) {
      const double m_new = fmax(m_run, tmax);
      const double alpha = m_new > m_run ? exp(m_run - m_new) : 1.0;   // 0 when nothing was summed before
      L *= alpha;
      m_run = m_new;
      if (out != nullptr) {
        const float af = (float)alpha;
#pragma unroll
        for (int b = 0; b < DB; ++b) O[b] *= af;
      }
    }
    double e[4], esum = 0.0;
#pragma unroll
    for (int v = 0; v < 4; ++v) {
      e[v] = sc[v] > -__builtin_inf() ? exp_softmax_f64(sc[v] - m_run) : 0.0;
      esum += e[v];
    }
    L += esum;
    if (out != nullptr) {
      if constexpr (kHalf) tile_pv<D>(vt, e, O);
      else tile_pv<D>(reinterpret_cast<const float *>(Vu), P, j0, g, c, e, O);
    }
  }

  // 2) the discarded pairs, every wave on its own: key tiles from Nh's tile to the last one that
  // holds a pair older than the window of the wave's last query.  The tile psi(K) phi(Q)^T is
  // R / 4 matrix instructions; entries of pairs that are cached for the lane's query are masked
  // out.  The next tile's value rows and psi operands are requested before this tile's arithmetic.
  double Lw = 0.0;                                         // sum of the low-rank entries, times e^{-m_run}
  int jt_lo = Nh / 16;
  const int jt_hi = (it * 16 + 14 - Nr) >= 0 ? (it * 16 + 14 - Nr) / 16 : -1;
  if (active && jt_lo <= jt_hi) {
    // m_run is finite for every query of the prompt: the diagonal tile held the query itself
    double em_run = m_run > -__builtin_inf() ? exp(-m_run) : 0.0;
    // phi of the lane's query: feature 4 s + g is this lane's operand of step s
    double fq[4];
#pragma unroll
    for (int s = 0; s < 4; ++s) {
      const int r = 4 * s + g;
      const float x = phi_q[r < R ? r : R - 1];
      fq[s] = r < R ? (double)x : 0.0;
    }
    // No weight of this query can exceed wb = phi(q) . max_j psi(k_j) (all features are >= 0), so
    // m rises to ln(wb) once, here, and every w e^{-m} handed to p V below stays in [0, 1]
    // without the sweep tracking a maximum.
    {
      const float *pm = psimax + ukv * (size_t)R;
      double wb = 0.0;
#pragma unroll
      for (int s = 0; s < 4; ++s) {
        const int r = 4 * s + g;
        wb = fma(fq[s], (double)pm[r < R ? r : R - 1], wb);  // fq is 0 past R
      }
      for (int r = 16 + g; r < R; r += 4) wb = fma((double)phi_q[r], (double)pm[r], wb);
      wb += __shfl_xor(wb, 16);
      wb += __shfl_xor(wb, 32);
      const double m_new = wb > 0.0 ? fmax(m_run, log(wb)) : m_run;
      if (m_new > m_run) {
        const double alpha = exp(m_run - m_new);
        L *= alpha;
        m_run = m_new;
        em_run = exp(-m_new);
        if (out != nullptr) {
          const float af = (float)alpha;
#pragma unroll
          for (int b = 0; b < DB; ++b) O[b] *= af;
        }
      }
    }
    // Pairs before 64 kbq were discarded before every query of this wave (and the first Nh are
    // left out of the prefix states): their share of Eq. 3 is phi(q) hpre[kbq] e^{-m} in the
    // numerator, on fp32 matrix tiles in the output layout of p V, and phi(q) zpre[kbq] e^{-m} in
    // the denominator.  Only the tiles from 64 kbq on are swept entry by entry.
    const int kbq = it * 16 - Nr > 0 ? (it * 16 - Nr) / kPrefixKeys : 0;
    if (kbq * kPrefixKeys > Nh) {
      const int nkb = P / kPrefixKeys + 1;
      const float *hk = hpre + (ukv * (size_t)nkb + kbq) * R * D;
      const float *zk = zpre + (ukv * (size_t)nkb + kbq) * R;
      double zsum = 0.0;
      // one step = features 4 s + g: f the lane's phi entry (0 past R), rc its clamped row
      auto prefix_step = [&](double f, int rc) {
        zsum = fma(f, (double)zk[rc], zsum);
        if (out != nullptr) {
          const float bf = (float)(f * em_run);
#pragma unroll
          for (int b = 0; b < DB; ++b) {
            const float a = hk[(size_t)rc * D + (kHalf ? DB * c + b : 16 * b + c)];
            O[b] = __builtin_amdgcn_mfma_f32_16x16x4f32(a, bf, O[b], 0, 0, 0);
          }
        }
      };
#pragma unroll
      for (int s = 0; s < 4; ++s)
        if (4 * s < R) prefix_step(fq[s], 4 * s + g < R ? 4 * s + g : R - 1);
      for (int s = 4; 4 * s < R; ++s) {
        const int r = 4 * s + g, rc = r < R ? r : R - 1;
        prefix_step(r < R ? (double)phi_q[rc] : 0.0, rc);
      }
      Lw += zsum * em_run;                                    // this lane group's features; the groups are added at the end
      if (jt_lo < kbq * (kPrefixKeys / 16)) jt_lo = kbq * (kPrefixKeys / 16);
    }
    auto psi_operands = [&](int j0, float (&a)[4]) {
      const int kr = j0 + c;                                  // a tile of the last, ragged query block can pass the prompt end
      const float *prow = psi_u + (size_t)(kr < P ? kr : P - 1) * R;
#pragma unroll
      for (int s = 0; s < 4; ++s) {                           // unconditional loads, features past R zeroed after
        const int r = 4 * s + g;
        const float x = prow[r < R ? r : R - 1];
        a[s] = r < R ? x : 0.f;
      }
    };
    VTile<D> vt_next;
    float pa_next[4];
    if constexpr (kHalf) vt_next.load(reinterpret_cast<const __half *>(Vu), P, jt_lo * 16, g, c);
    psi_operands(jt_lo * 16, pa_next);
    for (int jt = jt_lo; jt <= jt_hi; ++jt) {
      const int j0 = jt * 16;
      const VTile<D> vt = vt_next;
      float pa[4];
#pragma unroll
      for (int s = 0; s < 4; ++s) pa[s] = pa_next[s];
      const int jn = jt < jt_hi ? j0 + 16 : j0;
      if constexpr (kHalf) vt_next.load(reinterpret_cast<const __half *>(Vu), P, jn, g, c);
      psi_operands(jn, pa_next);
      v4d wt = {0.0, 0.0, 0.0, 0.0};
#pragma unroll
      for (int s = 0; s < 4; ++s)
        if (4 * s < R) wt = __builtin_amdgcn_mfma_f64_16x16x4f64((double)pa[s], fq[s], wt, 0, 0, 0);
      for (int s = 4; 4 * s < R; ++s) {
        const int r = 4 * s + g;
        const int kr = j0 + c < P ? j0 + c : P - 1;
        const double a = r < R ? (double)psi_u[(size_t)kr * R + r] : 0.0, b = r < R ? (double)phi_q[r] : 0.0;
        wt = __builtin_amdgcn_mfma_f64_16x16x4f64(a, b, wt, 0, 0, 0);
      }
      double e[4], wsum = 0.0;
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        const int kj = j0 + g + 4 * v;
        e[v] = (kj >= Nh && kj < qi - Nr) ? fmin(wt[v] * em_run, 1.0) : 0.0;
        wsum += e[v];
      }
      Lw += wsum;
      if (out != nullptr) {
        if constexpr (kHalf) tile_pv<D>(vt, e, O);
        else tile_pv<D>(reinterpret_cast<const float *>(Vu), P, j0, g, c, e, O);
      }
    }
  }
  double Ls = L;                                           // exponentials only
  L += Lw;
  L += __shfl_xor(L, 16);
  L += __shfl_xor(L, 32);
  Ls += __shfl_xor(Ls, 16);
  Ls += __shfl_xor(Ls, 32);
  if (active && qi < P) {
    if (g == 0) lse[u * (size_t)P + qi] = m_run + log(sparse_den ? Ls : L);
    if (out != nullptr) store_out<D>(out + (u * (size_t)P + qi) * D, g, O, (float)(1.0 / L));
  }
}

// -------------------------------------------------------------------------------------
// Column pass: one wave per block of 16 keys.  Sweeps the query tiles from the diagonal
// down and sums a_ij = e^{s_ij - lse_i} over the queries: the accumulated attention
// probability of each prompt token (H2O's score, Sec. 2.1).  No atomics: every column is
// owned by one wave and reduced in a fixed order.
// -------------------------------------------------------------------------------------
template <typename T, int D>
__global__ __launch_bounds__(64 * kPrefillWaves) void prefill_colpass_kernel(
    const T *__restrict__ Q, const T *__restrict__ K, unsigned U, int P,
    const double *__restrict__ lse, int G, double *__restrict__ colsum)
{
  constexpr int CH = D / 4;
  const int nblk = (P + 15) / 16;
  const int ngrp = (nblk + kPrefillWaves - 1) / kPrefillWaves;
  const PrefillBlock pb = prefill_block(blockIdx.x, ngrp);
  const int grp = pb.grp;                                 // early columns have the longest sweeps
  const size_t u = pb.u;
  const int l = threadIdx.x % 64, g = l / 16, c = l % 16;
  const int jt = grp * kPrefillWaves + (int)(threadIdx.x / 64);
  if (jt >= nblk || pb.u >= U) return;                    // wave-uniform; the waves share nothing
  const int j0 = jt * 16;
  const T *Ku = K + u * (size_t)P * D;
  const double scale = 1.0 / sqrt((double)D);

  double kd[CH];
  {
    Chunk<T, D> kraw;
    const int kr = j0 + c;
    kraw.load(Ku + (size_t)(kr < P ? kr : P - 1) * D, g);
#pragma unroll
    for (int s = 0; s < CH; ++s) kd[s] = kraw.get(s);
  }
  double cs[4] = {0.0, 0.0, 0.0, 0.0};
  for (int h = 0; h < G; ++h) {                           // the unit's query heads, one sweep each
  const T *Qu = Q + (u * G + h) * (size_t)P * D;
  const double *lse_u = lse + (u * G + h) * (size_t)P;
  Chunk<T, D> qraw;
  double lq;
  {
    const int qr = j0 + c < P ? j0 + c : P - 1;
    qraw.load(Qu + (size_t)qr * D, g);
    lq = lse_u[qr];
  }
  auto tile = [&](int it, const Chunk<T, D> &cur, double lcur, Chunk<T, D> &nxt, double &lnxt) {
    const int qi = it * 16 + c;
    {
      const int qn = (it + 1 < nblk ? qi + 16 : qi);
      const int qr = qn < P ? qn : P - 1;
      nxt.load(Qu + (size_t)qr * D, g);
      lnxt = lse_u[qr];
    }
    const v4d acc = tile_kq<T, D>(kd, cur);
#pragma unroll
    for (int v = 0; v < 4; ++v) {
      const double a = exp_softmax_f64(fma(acc[v], scale, -lcur));
      cs[v] += (qi < P && (j0 + g + 4 * v) <= qi) ? a : 0.0;
    }
  };
  Chunk<T, D> qother;
  double lother;
  for (int it = jt; it < nblk; it += 2) {
    tile(it, qraw, lq, qother, lother);
    if (it + 1 < nblk) tile(it + 1, qother, lother, qraw, lq);
  }
  }
#pragma unroll
  for (int v = 0; v < 4; ++v) {
#pragma unroll
    for (int o = 8; o > 0; o >>= 1) cs[v] += __shfl_xor(cs[v], o);
    const int kj = j0 + g + 4 * v;
    if (c == 0 && kj < P) colsum[u * (size_t)P + kj] = cs[v];
  }
}

// -------------------------------------------------------------------------------------
// Cheap column sums, fp16 storage only: the same sweep as the column pass on
// v_mfma_f32_16x16x32_f16 with fp32 accumulation and the fast fp32 exponential.  Their only
// use is to tell which tokens can possibly matter for the selection (prefill_band_kernel);
// every value that decides or is stored comes from the exact pass over those tokens.
// Lane (g, c) supplies elements 32 ks + 8 g .. + 7 of key row c (A) and of query row c (B);
// result register w holds S^T[key 4 g + w][query c].
// -------------------------------------------------------------------------------------
typedef _Float16 v8h __attribute__((ext_vector_type(8)));
constexpr int kApproxTiles = 4;    // key tiles (of 16) per wave: a query tile is loaded once for all of them
template <int D>
__global__ __launch_bounds__(64 * kPrefillWaves) void prefill_colapprox_kernel(
    const __half *__restrict__ Q, const __half *__restrict__ K, unsigned U, int P,
    const double *__restrict__ lse, int G, float *__restrict__ approx)
{
  constexpr int KS = D / 32, KT = kApproxTiles;
  const int nblk = (P + 15) / 16;
  const int nkb = (nblk + KT - 1) / KT;                   // groups of KT key tiles
  const int ngrp = (nkb + kPrefillWaves - 1) / kPrefillWaves;
  const PrefillBlock pb = prefill_block(blockIdx.x, ngrp);
  const size_t u = pb.u;
  const int l = threadIdx.x % 64, g = l / 16, c = l % 16;
  const int kb = pb.grp * kPrefillWaves + (int)(threadIdx.x / 64);
  if (kb >= nkb || pb.u >= U) return;                     // wave-uniform; the waves share nothing
  const int jt0 = kb * KT, j0 = jt0 * 16;
  const __half *Ku = K + u * (size_t)P * D;
  const float scale = (float)(1.0 / sqrt((double)D));
  auto load_row = [&](const __half *row, v8h (&dst)[KS]) {
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) dst[ks] = *reinterpret_cast<const v8h *>(row + 32 * ks + 8 * g);
  };
  v8h ka[KT][KS], qa[KS];
#pragma unroll
  for (int t = 0; t < KT; ++t) {
    const int kr = j0 + 16 * t + c;
    load_row(Ku + (size_t)(kr < P ? kr : P - 1) * D, ka[t]);
  }
  float cs[KT][4];
#pragma unroll
  for (int t = 0; t < KT; ++t)
#pragma unroll
    for (int w = 0; w < 4; ++w) cs[t][w] = 0.f;
  for (int h = 0; h < G; ++h) {                           // the unit's query heads, one sweep each
  const __half *Qu = Q + (u * G + h) * (size_t)P * D;
  const double *lse_u = lse + (u * G + h) * (size_t)P;
  float lq;
  {
    const int qr = j0 + c < P ? j0 + c : P - 1;
    load_row(Qu + (size_t)qr * D, qa);
    lq = (float)lse_u[qr];
  }
  // one query tile: request the tile after it into `nxt`, then multiply `cur` (two buffers
  // that swap roles, so that no register copy has to wait for the request just made)
  auto tile = [&](int it, const v8h (&cur)[KS], float lcur, v8h (&nxt)[KS], float &lnxt) {
    const int qi = it * 16 + c;
    {
      const int qx = (it + 1 < nblk ? qi + 16 : qi);
      const int qr = qx < P ? qx : P - 1;
      load_row(Qu + (size_t)qr * D, nxt);
      lnxt = (float)lse_u[qr];
    }
#pragma unroll
    for (int t = 0; t < KT; ++t) {
      if (jt0 + t > it) continue;                         // key tile wholly after these queries (uniform)
      v4f acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(ka[t][ks], cur[ks], acc, 0, 0, 0);
#pragma unroll
      for (int w = 0; w < 4; ++w) {
        const int kj = j0 + 16 * t + 4 * g + w;
        const float a = __expf(fmaf(acc[w], scale, -lcur));
        cs[t][w] += (qi < P && kj <= qi) ? a : 0.f;
      }
    }
  };
  v8h qb[KS];
  float lb;
  for (int it = jt0; it < nblk; it += 2) {
    tile(it, qa, lq, qb, lb);
    if (it + 1 < nblk) tile(it + 1, qb, lb, qa, lq);
  }
  }
#pragma unroll
  for (int t = 0; t < KT; ++t)
#pragma unroll
    for (int w = 0; w < 4; ++w) {
#pragma unroll
      for (int o = 8; o > 0; o >>= 1) cs[t][w] += __shfl_xor(cs[t][w], o);
      const int kj = j0 + 16 * t + 4 * g + w;
      if (c == 0 && kj < P) approx[u * (size_t)P + kj] = cs[t][w];
    }
}

// -------------------------------------------------------------------------------------
// The largest score magnitude a unit's prompt can produce: max_i |q_i| max_j |k_j| / sqrt(D)
// over its tokens and query heads (>= |q_i . k_j| / sqrt(D) for every pair).  It bounds the rounding
// error of the cheap column sums (below).  One block per unit, a row per D / 8 lanes.
// -------------------------------------------------------------------------------------
template <int D>
__global__ __launch_bounds__(256) void prefill_scorebound_kernel(const __half *__restrict__ Q,
                                                                 const __half *__restrict__ K, int P, int G,
                                                                 float *__restrict__ bound)
{
  constexpr int LPR = D / 8, RPB = 256 / LPR;
  __shared__ float s_max[2][256 / kWave];
  const size_t u = blockIdx.x;
  const int tid = threadIdx.x, lr = tid % LPR, rb = tid / LPR;
  float mx[2] = {0.f, 0.f};                               // largest squared norm: queries, keys
  for (int which = 0; which < 2; ++which) {
    const __half *base = which ? K + u * (size_t)P * D : Q + u * (size_t)G * P * D;
    const long rows = which ? P : (long)G * P;
    for (long r = rb; r < rows; r += RPB) {
      const uint4 raw = *reinterpret_cast<const uint4 *>(base + r * D + lr * 8);
      const __half2 *h2 = reinterpret_cast<const __half2 *>(&raw);
      float ss = 0.f;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const float2 f = __half22float2(h2[i]);
        ss = fmaf(f.x, f.x, fmaf(f.y, f.y, ss));
      }
#pragma unroll
      for (int o = LPR / 2; o > 0; o >>= 1) ss += __shfl_xor(ss, o);
      mx[which] = fmaxf(mx[which], ss);
    }
  }
#pragma unroll
  for (int which = 0; which < 2; ++which) {
#pragma unroll
    for (int o = kWave / 2; o > 0; o >>= 1) mx[which] = fmaxf(mx[which], __shfl_xor(mx[which], o));
    if (tid % kWave == 0) s_max[which][tid / kWave] = mx[which];
  }
  __syncthreads();
  if (tid == 0) {
    float mq = 0.f, mk = 0.f;
    for (int w = 0; w < 256 / kWave; ++w) {
      mq = fmaxf(mq, s_max[0][w]);
      mk = fmaxf(mk, s_max[1][w]);
    }
    // rounded up a little: the squared norms above carry fp32 rounding themselves
    bound[u] = sqrtf(mq) * sqrtf(mk) * (float)(1.0 / sqrt((double)D)) * 1.001f;
  }
}

// -------------------------------------------------------------------------------------
// Which tokens can matter, from the cheap column sums.  A cheap sum a~ and the exact one a
// satisfy |a~ - a| <= eps a + tau with
//   eps = 2^-24 ((D + 6) M + 3 ln P + G P / 16 + 6),   M = the unit's score bound (above):
// D M for the fp32 accumulation of the D exact fp16 products of a score, 5 M + 3 ln P for the
// rounded 1 / sqrt(D), the row's log-sum rounded to fp32 (|lse| <= M + ln P), the fused
// multiply-add and the scaling inside the fast exponential (|s - lse| <= 2 M + ln P each), 2
// for the exponential itself, G P / 16 + 4 for a lane's running sum and the four lane exchanges;
// tau = 2^-100 covers terms flushed to zero.  The band used is twice that, and at least kBand
// (at the benchmark shapes eps is a tenth of kBand; the band only grows for prompts with far
// larger queries and keys).  With every cheap value within the band of the exact one, a token
// is surely a heavy hitter if fewer than Nh others could possibly be larger, surely discarded
// if at least Nh others are surely larger, and in doubt otherwise.
// flag[j] = 1 kept for sure (heavy or recent), 0 discarded for sure, 2 in doubt.
// One thread per token.   grid = U * ceil(P / 256), block = 256.
// -------------------------------------------------------------------------------------
constexpr float kBand = 1.0f / 256.0f;
__host__ __device__ inline float colapprox_error_bound(float M, int D, int P, int G)
{
  return 5.9604645e-08f * ((float)(D + 6) * M + 3.f * logf((float)P) + (float)G * (float)P / 16.f + 6.f);
}
__global__ __launch_bounds__(256) void prefill_band_kernel(const float *__restrict__ approx,
                                                           const float *__restrict__ bound, int D, int G, int P,
                                                           int Nh, int Nr, int32_t *__restrict__ flag)
{
  const int nb = (P + 255) / 256;
  const size_t u = blockIdx.x / nb;
  const int j = (int)(blockIdx.x % nb) * 256 + (int)threadIdx.x;
  if (j >= P) return;
  const float *a = approx + u * (size_t)P;
  const float band = fmaxf(kBand, 2.f * colapprox_error_bound(bound[u], D, P, G));
  const float tau = 7.8886091e-31f;                      // 2^-100
  const int ncand = P - Nr;
  int f = 1;                                    // recent
  if (j < ncand) {
    const float lo = a[j] * (1.f - band) - tau, hi = a[j] * (1.f + band) + tau;
    int maybe_larger = 0, surely_larger = 0;
    for (int i = 0; i < ncand; ++i) {
      const float b = a[i];
      maybe_larger += (b * (1.f + band) + tau >= lo) ? 1 : 0;   // counts j itself
      surely_larger += (b * (1.f - band) - tau > hi) ? 1 : 0;
    }
    f = (maybe_larger - 1 < Nh) ? 1 : (surely_larger >= Nh ? 0 : 2);
  }
  flag[u * (size_t)P + j] = f;
}

// -------------------------------------------------------------------------------------
// List of the tokens whose exact column sum is wanted (flag != 0), ascending, per unit.
// grid = U, block = 256.
// -------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void prefill_compact_kernel(const int32_t *__restrict__ flag, int P,
                                                              int32_t *__restrict__ list,
                                                              int32_t *__restrict__ count)
{
  __shared__ int s_cnt[256];
  const size_t u = blockIdx.x;
  const int tid = threadIdx.x;
  const int32_t *f = flag + u * (size_t)P;
  int32_t *out = list + u * (size_t)P;
  const int chunk = (P + 255) / 256;
  const int lo = tid * chunk < P ? tid * chunk : P, hi = (lo + chunk < P) ? lo + chunk : P;
  int cnt = 0;
  for (int j = lo; j < hi; ++j) cnt += f[j] != 0 ? 1 : 0;
  s_cnt[tid] = cnt;
  __syncthreads();
  int base = 0;
  for (int t = 0; t < tid; ++t) base += s_cnt[t];
  for (int j = lo; j < hi; ++j)
    if (f[j] != 0) out[base++] = j;
  if (tid == 255) count[u] = base;
}

// -------------------------------------------------------------------------------------
// Exact column sums of listed tokens only: the column pass with 16 listed keys per wave in
// place of 16 consecutive ones.  The sweep starts at the query tile of the wave's earliest
// key; a key takes part from its own position on.  The length of the list is only known on
// the device: a unit gets enough blocks for a list a little longer than the budget, and its
// waves loop should the list be longer.   grid = ceil(U / 8) * 8 * blocks_per_unit.
// -------------------------------------------------------------------------------------
template <typename T, int D>
__global__ __launch_bounds__(64 * kPrefillWaves) void prefill_colexact_kernel(
    const T *__restrict__ Q, const T *__restrict__ K, unsigned U, int P, const double *__restrict__ lse,
    const int32_t *__restrict__ list, const int32_t *__restrict__ count, int blocks_per_unit, int G,
    double *__restrict__ colsum)
{
  constexpr int CH = D / 4;
  const int nblk = (P + 15) / 16;
  const PrefillBlock pb = prefill_block(blockIdx.x, blocks_per_unit);
  const size_t u = pb.u;
  const int l = threadIdx.x % 64, g = l / 16, c = l % 16;
  if (pb.u >= U) return;
  const int n = count[u];
  const T *Ku = K + u * (size_t)P * D;
  const double scale = 1.0 / sqrt((double)D);
  // tiles of 16 listed keys, dealt to the unit's waves in turn (the list is ascending, so
  // the long sweeps come first); wave-uniform, the waves share nothing
  for (int lt = pb.grp * kPrefillWaves + (int)(threadIdx.x / 64); lt * 16 < n;
       lt += blocks_per_unit * kPrefillWaves) {
    const int32_t *li = list + u * (size_t)P + lt * 16;
    const int nk = n - lt * 16 < 16 ? n - lt * 16 : 16;   // listed keys of this tile
    double kd[CH];
    {
      Chunk<T, D> kraw;
      kraw.load(Ku + (size_t)li[c < nk ? c : 0] * D, g);
#pragma unroll
      for (int s = 0; s < CH; ++s) kd[s] = kraw.get(s);
    }
    int kjv[4];                                           // positions of the lane's four keys
#pragma unroll
    for (int v = 0; v < 4; ++v) kjv[v] = g + 4 * v < nk ? li[g + 4 * v] : INT_MAX;
    const int it0 = li[0] / 16;
    double cs[4] = {0.0, 0.0, 0.0, 0.0};
    for (int h = 0; h < G; ++h) {                         // the unit's query heads, one sweep each
    const T *Qu = Q + (u * G + h) * (size_t)P * D;
    const double *lse_u = lse + (u * G + h) * (size_t)P;
    Chunk<T, D> qraw;
    double lq;
    {
      const int qr = it0 * 16 + c < P ? it0 * 16 + c : P - 1;
      qraw.load(Qu + (size_t)qr * D, g);
      lq = lse_u[qr];
    }
    auto tile = [&](int it, const Chunk<T, D> &cur, double lcur, Chunk<T, D> &nxt, double &lnxt) {
      const int qi = it * 16 + c;
      {
        const int qn = (it + 1 < nblk ? qi + 16 : qi);
        const int qr = qn < P ? qn : P - 1;
        nxt.load(Qu + (size_t)qr * D, g);
        lnxt = lse_u[qr];
      }
      const v4d acc = tile_kq<T, D>(kd, cur);
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        const double a = exp_softmax_f64(fma(acc[v], scale, -lcur));
        cs[v] += (qi < P && kjv[v] <= qi) ? a : 0.0;
      }
    };
    Chunk<T, D> qother;
    double lother;
    for (int it = it0; it < nblk; it += 2) {
      tile(it, qraw, lq, qother, lother);
      if (it + 1 < nblk) tile(it + 1, qother, lother, qraw, lq);
    }
    }
#pragma unroll
    for (int v = 0; v < 4; ++v) {
#pragma unroll
      for (int o = 8; o > 0; o >>= 1) cs[v] += __shfl_xor(cs[v], o);
      if (c == 0 && kjv[v] != INT_MAX) colsum[u * (size_t)P + kjv[v]] = cs[v];
    }
  }
}

// -------------------------------------------------------------------------------------
// Settles the tokens in doubt with their exact column sums: the heavy set is the tokens kept
// for sure plus the best of those in doubt, by (column sum, position) as in the rank kernel.
// keep[j] = 1 / 0.   grid = U, block = 256.
// -------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void prefill_refine_kernel(const double *__restrict__ colsum,
                                                             const int32_t *__restrict__ flag, int P, int Nh,
                                                             int Nr, int32_t *__restrict__ keep)
{
  constexpr int kCap = 1024;                    // tokens in doubt held in the LDS (a handful in practice)
  __shared__ int s_sure, s_nd;
  __shared__ int s_idx[kCap];
  __shared__ double s_val[kCap];
  const size_t u = blockIdx.x;
  const int tid = threadIdx.x;
  const double *cs = colsum + u * (size_t)P;
  const int32_t *f = flag + u * (size_t)P;
  int32_t *out = keep + u * (size_t)P;
  const int ncand = P - Nr;
  if (tid == 0) s_sure = s_nd = 0;
  __syncthreads();
  int mine = 0;
  for (int j = tid; j < P; j += 256) {
    const int fj = f[j];
    mine += (fj == 1 && j < ncand) ? 1 : 0;
    if (fj == 2) {
      const int k = atomicAdd(&s_nd, 1);
      if (k < kCap) {
        s_idx[k] = j;
        s_val[k] = cs[j];
      }
    }
    out[j] = fj == 1 ? 1 : 0;
  }
  if (mine) atomicAdd(&s_sure, mine);
  __syncthreads();
  const int need = Nh - s_sure;                 // heavy slots left for the tokens in doubt
  const int nd = s_nd;
  if (nd <= kCap) {
    for (int k = tid; k < nd; k += 256) {
      const double a = s_val[k];
      const int j = s_idx[k];
      int larger = 0;
      for (int i = 0; i < nd; ++i) larger += (s_val[i] > a || (s_val[i] == a && s_idx[i] > j)) ? 1 : 0;
      out[j] = larger < need ? 1 : 0;
    }
  } else {
    for (int j = tid; j < ncand; j += 256) {
      if (f[j] != 2) continue;
      const double a = cs[j];
      int larger = 0;
      for (int i = 0; i < ncand; ++i) {
        if (f[i] != 2) continue;
        const double b = cs[i];
        larger += (b > a || (b == a && i > j)) ? 1 : 0;
      }
      out[j] = larger < need ? 1 : 0;
    }
  }
}

// -------------------------------------------------------------------------------------
// Selection: the last Nr tokens are recent; among the others the Nh largest (column sum,
// position) pairs are heavy hitters; everything else is discarded.  Exact rank counting,
// no sort: token j is heavy iff fewer than Nh candidates are larger.  Under Lambda-masking
// (Sec. 4, "Setup") the first Nh tokens take the place of the heavy hitters.
// One thread per token: keep[j] = 1 / 0.   grid = U * ceil(P / 256), block = 256.
// -------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void prefill_rank_kernel(const double *__restrict__ colsum, int P,
                                                           int Nh, int Nr, int lambda,
                                                           int32_t *__restrict__ keep_of)
{
  const int nb = (P + 255) / 256;
  const size_t u = blockIdx.x / nb;
  const int j = (int)(blockIdx.x % nb) * 256 + (int)threadIdx.x;
  if (j >= P) return;
  const double *cs = colsum + u * (size_t)P;
  const int C = Nh + Nr;
  const int ncand = P - Nr;                     // positions < P - Nr compete for the heavy slots
  int keep = 1;
  if (P > C && lambda) {
    keep = (j < Nh || j >= ncand) ? 1 : 0;
  } else if (P > C && j < ncand) {
    const double a = cs[j];
    int larger = 0;
    for (int i = 0; i < ncand; ++i) {
      const double b = cs[i];
      larger += (b > a || (b == a && i > j)) ? 1 : 0;
    }
    keep = larger < Nh ? 1 : 0;
  }
  keep_of[u * (size_t)P + j] = keep;
}

// -------------------------------------------------------------------------------------
// Finalize, one workgroup per unit: kept tokens get slots in ascending position (or, for the
// prompt taken token by token under Lambda-masking, the slots that in-place replacement would
// have left them in); their
// rows are gathered into the cache (acc = column sum, pos, psi), unused slots cleared; the
// discarded pairs build H = sum psi(k)^T v, z = sum psi(k) (Eq. 6) in fp64.
// For the state, wave w owns D / 4 columns of H, two per lane, and its lanes split the
// tokens between them (interleaved parts, combined by lane exchange at the end), R in
// chunks of RC rows.  slot_of: in 1 / 0 (kept / discarded), out slot index / -1.
// grid = U, block = 256, dynamic LDS = C ints.
// -------------------------------------------------------------------------------------
__device__ inline void load_pair(const __half *p, float &a, float &b)
{
  const __half2 h = *reinterpret_cast<const __half2 *>(p);
  a = __low2float(h);
  b = __high2float(h);
}
__device__ inline void load_pair(const float *p, float &a, float &b)
{
  const float2 f = *reinterpret_cast<const float2 *>(p);
  a = f.x;
  b = f.y;
}

template <typename T, int D, int RC>
__global__ __launch_bounds__(256) void prefill_finalize_kernel(
    const T *__restrict__ K, const T *__restrict__ V, int P, const double *__restrict__ colsum,
    int32_t *__restrict__ slot_of, const float *__restrict__ psi_all, int C, int R,
    T *__restrict__ k_cache, T *__restrict__ v_cache, double *__restrict__ acc,
    int32_t *__restrict__ pos, float *__restrict__ psi, float *__restrict__ H,
    double *__restrict__ z, int32_t *__restrict__ n_seen, int32_t *__restrict__ pend_slot, int ring_nh)
{
  extern __shared__ int s_tok[];                           // [C] token held by each slot
  __shared__ int s_cnt[256];
  const size_t u = blockIdx.x;
  const int tid = threadIdx.x, wave = tid / 64, lane = tid % 64;
  const T *Ku = K + u * (size_t)P * D, *Vu = V + u * (size_t)P * D;
  int32_t *so = slot_of + u * (size_t)P;
  const float *pa = psi_all + u * (size_t)P * R;
  const int kept = P < C ? P : C;

  // 1) slot = number of kept tokens before j: per-thread contiguous chunk + the 256 counts
  {
    const int chunk = (P + 255) / 256;
    const int lo = tid * chunk < P ? tid * chunk : P, hi = (lo + chunk < P) ? lo + chunk : P;
    int cnt = 0;
    for (int j = lo; j < hi; ++j) cnt += so[j];
    s_cnt[tid] = cnt;
    __syncthreads();
    int base = 0;
    for (int t = 0; t < tid; ++t) base += s_cnt[t];
    for (int j = lo; j < hi; ++j) {
      const int keep = so[j];
      // ring_nh >= 0: the slots as in-place replacement leaves them when the first ring_nh tokens
      // stay and the others pass through the remaining slots in turn (Sec. 3.2)
      const int slot = (ring_nh < 0 || j < ring_nh || P <= C || C <= ring_nh) ? base : ring_nh + (j - ring_nh) % (C - ring_nh);
      so[j] = keep ? slot : -1;
      if (keep && slot < C) s_tok[slot] = j;
      base += keep;
    }
  }
  __syncthreads();

  // 2) gather: rows moved as 16-byte vectors, 64 / kVecs slots per wave at a time
  constexpr int kVecs = D * (int)sizeof(T) / 16;           // per row: 8, 16 or 32
  constexpr int kSlotsPerWave = 64 / kVecs;
  for (int s = wave * kSlotsPerWave + lane / kVecs; s < C; s += 4 * kSlotsPerWave) {
    const size_t slot = u * C + s;
    const int i = lane % kVecs;
    if (s < kept) {
      const int j = s_tok[s];
      reinterpret_cast<uint4 *>(k_cache + slot * D)[i] = reinterpret_cast<const uint4 *>(Ku + (size_t)j * D)[i];
      reinterpret_cast<uint4 *>(v_cache + slot * D)[i] = reinterpret_cast<const uint4 *>(Vu + (size_t)j * D)[i];
      if (i == 0) {
        acc[slot] = colsum[u * (size_t)P + j];
        pos[slot] = j;
      }
      for (int r = i; r < R; r += kVecs) psi[slot * R + r] = pa[(size_t)j * R + r];
    } else {
      if (i == 0) {
        acc[slot] = 0.0;
        pos[slot] = -1;
      }
      for (int r = i; r < R; r += kVecs) psi[slot * R + r] = 0.f;
    }
  }

  // 3) state of the discarded pairs.  Kept tokens go through the same arithmetic with a zero
  // weight, so that nothing in the loop depends on a load and iterations overlap.
  constexpr int LW = D / 8, PARTS = 64 / LW;               // lanes per token (2 columns each), parts
  const int col = wave * (D / 4) + 2 * (lane % LW), part = lane / LW;
  const bool vec4 = R % 4 == 0;                            // psi rows readable as 16-byte vectors
  constexpr int kUnroll = RC >= 16 ? 2 : 4;                // tokens in flight per lane (register budget)
  for (int r0 = 0; r0 < R; r0 += RC) {
    const int rn = R - r0 < RC ? R - r0 : RC;
    double h0[RC], h1[RC], zs[RC];
#pragma unroll
    for (int r = 0; r < RC; ++r) h0[r] = h1[r] = zs[r] = 0.0;
    auto token = [&](int j, const float (&gj)[RC]) {
      const double w = so[j] < 0 ? 1.0 : 0.0;
      float vf0, vf1;
      load_pair(Vu + (size_t)j * D + col, vf0, vf1);
      const double v0 = w * (double)vf0, v1 = w * (double)vf1;
#pragma unroll
      for (int r = 0; r < RC; ++r) {
        const double g = (double)gj[r];
        h0[r] = fma(g, v0, h0[r]);
        h1[r] = fma(g, v1, h1[r]);
        zs[r] = fma(g, w, zs[r]);
      }
    };
    // rows past R repeat row 0 (unconditional loads); their sums are never stored
    if (vec4) {
#pragma unroll kUnroll
      for (int j = part; j < P; j += PARTS) {
        const float *pj = pa + (size_t)j * R + r0;
        float gj[RC];
#pragma unroll
        for (int r4 = 0; r4 < RC / 4; ++r4)
          *reinterpret_cast<float4 *>(gj + 4 * r4) = *reinterpret_cast<const float4 *>(pj + (4 * r4 < rn ? 4 * r4 : 0));
        token(j, gj);
      }
    } else {
#pragma unroll kUnroll
      for (int j = part; j < P; j += PARTS) {
        const float *pj = pa + (size_t)j * R + r0;
        float gj[RC];
#pragma unroll
        for (int r = 0; r < RC; ++r) gj[r] = pj[r < rn ? r : 0];
        token(j, gj);
      }
    }
#pragma unroll
    for (int r = 0; r < RC; ++r) {
#pragma unroll
      for (int o = LW; o < 64; o <<= 1) {
        h0[r] += __shfl_xor(h0[r], o);
        h1[r] += __shfl_xor(h1[r], o);
        zs[r] += __shfl_xor(zs[r], o);
      }
      if (r < rn && part == 0) {
        H[(u * R + r0 + r) * D + col] = (float)h0[r];
        H[(u * R + r0 + r) * D + col + 1] = (float)h1[r];
      }
      if (r < rn && tid == 0) z[u * R + r0 + r] = zs[r];
    }
  }
  if (tid == 0) {
    n_seen[u] = P;
    pend_slot[u] = -1;
  }
}

template <typename T, int D>
static hipError_t launch_prefill_t(const PrefillArgs &a, hipStream_t st)
{
  const lessdec_desc *d = a.d;
  const int P = a.P, C = d->n_heavy + d->n_recent;
  const unsigned U = (unsigned)d->batch * d->heads;
  const int G = d->q_per_kv > 1 ? d->q_per_kv : 1;          // query heads per unit
  const unsigned tiles = (unsigned)(((P + 15) / 16 + kPrefillWaves - 1) / kPrefillWaves);
  const unsigned grid = (U + kXcds - 1) / kXcds * kXcds * tiles;
  const bool lambda = (d->flags & LESSDEC_FLAG_LAMBDA) != 0;
  // the prompt taken token by token under Lambda-masking, all rows at once (needs P > C: inside
  // the budget nothing is discarded and the regular rows are the same)
  const bool masked = a.masked && lambda && P > C;
  const int ring_nh = masked ? d->n_heavy : -1;
  hipError_t e;
  auto key_features = [&]() -> hipError_t {
    if (mlp_mfma_supported(d->dtype, d->head_dim, d->hidden, d->rank)) {
      MlpArgs fm;
      fm.B = d->batch; fm.Hh = d->heads; fm.rpu = P; fm.D = d->head_dim; fm.Rp = d->hidden; fm.R = d->rank;
      fm.x = (const __half *)a.K; fm.W1 = (const __half *)d->Wk1; fm.W2 = (const __half *)d->Wk2;
      fm.W3 = (const __half *)d->Wk3; fm.out = a.psi_all;
      return launch_mlp(fm, st);
    }
    FeatmapArgs fa;
    fa.x = a.K; fa.W1 = d->Wk1; fa.W2 = d->Wk2; fa.W3 = d->Wk3; fa.out = a.psi_all; fa.out_f64 = 0;
    fa.B = d->batch; fa.Hh = d->heads; fa.rpu = P; fa.D = d->head_dim; fa.Rp = d->hidden; fa.R = d->rank;
    return launch_featmap_generic(fa, d->dtype, st);
  };
  if (masked) {
    // psi of every prompt key, phi of every prompt query (Eq. 1, Eq. 2), then the masked rows
    if ((e = key_features()) != hipSuccess) return e;
    if (mlp_mfma_supported(d->dtype, d->head_dim, d->hidden, d->rank)) {
      MlpArgs fm;
      fm.B = d->batch; fm.Hh = d->heads * G; fm.rpu = P; fm.D = d->head_dim; fm.Rp = d->hidden; fm.R = d->rank;
      fm.x = (const __half *)a.Q; fm.W1 = (const __half *)d->Wq1; fm.W2 = (const __half *)d->Wq2;
      fm.W3 = nullptr; fm.out = a.phi_all;
      e = launch_mlp(fm, st);
    } else {
      FeatmapArgs fa;
      fa.x = a.Q; fa.W1 = d->Wq1; fa.W2 = d->Wq2; fa.W3 = nullptr; fa.out = a.phi_all; fa.out_f64 = 0;
      fa.B = d->batch; fa.Hh = d->heads * G; fa.rpu = P; fa.D = d->head_dim; fa.Rp = d->hidden; fa.R = d->rank;
      e = launch_featmap_generic(fa, d->dtype, st);
    }
    if (e != hipSuccess) return e;
    prefill_psimax_kernel<<<U, 256, 0, st>>>(a.psi_all, P, d->rank, a.psimax);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    {
      const int rc = (d->rank + 256 / D - 1) / (256 / D);   // rows of H per thread
#define LESSDEC_PREFIX(RC) prefill_prefix_kernel<T, D, RC><<<U, 256, 0, st>>>((const T *)a.V, a.psi_all, P, d->rank, \
                                                                              d->n_heavy, a.hpre, a.zpre)
      if (rc <= 4) LESSDEC_PREFIX(4); else if (rc <= 8) LESSDEC_PREFIX(8);
      else if (rc <= 16) LESSDEC_PREFIX(16); else LESSDEC_PREFIX(32);
#undef LESSDEC_PREFIX
    }
    if ((e = hipGetLastError()) != hipSuccess) return e;
    prefill_maskedrows_kernel<T, D><<<(U * G + kXcds - 1) / kXcds * kXcds * tiles, 64 * kPrefillWaves, 0, st>>>(
        (const T *)a.Q, (const T *)a.K, (const T *)a.V, U * G, G, P, a.phi_all, a.psi_all, a.psimax, a.hpre, a.zpre, d->rank,
        d->n_heavy, d->n_recent, (d->flags & LESSDEC_FLAG_SPARSE_DENOM) ? 1 : 0, a.lse, (T *)a.out);
  } else {
    prefill_rowpass_kernel<T, D><<<(U * G + kXcds - 1) / kXcds * kXcds * tiles, 64 * kPrefillWaves, 0, st>>>(
        (const T *)a.Q, (const T *)a.K, (const T *)a.V, U * G, G, P, a.lse, (T *)a.out);
  }
  e = hipGetLastError();
  if (e != hipSuccess) return e;
  // Column sums and selection.  Exact sums are needed of the kept tokens (they become the
  // accumulated scores) and of those whose rank is in doubt; with fp16 storage the cheap pass
  // tells which those are, with Lambda-masking the kept set is known beforehand.  Otherwise
  // (fp32 storage, or a prompt inside the budget) every column is summed exactly.
  const unsigned rank_grid = U * (unsigned)((P + 255) / 256);
  int32_t *keep = a.slot_of;
  if (P > C && (lambda || sizeof(T) == 2)) {
    if (lambda) {
      prefill_rank_kernel<<<rank_grid, 256, 0, st>>>(a.colsum, P, d->n_heavy, d->n_recent, 1, a.slot_of);
    } else {
      if constexpr (sizeof(T) == 2) {
        const unsigned agrid = (U + kXcds - 1) / kXcds * kXcds *
                               (unsigned)((((P + 15) / 16 + kApproxTiles - 1) / kApproxTiles + kPrefillWaves - 1) /
                                          kPrefillWaves);
        prefill_colapprox_kernel<D><<<agrid, 64 * kPrefillWaves, 0, st>>>((const __half *)a.Q, (const __half *)a.K, U,
                                                                         P, a.lse, G, a.approx);
        if ((e = hipGetLastError()) != hipSuccess) return e;
        prefill_scorebound_kernel<D><<<U, 256, 0, st>>>((const __half *)a.Q, (const __half *)a.K, P, G, a.bound);
        if ((e = hipGetLastError()) != hipSuccess) return e;
      }
      prefill_band_kernel<<<rank_grid, 256, 0, st>>>(a.approx, a.bound, D, G, P, d->n_heavy, d->n_recent, a.slot_of);
    }
    if ((e = hipGetLastError()) != hipSuccess) return e;
    prefill_compact_kernel<<<U, 256, 0, st>>>(a.slot_of, P, a.list, a.count);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    const int bpu = (C + 32 + 16 * kPrefillWaves - 1) / (16 * kPrefillWaves);
    prefill_colexact_kernel<T, D><<<(U + kXcds - 1) / kXcds * kXcds * (unsigned)bpu, 64 * kPrefillWaves, 0, st>>>(
        (const T *)a.Q, (const T *)a.K, U, P, a.lse, a.list, a.count, bpu, G, a.colsum);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    if (!lambda) {
      prefill_refine_kernel<<<U, 256, 0, st>>>(a.colsum, a.slot_of, P, d->n_heavy, d->n_recent, a.list);
      keep = a.list;
    }
  } else {
    prefill_colpass_kernel<T, D><<<grid, 64 * kPrefillWaves, 0, st>>>((const T *)a.Q, (const T *)a.K, U, P,
                                                                     a.lse, G, a.colsum);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    prefill_rank_kernel<<<rank_grid, 256, 0, st>>>(a.colsum, P, d->n_heavy, d->n_recent, lambda ? 1 : 0,
                                                   a.slot_of);
  }
  if ((e = hipGetLastError()) != hipSuccess) return e;
  if (!masked && (e = key_features()) != hipSuccess) return e;
  const size_t lds = (size_t)C * sizeof(int);
  if (d->rank <= 4)
    prefill_finalize_kernel<T, D, 4><<<U, 256, lds, st>>>(
      (const T *)a.K, (const T *)a.V, P, a.colsum, keep, a.psi_all, C, d->rank, (T *)d->k_cache,
      (T *)d->v_cache, d->acc, d->pos, d->psi, d->H, d->z, d->n_seen, d->pend_slot, ring_nh);
  else if (d->rank <= 8)
    prefill_finalize_kernel<T, D, 8><<<U, 256, lds, st>>>(
      (const T *)a.K, (const T *)a.V, P, a.colsum, keep, a.psi_all, C, d->rank, (T *)d->k_cache,
      (T *)d->v_cache, d->acc, d->pos, d->psi, d->H, d->z, d->n_seen, d->pend_slot, ring_nh);
  else
    prefill_finalize_kernel<T, D, 16><<<U, 256, lds, st>>>(
      (const T *)a.K, (const T *)a.V, P, a.colsum, keep, a.psi_all, C, d->rank, (T *)d->k_cache,
      (T *)d->v_cache, d->acc, d->pos, d->psi, d->H, d->z, d->n_seen, d->pend_slot, ring_nh);
  return hipGetLastError();
}

// -------------------------------------------------------------------------------------
// Row staging for the prompt taken token by token: one 16-byte vector per thread.
// -------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void prompt_rows_kernel(const uint4 *__restrict__ Q, const uint4 *__restrict__ K,
                                                          const uint4 *__restrict__ V, uint4 *__restrict__ out,
                                                          uint4 *__restrict__ qs, uint4 *__restrict__ ks,
                                                          uint4 *__restrict__ vs, const uint4 *__restrict__ outs,
                                                          unsigned U, int G, int P, int vecs, int gather,
                                                          int scatter)
{
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;   // vector index in [U * G, vecs]
  if (i >= (size_t)U * G * vecs) return;
  const size_t ug = i / vecs, c = i % vecs;                  // query row (unit, head)
  if (scatter >= 0) out[(ug * P + scatter) * vecs + c] = outs[i];
  if (gather >= 0) {
    qs[i] = Q[(ug * P + gather) * vecs + c];
    if (ug % G == 0) {                                       // the unit's key and value rows, once
      const size_t u = ug / G;
      ks[u * vecs + c] = K[(u * P + gather) * vecs + c];
      vs[u * vecs + c] = V[(u * P + gather) * vecs + c];
    }
  }
}

hipError_t launch_prompt_rows(const PromptRowsArgs &a, int gather, int scatter, hipStream_t st)
{
  const int vecs = a.D * (a.dtype == LESSDEC_DTYPE_F16 ? 2 : 4) / 16;
  const size_t n = (size_t)a.U * a.G * vecs;
  prompt_rows_kernel<<<(unsigned)((n + 255) / 256), 256, 0, st>>>(
      (const uint4 *)a.Q, (const uint4 *)a.K, (const uint4 *)a.V, (uint4 *)a.out, (uint4 *)a.qs, (uint4 *)a.ks,
      (uint4 *)a.vs, (const uint4 *)a.outs, a.U, a.G, a.P, vecs, gather, scatter);
  return hipGetLastError();
}

hipError_t launch_prefill(const PrefillArgs &a, hipStream_t st)
{
  const int D = a.d->head_dim;
  if (a.d->dtype == LESSDEC_DTYPE_F16)
    return D == 128 ? launch_prefill_t<__half, 128>(a, st) : launch_prefill_t<__half, 64>(a, st);
  return D == 128 ? launch_prefill_t<float, 128>(a, st) : launch_prefill_t<float, 64>(a, st);
}

}  // namespace lessdec
