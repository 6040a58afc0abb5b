// Wave-level helpers shared by the decode-step kernels (gfx950, wave64): DPP reductions,
// non-temporal 16-byte loads, and the encoding of the work a step leaves pending.
#pragma once

#include "lessdec_common.h"
#include "lessdec_internal.h"

namespace lessdec {

typedef unsigned int u4v __attribute__((ext_vector_type(4)));

// ---- cross-lane helpers (DPP within 16-lane rows, readlane across rows) -------------------
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
// Stores of state that go through the L2 to memory as they are issued (system scope).  A line
// that stays dirty in an L2 is written back when the kernel ends, before the next launch can
// start: with 16 MB written per launch that takes 2.4 us after plain stores, 1.3 us after
// non-temporal ones and under 0.1 us after these.
__device__ inline void store_wt(double *p, double v) { __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM); }
__device__ inline void store_wt(float *p, float v) { __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM); }
__device__ inline void store_wt(int *p, int v) { __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM); }
__device__ inline void store_wt8(void *p, const uint2 &v)
{
  unsigned long long t;
  __builtin_memcpy(&t, &v, 8);
  __hip_atomic_store(reinterpret_cast<unsigned long long *>(p), t, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
}
// 16 bytes per lane at base + offset: base must be the same for the whole wave (it goes into a
// buffer descriptor, which is how a 16-byte store gets its scope bits)
__device__ inline void store_wt16(void *base, int offset_bytes, const uint4 &v)
{
  const __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc(base, 0, 0x7fffffff, 0x00020000);
  u4v t;
  __builtin_memcpy(&t, &v, 16);
  __builtin_amdgcn_raw_buffer_store_b128(t, rs, offset_bytes, 0, 17 /* sc0 sc1 */);
}
__device__ inline void store_wt16(void *base, int offset_bytes, const float4 &v)
{
  uint4 t;
  __builtin_memcpy(&t, &v, 16);
  store_wt16(base, offset_bytes, t);
}

template <typename T>
__device__ inline typename Store<T>::Vec buffer_load_nt(__amdgpu_buffer_rsrc_t rsrc, int voffset, int soffset)
{
  typename Store<T>::Vec v;
  const u4v t = __builtin_amdgcn_raw_buffer_load_b128(rsrc, voffset, soffset, 2 /* nt */);
  __builtin_memcpy(&v.raw, &t, 16);
  return v;
}

// The pending work a step leaves behind (pend_slot): -1 nothing; otherwise the low bits name
// a slot.  Slot s < C: psi[s] is to become the psi of the key that now sits there (kept in
// pend_psi) and, unless kPendNoFold is set, the pair that sat there before (psi still in
// psi[s], value row in pend_v) is to be folded into H, z.  Slot C: the step's own pair was
// discarded; its psi is the pend_psi entry itself.
struct Pending {
  int slot;
  bool fold;
};
// A word that no step wrote (buffers never reset) still decodes to a slot in [-1, C]: every use
// of the slot is then an access inside the unit's own arrays.
__device__ inline Pending decode_pending(int ps, int C)
{
  Pending p;
  const int s = ps & 0xffff;
  p.slot = ps < 0 ? -1 : (s < C ? s : C);
  p.fold = ps >= 0 && !(ps & kPendNoFold);
  return p;
}
// Tokens seen by a unit, as loaded: a step on buffers that were never reset must stay inside the
// unit's arrays whatever the word holds, so a negative count reads as an empty cache (and a huge
// one stays clear of overflow when it is advanced and compared with positions).
__device__ inline int sane_n_seen(int n) { return n < 0 ? 0 : (n > (1 << 30) ? (1 << 30) : n); }

}  // namespace lessdec
