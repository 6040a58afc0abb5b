// Feature maps phi, psi (Eq. 1, Eq. 2) on the matrix cores, fp16 storage.
//
// Both layers of the MLP run on v_mfma_f32_16x16x32_f16 (wave64; lane = 16 g + c; A and B
// take 8 consecutive k from lane (g, i) for matrix row / column i; result register w of
// lane (g, c) is element [4 g + w][c]).
//
// Layer 1, H1 = W1 X^T with M = hidden units, N = 16 rows of x, K = D: fp16 x fp16 products
// are exact in fp32, only the fp32 accumulation rounds.  A wave takes 32 hidden units (two
// M-tiles) at a time, applies GELU in registers, and feeds the result straight into
// layer 2, out = W2 gelu(H1), as the B operand: lane group g already holds the hidden units
// {4 g .. 4 g + 3} of each of the two tiles, which become its 8 k-slots (the A operand, W2,
// is loaded in the same order).  The activations are fp32, so they go through the fp16
// matrix core as hi + lo (two MFMAs): hi = fp16(a), lo = fp16(a - hi) keeps 22 bits, the
// same class of error as the fp32 accumulation.  The hidden activations never leave the
// registers.
#pragma once

#include "lessdec_common.h"
#include "lessdec_internal.h"

namespace lessdec {

// An entry of the per-step exchange between the feature-map jobs and the attention waves that no
// job has written yet: a NaN that no sum of finite products can be (all bits set; a caller clears
// a workspace with a byte fill of 0xFF).
constexpr unsigned kMlpEmpty = 0xffffffffu;

typedef _Float16 v8h __attribute__((ext_vector_type(8)));
typedef _Float16 v4h __attribute__((ext_vector_type(4)));
typedef float v4f __attribute__((ext_vector_type(4)));

// Weights of one group of 32 hidden units, in operand order.
template <int D>
struct MlpTiles {
  v8h a0[D / 32], a1[D / 32];   // layer 1: hidden units hid + c and hid + 16 + c, all of D
  v8h a2;                       // layer 2: row r = c of W2 (c < R), the 8 hidden units of lane group g
};

template <int D>
__device__ inline MlpTiles<D> mlp_load_tiles(const __half *__restrict__ W1, const __half *__restrict__ W2,
                                             int Rp, int R, int hid, int g, int c)
{
  MlpTiles<D> t;
  const __half *w1a = W1 + (size_t)(hid + c) * D + 8 * g;
  const __half *w1b = w1a + (size_t)16 * D;
#pragma unroll
  for (int ks = 0; ks < D / 32; ++ks) {
    t.a0[ks] = *reinterpret_cast<const v8h *>(w1a + 32 * ks);
    t.a1[ks] = *reinterpret_cast<const v8h *>(w1b + 32 * ks);
  }
  // rows c >= R of the layer-2 operand repeat row 0 (loaded unconditionally, so that nothing
  // here waits for a load): their outputs are never looked at
  const __half *w2 = W2 + (size_t)(c < R ? c : 0) * Rp + hid + 4 * g;
  const v4h lo = *reinterpret_cast<const v4h *>(w2);
  const v4h hi = *reinterpret_cast<const v4h *>(w2 + 16);
  t.a2 = v8h{lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
  return t;
}

// One wave, one group of 32 hidden units, 16 rows of x held in bx (lane (g, c): row c,
// elements 32 ks + 8 g ..): adds W2[:, group] gelu(W1[group] x^T) to c2, whose register w
// is output r = 4 g + w of row c.
template <int D>
__device__ inline void mlp_apply_tiles(const MlpTiles<D> &t, const v8h (&bx)[D / 32], v4f &c2)
{
  v4f h0 = {0.f, 0.f, 0.f, 0.f}, h1 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int ks = 0; ks < D / 32; ++ks) {
    h0 = __builtin_amdgcn_mfma_f32_16x16x32_f16(t.a0[ks], bx[ks], h0, 0, 0, 0);
    h1 = __builtin_amdgcn_mfma_f32_16x16x32_f16(t.a1[ks], bx[ks], h1, 0, 0, 0);
  }
  // h0[w], h1[w]: hidden units hid + 4 g + w and hid + 16 + 4 g + w of row c
  v8h bhi, blo;
#pragma unroll
  for (int w = 0; w < 4; ++w) {
    const float x0 = gelu_fast_f32(h0[w]), x1 = gelu_fast_f32(h1[w]);
    const _Float16 s0 = (_Float16)x0, s1 = (_Float16)x1;
    bhi[w] = s0;
    bhi[4 + w] = s1;
    blo[w] = (_Float16)(x0 - (float)s0);
    blo[4 + w] = (_Float16)(x1 - (float)s1);
  }
  c2 = __builtin_amdgcn_mfma_f32_16x16x32_f16(t.a2, bhi, c2, 0, 0, 0);
  c2 = __builtin_amdgcn_mfma_f32_16x16x32_f16(t.a2, blo, c2, 0, 0, 0);
}

// Row c of x in operand order.  The loads are unconditional (a select on validity would
// make the caller wait for them on the spot): for a padding row pass any readable row, its
// outputs are never looked at.
template <int D>
__device__ inline void mlp_load_row(const __half *xr, int g, v8h (&bx)[D / 32])
{
#pragma unroll
  for (int ks = 0; ks < D / 32; ++ks) bx[ks] = *reinterpret_cast<const v8h *>(xr + 32 * ks + 8 * g);
}

// One job of a decode step's feature maps: (head, map, part of kMlpPartHidden hidden units,
// chunk of 64 batch rows), done by a block of four waves of 16 rows each that take the same two
// groups of 32 hidden units, so the head's weights are read once per 64 rows.  wave: 0..3 within
// the job; every thread of the block must call (one barrier inside).
// The job's 64 rows of W1 are contiguous in memory: the block fetches them with whole-line loads
// (a wave instruction = 1 KiB = four rows) into the LDS, once for its four waves, and the waves
// pick their matrix operands out of the LDS.  Operand-shaped loads from memory (16 rows x 64
// bytes per instruction, by each of the four waves) put nine times as many cache-line requests
// on the compute unit's memory pipeline, which is what slows waves streaming the cache next to
// it when this job runs inside the attention launch.  Rows are padded by 16 bytes in the LDS so
// that the 16 lanes of an operand read (same 16-byte column, 16 rows) fall into different banks.
// x: the map's rows [B, Hh, .], row b of head h at x + (b Hh + h) x_stride (x_stride = D when the
// rows are packed); W1, W2: the head's; the part's share of the layer-2 pre-activation r of unit
// b Hh + h goes to dst_map[unit * ustride + part * mlp_entry_stride(R) + r].  COHERENT: the readers run
// in the same launch, possibly on another XCD whose L2 is not coherent with this one's: the results
// go out as device-scope stores (written through).
// NWJ: the waves of one job (4: the chunk is 64 batch rows; 2: 32 rows, and two jobs share a block
// of four waves, which keeps batches of up to 32 rows from leaving half of every block idle).
// s_w1: the job's own mlp_slab_bytes(D) of LDS, 16-byte aligned; valid: false for the filler job of
// a block past the last job (it works on the last job's data and stores nothing); wave: 0..NWJ-1.
__host__ __device__ constexpr int mlp_slab_bytes(int D) { return kMlpPartHidden * (D * 2 + 16); }
template <int D, bool COHERENT, int NWJ>
__device__ __forceinline__ void mlp_parts_core(const __half *x, const __half *W1, const __half *W2, int Hh, int h, int Rp,
                                      int R, int B, int x_stride, float *dst_map, size_t ustride, int part, int chunk,
                                      unsigned char *s_w1, bool valid, int wave, int l)
{
  constexpr int kRowBytes = D * 2, kStride = kRowBytes + 16, kChunks = kRowBytes / 16;
  const int g = l / 16, c = l % 16;
  const int row = chunk * (16 * NWJ) + wave * 16 + c;      // batch row of MFMA column c
  const bool rowv = valid && row < B;
  const size_t u = (size_t)(rowv ? row : 0) * Hh + h;
  v8h bx[D / 32];
  mlp_load_row<D>(x + u * (size_t)x_stride, g, bx);        // padding: any row
  const int hid = part * kMlpPartHidden;
  const bool two = hid + 32 < Rp;                          // the last part may hold one group
  // the job's rows of W1, whole lines (rows past the last hidden unit repeat it: never used)
  constexpr int kPerThread = kMlpPartHidden * kChunks / (64 * NWJ);
  uint4 wreg[kPerThread];
  const int tid = wave * 64 + l;
#pragma unroll
  for (int i = 0; i < kPerThread; ++i) {
    const int idx = tid + 64 * NWJ * i, wr = idx / kChunks, ch = idx % kChunks;
    const int hr = hid + wr < Rp ? hid + wr : Rp - 1;
    wreg[i] = *reinterpret_cast<const uint4 *>(W1 + (size_t)hr * D + ch * 8);
  }
  // layer 2: row r = c of W2 (c < R), the 8 hidden units of lane group g in each group of 32
  v8h a2[2];
#pragma unroll
  for (int grp = 0; grp < 2; ++grp) {
    const __half *w2 = W2 + (size_t)(c < R ? c : 0) * Rp + (grp == 0 || two ? hid + 32 * grp : hid) + 4 * g;
    const v4h lo = *reinterpret_cast<const v4h *>(w2);
    const v4h hi = *reinterpret_cast<const v4h *>(w2 + 16);
    a2[grp] = v8h{lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
  }
#pragma unroll
  for (int i = 0; i < kPerThread; ++i) {
    const int idx = tid + 64 * NWJ * i, wr = idx / kChunks, ch = idx % kChunks;
    *reinterpret_cast<uint4 *>(s_w1 + wr * kStride + ch * 16) = wreg[i];
  }
  __syncthreads();
  auto tiles = [&](int grp) {
    MlpTiles<D> t;
#pragma unroll
    for (int ks = 0; ks < D / 32; ++ks) {
      t.a0[ks] = *reinterpret_cast<const v8h *>(s_w1 + (32 * grp + c) * kStride + (32 * ks + 8 * g) * 2);
      t.a1[ks] = *reinterpret_cast<const v8h *>(s_w1 + (32 * grp + 16 + c) * kStride + (32 * ks + 8 * g) * 2);
    }
    t.a2 = grp == 0 ? a2[0] : a2[1];                       // (a select: an index would put a2 into scratch memory)
    return t;
  };
  const MlpTiles<D> t0 = tiles(0);
  const MlpTiles<D> t1 = tiles(two ? 1 : 0);
  v4f c2 = {0.f, 0.f, 0.f, 0.f};
  mlp_apply_tiles<D>(t0, bx, c2);
  if (two) mlp_apply_tiles<D>(t1, bx, c2);
  // c2[w]: output r = 4 g + w of row c
  const int rp = mlp_entry_stride(R);
  if (rowv && 4 * g < rp) {                                // outputs past the rank are not kept
    float *dst = dst_map + u * ustride + (size_t)part * rp + 4 * g;
    if constexpr (COHERENT) {
      unsigned long long lo, hi;
      const float2 a = {c2[0], c2[1]}, bq = {c2[2], c2[3]};
      __builtin_memcpy(&lo, &a, 8);
      __builtin_memcpy(&hi, &bq, 8);
      __hip_atomic_store(reinterpret_cast<unsigned long long *>(dst), lo, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      __hip_atomic_store(reinterpret_cast<unsigned long long *>(dst) + 1, hi, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    } else {
      *reinterpret_cast<float4 *>(dst) = float4{c2[0], c2[1], c2[2], c2[3]};
    }
  }
}

// The jobs of a block of four waves for a step whose two maps have the same heads (one query head
// per key head): 4 / NWJ jobs, block b taking jobs b * (4 / NWJ) + ..; job = ((chunk * nparts +
// part) * 2 + map) * Hh + head: head fastest, so with Hh a multiple of 8 a head's jobs, and later
// its readers, share an XCD and its L2.  out[((u * 2 + map) * nparts + part) * mlp_entry_stride(R) + r]: a
// unit's entries lie together, its wave reads and clears them as one piece.  slabs: (4 / NWJ) *
// mlp_slab_bytes(D) of LDS.  wave4: 0..3 within the block; every thread of the block must call.
__host__ __device__ inline int mlp_parts_jobs(int Hh, int Rp, int B, int nwj)
{
  return Hh * 2 * mlp_nparts(Rp) * ((B + 16 * nwj - 1) / (16 * nwj));
}
__host__ __device__ inline int mlp_parts_nwj(int B) { return B <= 32 ? 2 : 4; }
__host__ __device__ inline int mlp_parts_blocks(int Hh, int Rp, int B)
{
  const int nwj = mlp_parts_nwj(B), per = 4 / nwj;
  return (mlp_parts_jobs(Hh, Rp, B, nwj) + per - 1) / per;
}
template <int D, bool COHERENT, int NWJ>
__device__ __forceinline__ void mlp_parts_job(const __half *q, const __half *k, const __half *Wq1, const __half *Wk1,
                                     const __half *Wq2, const __half *Wk2, int Hh, int Rp, int R, int B,
                                     int x_stride, float *out, int block, unsigned char *slabs, int wave4, int l)
{
  const int nparts = mlp_nparts(Rp), rp = mlp_entry_stride(R);
  const int sub = wave4 / NWJ, njobs = mlp_parts_jobs(Hh, Rp, B, NWJ);
  const int job = block * (4 / NWJ) + sub;
  int b = job < njobs ? job : njobs - 1;
  const int h = b % Hh; b /= Hh;
  const int map = b % 2; b /= 2;
  const int part = b % nparts;
  const int chunk = b / nparts;
  mlp_parts_core<D, COHERENT, NWJ>(map ? k : q, (map ? Wk1 : Wq1) + (size_t)h * Rp * D,
                                   (map ? Wk2 : Wq2) + (size_t)h * R * Rp, Hh, h, Rp, R, B, x_stride,
                                   out + (size_t)map * nparts * rp, (size_t)2 * nparts * rp, part, chunk,
                                   slabs + sub * mlp_slab_bytes(D), job < njobs, wave4 % NWJ, l);
}
// the same with the job width chosen from the batch
template <int D, bool COHERENT>
__device__ __forceinline__ void mlp_parts_block(const __half *q, const __half *k, const __half *Wq1, const __half *Wk1,
                                       const __half *Wq2, const __half *Wk2, int Hh, int Rp, int R, int B,
                                       int x_stride, float *out, int block, unsigned char *slabs, int wave4, int l)
{
  if (mlp_parts_nwj(B) == 2)
    mlp_parts_job<D, COHERENT, 2>(q, k, Wq1, Wk1, Wq2, Wk2, Hh, Rp, R, B, x_stride, out, block, slabs, wave4, l);
  else
    mlp_parts_job<D, COHERENT, 4>(q, k, Wq1, Wk1, Wq2, Wk2, Hh, Rp, R, B, x_stride, out, block, slabs, wave4, l);
}

// Job of a step with G query heads per key head: phi over the B x (Hk G) query rows with a weight
// set per query head, psi over the B x Hk key rows.  Jobs 0 .. nq - 1 (nq = Hk G nparts chunks) are
// phi's, head fastest; the rest psi's.  Entries: [query row][part] for phi, then [unit][part] for psi.
// slab: mlp_slab_bytes(D) of LDS.  A job index past the last job (mlp_parts_gq_jobs) is a filler: it
// works on the last job's data and stores nothing.
__host__ __device__ inline int mlp_parts_gq_jobs(int Hk, int G, int Rp, int B)
{
  return Hk * (G + 1) * mlp_nparts(Rp) * ((B + 63) / 64);
}
template <int D, bool COHERENT>
__device__ __forceinline__ void mlp_parts_gq_job(const __half *q, const __half *k, const __half *Wq1, const __half *Wk1,
                                        const __half *Wq2, const __half *Wk2, int Hk, int G, int Rp, int R, int B,
                                        float *out, int job_, unsigned char *slab, int wave, int l)
{
  const int nparts = mlp_nparts(Rp), rp = mlp_entry_stride(R), chunks = (B + 63) / 64;
  const int Hq = Hk * G, nq = Hq * nparts * chunks, njobs = mlp_parts_gq_jobs(Hk, G, Rp, B);
  const int job = job_ < njobs ? job_ : njobs - 1;
  const bool psi = job >= nq;
  int b = psi ? job - nq : job;
  const int Hh = psi ? Hk : Hq;
  const int h = b % Hh; b /= Hh;
  const int part = b % nparts;
  const int chunk = b / nparts;
  float *dst = psi ? out + (size_t)B * Hq * nparts * rp : out;
  mlp_parts_core<D, COHERENT, 4>(psi ? k : q, (psi ? Wk1 : Wq1) + (size_t)h * Rp * D,
                                 (psi ? Wk2 : Wq2) + (size_t)h * R * Rp, Hh, h, Rp, R, B, D, dst, (size_t)nparts * rp,
                                 part, chunk, slab, job_ < njobs, wave, l);
}

}  // namespace lessdec
