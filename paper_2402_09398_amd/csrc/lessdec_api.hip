// C ABI of lessdec: argument checks, workspace carve-up, kernel launches.  Nothing here
// allocates, synchronises or keeps state between calls.
#include <math.h>

#include <mutex>

#include "lessdec_internal.h"

// Built-in scratch of lessdec_step_static: part of the code object, so every GPU the library
// runs on holds its own copy at its own address for the life of the process.  In host code the
// name is only a handle for hipGetSymbolAddress; kernels get the looked-up address as an argument.
// (No `used` attribute here: the compiler gives a static device variable that host code refers to
// a global symbol in the code object, which is what the runtime's lookup needs; marked `used` it
// stays a local symbol and the lookup aborts the process.)
static __device__ __align__(256) unsigned char scratch[LESSDEC_STATIC_SCRATCH_BYTES];

namespace {

using namespace lessdec;

inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }
inline bool aligned(const void *p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }

struct Shape {
  size_t U, C, D, R, Rp, G;
};

bool shape_ok(const lessdec_desc *d, Shape *s)
{
  if (!d) return false;
  if (d->batch < 1 || d->heads < 1) return false;
  if (d->head_dim != 64 && d->head_dim != 128) return false;
  if (d->n_heavy < 0 || d->n_recent < 0) return false;
  const long C = (long)d->n_heavy + d->n_recent;
  if (C < 1 || C > LESSDEC_MAX_CAPACITY) return false;
  if (d->rank < 1 || d->rank > LESSDEC_MAX_RANK) return false;
  if (d->hidden < 1 || d->hidden > LESSDEC_MAX_HIDDEN) return false;
  if (d->dtype != LESSDEC_DTYPE_F32 && d->dtype != LESSDEC_DTYPE_F16) return false;
  if (d->flags & ~(LESSDEC_FLAG_SPARSE_DENOM | LESSDEC_FLAG_LAMBDA | LESSDEC_FLAG_PROMPT_STEPWISE)) return false;
  if ((long)d->batch * d->heads > (1L << 30)) return false;
  if (d->q_per_kv < 0 || d->q_per_kv > LESSDEC_MAX_Q_PER_KV) return false;
  if (d->q_per_kv > 1 && C > 2047) return false;
  s->U = (size_t)d->batch * d->heads;
  s->C = (size_t)C;
  s->D = (size_t)d->head_dim;
  s->R = (size_t)d->rank;
  s->Rp = (size_t)d->hidden;
  s->G = d->q_per_kv > 1 ? (size_t)d->q_per_kv : 1;
  return true;
}

// Workspace: [ f_phi U*R f64 | f_psi U*R f32 | mlp_parts 2*ceil(R'/64)*U*16 f32 |
//              prefill: 4 staged rows U*D (4 bytes each) | lse U*G*P f64, colsum U*P f64 | approx U*P f32, list U*P i32, count U i32, bound U f32 | slot_of U*P i32 | psi_all U*P*R f32 | phi_all U*G*P*R f32, psimax U*R f32, hpre U*(P/64+1)*R*D f32, zpre U*(P/64+1)*R f32 (masked prompt only) ],
// every part 256-byte aligned.
struct Workspace {
  size_t off_fphi, off_fpsi, off_parts, off_gqa, off_stage, off_lse, off_colsum, off_approx, off_list, off_count, off_bound, off_slot,
      off_psiall, off_phiall, off_psimax, off_hpre, off_zpre, total;
};

Workspace carve(const Shape &s, size_t P, unsigned flags)
{
  Workspace w;
  size_t o = 0;
  w.off_fphi = o; o = align_up(o + s.U * s.G * s.R * sizeof(double), 256);
  w.off_fpsi = o; o = align_up(o + s.U * s.R * sizeof(float), 256);
  w.off_parts = o; o = align_up(o + (s.G > 1 ? s.G + 1 : 2) * (size_t)mlp_nparts((int)s.Rp) * s.U * 16 * sizeof(float), 256);
  w.off_gqa = o; o = align_up(o + (s.G > 1 ? s.U * gqa_head_blocks((long)s.U, (int)s.G) * (s.C + 2) * sizeof(double) : 0), 256);
  w.off_stage = o; o = align_up(o + (P ? 4 * s.U * s.G * s.D * sizeof(float) : 0), 256);
  w.off_lse = o; o = align_up(o + s.U * s.G * P * sizeof(double), 256);
  w.off_colsum = o; o = align_up(o + s.U * P * sizeof(double), 256);
  w.off_approx = o; o = align_up(o + s.U * P * sizeof(float), 256);
  w.off_list = o; o = align_up(o + s.U * P * sizeof(int32_t), 256);
  w.off_count = o; o = align_up(o + (P ? s.U * sizeof(int32_t) : 0), 256);
  w.off_bound = o; o = align_up(o + (P ? s.U * sizeof(float) : 0), 256);
  w.off_slot = o; o = align_up(o + s.U * P * sizeof(int32_t), 256);
  w.off_psiall = o; o = align_up(o + s.U * P * s.R * sizeof(float), 256);
  // phi of every prompt query: only for Lambda-masking taken through the prompt token by token
  const bool masked = (flags & LESSDEC_FLAG_LAMBDA) && (flags & LESSDEC_FLAG_PROMPT_STEPWISE);
  w.off_phiall = o; o = align_up(o + (masked ? s.U * s.G * P * s.R * sizeof(float) : 0), 256);
  w.off_psimax = o; o = align_up(o + (masked && P ? s.U * s.R * sizeof(float) : 0), 256);
  const size_t nkb = P / 64 + 1;                            // prefix states of the masked prompt, one per 64 keys
  w.off_hpre = o; o = align_up(o + (masked && P ? s.U * nkb * s.R * s.D * sizeof(float) : 0), 256);
  w.off_zpre = o; o = align_up(o + (masked && P ? s.U * nkb * s.R * sizeof(float) : 0), 256);
  w.total = o;
  return w;
}

int check_desc(const lessdec_desc *d, Shape *s, size_t P)
{
  if (!shape_ok(d, s)) return LESSDEC_EINVAL;
  if (!d->k_cache || !d->v_cache || !d->acc || !d->pos || !d->psi || !d->H || !d->z || !d->n_seen ||
      !d->pend_slot || !d->pend_v || !d->pend_psi)
    return LESSDEC_EINVAL;
  if (!d->Wq1 || !d->Wq2 || !d->Wk1 || !d->Wk2 || !d->Wk3) return LESSDEC_EINVAL;
  if (!aligned(d->k_cache, 16) || !aligned(d->v_cache, 16) || !aligned(d->acc, 8) ||
      !aligned(d->z, 8) || !aligned(d->H, 16) || !aligned(d->psi, 16) || !aligned(d->pos, 4) ||
      !aligned(d->n_seen, 4) || !aligned(d->pend_slot, 4) || !aligned(d->pend_v, 16) ||
      !aligned(d->pend_psi, 4))
    return LESSDEC_EINVAL;
  if (!aligned(d->Wq1, 16) || !aligned(d->Wq2, 16) || !aligned(d->Wk1, 16) ||
      !aligned(d->Wk2, 16) || !aligned(d->Wk3, d->dtype == LESSDEC_DTYPE_F16 ? 16 : 4))
    return LESSDEC_EINVAL;
  if (!d->workspace || !aligned(d->workspace, 256)) return LESSDEC_EWORKSPACE;
  if (d->workspace_bytes < carve(*s, P, d->flags).total) return LESSDEC_EWORKSPACE;
  return LESSDEC_OK;
}

StepArgs state_args(const lessdec_desc *desc, const Shape &s)
{
  StepArgs a;
  a.C = (int)s.C; a.Nh = desc->n_heavy; a.Nr = desc->n_recent; a.R = desc->rank; a.Rp = desc->hidden;
  a.flags = desc->flags;
  a.k_cache = desc->k_cache; a.v_cache = desc->v_cache; a.acc = desc->acc; a.pos = desc->pos;
  a.psi = desc->psi; a.H = desc->H; a.z = desc->z; a.n_seen = desc->n_seen;
  a.pend_slot = desc->pend_slot; a.pend_v = desc->pend_v; a.pend_psi = desc->pend_psi;
  a.q = a.k = a.v = nullptr; a.out = nullptr; a.evicted_pos = nullptr; a.x_stride = desc->head_dim;
  a.U = (int)s.U; a.Hh = desc->heads; a.B = desc->batch;
  a.f_phi = nullptr; a.f_phi32 = nullptr; a.f_psi = nullptr; a.mlp_parts = nullptr; a.mlp_out = nullptr;
  a.gqa_parts = nullptr;
  a.Wk3 = desc->Wk3; a.Wk2 = desc->Wk2;
  return a;
}

// The streaming decode path (one wave per unit) serves this descriptor.
bool use_wpu(const lessdec_desc *desc, const Shape &s)
{
  return s.G == 1 && desc->batch < 65536 && desc->heads < 65536 &&
         wpu_supported(desc->dtype, desc->head_dim, (int)s.C, desc->hidden, desc->rank);
}

// Several query heads per unit on the streaming kernel, which finishes the feature maps itself
// from their parts.
bool gq_parts(const lessdec_desc *desc, const Shape &s)
{
  return s.G > 1 && desc->batch < 65536 && desc->heads < 65536 &&
         gqs_supported(desc->dtype, desc->head_dim, (int)s.C, desc->rank, (int)s.G) &&
         mlp_mfma_supported(desc->dtype, desc->head_dim, desc->hidden, desc->rank) && gqs_takes_parts(desc->hidden);
}

MlpPartsArgs parts_args(const lessdec_desc *desc, const void *q, const void *k, float *out)
{
  MlpPartsArgs fm;
  fm.q = (const __half *)q; fm.k = (const __half *)k;
  fm.Wq1 = (const __half *)desc->Wq1; fm.Wq2 = (const __half *)desc->Wq2;
  fm.Wk1 = (const __half *)desc->Wk1; fm.Wk2 = (const __half *)desc->Wk2;
  fm.out = out;
  fm.B = desc->batch; fm.Hh = desc->heads; fm.D = desc->head_dim; fm.Rp = desc->hidden; fm.R = desc->rank;
  return fm;
}

// The per-step exchange array of the streaming path starts out empty (see wpu_step_kernel).
hipError_t empty_exchange(const lessdec_desc *desc, const Shape &s, hipStream_t st)
{
  if (!use_wpu(desc, s) && !gq_parts(desc, s)) return hipSuccess;
  const Workspace w = carve(s, 0, desc->flags);
  return launch_fill_empty(reinterpret_cast<float *>(static_cast<char *>(desc->workspace) + w.off_parts),
                           (s.G > 1 ? s.G + 1 : 2) * (size_t)mlp_nparts((int)s.Rp) * s.U * 16, st);
}

// Device address of `scratch` on the current device, looked up once per device.
constexpr int kMaxDevices = 64;
void *g_scratch_addr[kMaxDevices];
std::mutex g_scratch_mutex;

int static_scratch(void **addr)
{
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return LESSDEC_EHIP;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_addr[dev]) {
    void *p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return LESSDEC_EHIP;
    g_scratch_addr[dev] = p;
  }
  *addr = g_scratch_addr[dev];
  return LESSDEC_OK;
}

}  // namespace

extern "C" {

size_t lessdec_workspace_bytes(const lessdec_desc *desc, int32_t max_prompt)
{
  Shape s;
  if (!shape_ok(desc, &s) || max_prompt < 0) return 0;
  return carve(s, (size_t)max_prompt, desc->flags).total;
}

int lessdec_state_reset(const lessdec_desc *desc, void *hip_stream)
{
  Shape s;
  int rc = check_desc(desc, &s, 0);
  if (rc) return rc;
  if (empty_exchange(desc, s, (hipStream_t)hip_stream) != hipSuccess) return LESSDEC_EHIP;
  return launch_reset(desc, (hipStream_t)hip_stream) == hipSuccess ? LESSDEC_OK : LESSDEC_EHIP;
}

int lessdec_state_sync(const lessdec_desc *desc, void *hip_stream)
{
  Shape s;
  int rc = check_desc(desc, &s, 0);
  if (rc) return rc;
  const StepArgs a = state_args(desc, s);
  return launch_state_sync(a, desc->dtype, desc->head_dim, (hipStream_t)hip_stream) == hipSuccess
             ? LESSDEC_OK : LESSDEC_EHIP;
}

}  // extern "C"

namespace {

// x_stride: elements between the rows of consecutive units in q, k, v, out (head_dim for the
// packed [B,Hh,D] rows of the public calls; the streaming path alone takes other values).
int step_features_impl(const lessdec_desc *desc, const void *q, const void *k, int x_stride, void *hip_stream)
{
  Shape s;
  int rc = check_desc(desc, &s, 0);
  if (rc) return rc;
  if (!q || !k || !aligned(q, 16) || !aligned(k, 16)) return LESSDEC_EINVAL;
  hipStream_t st = (hipStream_t)hip_stream;
  const Workspace w = carve(s, 0, desc->flags);
  char *ws = static_cast<char *>(desc->workspace);
  if (use_wpu(desc, s)) {
    // matrix-core feature maps up to the layer-2 sums
    MlpPartsArgs fm = parts_args(desc, q, k, reinterpret_cast<float *>(ws + w.off_parts));
    fm.x_stride = x_stride;
    return launch_mlp_parts(fm, st) == hipSuccess ? LESSDEC_OK : LESSDEC_EHIP;
  }
  if (x_stride != desc->head_dim) return LESSDEC_EINVAL;
  if (gq_parts(desc, s)) {
    // several query heads per unit, streaming kernel: both maps up to the layer-2 sums
    MlpPartsArgs fm = parts_args(desc, q, k, reinterpret_cast<float *>(ws + w.off_parts));
    return launch_mlp_parts_gq(fm, (int)s.G, st) == hipSuccess ? LESSDEC_OK : LESSDEC_EHIP;
  }
  if (s.G > 1 && mlp_mfma_supported(desc->dtype, desc->head_dim, desc->hidden, desc->rank)) {
    // several query heads per unit: both maps complete on the matrix cores, fp32 results
    MlpArgs fm;
    fm.B = desc->batch; fm.rpu = 1; fm.D = desc->head_dim; fm.Rp = desc->hidden; fm.R = desc->rank;
    fm.Hh = desc->heads * (int)s.G;                     // q rows [B,Hh,G]: query head h G + g
    fm.x = (const __half *)q; fm.W1 = (const __half *)desc->Wq1; fm.W2 = (const __half *)desc->Wq2;
    fm.W3 = nullptr; fm.out = reinterpret_cast<float *>(ws + w.off_fphi);
    MlpArgs fk = fm;
    fk.Hh = desc->heads;
    fk.x = (const __half *)k; fk.W1 = (const __half *)desc->Wk1; fk.W2 = (const __half *)desc->Wk2;
    fk.W3 = (const __half *)desc->Wk3; fk.out = reinterpret_cast<float *>(ws + w.off_fpsi);
    return launch_mlp_pair(fm, fk, st) == hipSuccess ? LESSDEC_OK : LESSDEC_EHIP;
  }
  // general path: phi(q), psi(k) in fp64
  FeatmapArgs fa;
  fa.B = desc->batch; fa.Hh = desc->heads * (int)s.G; fa.rpu = 1;   // q rows [B,Hh,G]: query head h G + g
  fa.D = desc->head_dim; fa.Rp = desc->hidden; fa.R = desc->rank;
  fa.x = q; fa.W1 = desc->Wq1; fa.W2 = desc->Wq2; fa.W3 = nullptr;
  fa.out = reinterpret_cast<double *>(ws + w.off_fphi); fa.out_f64 = 1;
  if (launch_featmap_generic(fa, desc->dtype, st) != hipSuccess) return LESSDEC_EHIP;
  fa.Hh = desc->heads;
  fa.x = k; fa.W1 = desc->Wk1; fa.W2 = desc->Wk2; fa.W3 = desc->Wk3;
  fa.out = reinterpret_cast<float *>(ws + w.off_fpsi); fa.out_f64 = 0;
  if (launch_featmap_generic(fa, desc->dtype, st) != hipSuccess) return LESSDEC_EHIP;
  return LESSDEC_OK;
}

int step_attend_impl(const lessdec_desc *desc, const void *q, const void *k, const void *v, void *out,
                     int32_t *evicted_pos, int x_stride, void *hip_stream)
{
  Shape s;
  int rc = check_desc(desc, &s, 0);
  if (rc) return rc;
  if (!q || !k || !v || !out) return LESSDEC_EINVAL;
  if (!aligned(q, 16) || !aligned(k, 16) || !aligned(v, 16) || !aligned(out, 16) ||
      !aligned(evicted_pos, 4))
    return LESSDEC_EINVAL;
  hipStream_t st = (hipStream_t)hip_stream;
  StepArgs a = state_args(desc, s);
  a.q = q; a.k = k; a.v = v; a.out = out; a.evicted_pos = evicted_pos; a.x_stride = x_stride;
  const Workspace w = carve(s, 0, desc->flags);
  char *ws = static_cast<char *>(desc->workspace);
  if (x_stride != desc->head_dim && !use_wpu(desc, s)) return LESSDEC_EINVAL;
  if (s.G > 1) {
    if (mlp_mfma_supported(desc->dtype, desc->head_dim, desc->hidden, desc->rank))
      a.f_phi32 = reinterpret_cast<float *>(ws + w.off_fphi);
    else
      a.f_phi = reinterpret_cast<double *>(ws + w.off_fphi);
    a.f_psi = reinterpret_cast<float *>(ws + w.off_fpsi);
    a.gqa_parts = reinterpret_cast<double *>(ws + w.off_gqa);
    if (gq_parts(desc, s)) a.mlp_parts = a.mlp_out = reinterpret_cast<float *>(ws + w.off_parts);
    if (gqs_supported(desc->dtype, desc->head_dim, (int)s.C, desc->rank, (int)s.G))
      return launch_step_gqs(a, (int)s.G, desc->head_dim, st) == hipSuccess ? LESSDEC_OK : LESSDEC_EHIP;
    return launch_step_gqa(a, (int)s.G, desc->dtype, desc->head_dim, st) == hipSuccess ? LESSDEC_OK : LESSDEC_EHIP;
  }
  if (use_wpu(desc, s)) {
    a.mlp_parts = a.mlp_out = reinterpret_cast<float *>(ws + w.off_parts);     // one wave per unit
    return launch_step_wpu(a, desc->head_dim, st) == hipSuccess ? LESSDEC_OK : LESSDEC_EHIP;
  }
  a.f_phi = reinterpret_cast<double *>(ws + w.off_fphi);           // one block per unit
  a.f_psi = reinterpret_cast<float *>(ws + w.off_fpsi);
  return launch_step(a, desc->dtype, desc->head_dim, st) == hipSuccess ? LESSDEC_OK : LESSDEC_EHIP;
}

int step_impl(const lessdec_desc *desc, const void *q, const void *k, const void *v, void *out,
              int32_t *evicted_pos, int x_stride, void *hip_stream)
{
  // argument checks of both halves first, so that nothing is launched on an error
  Shape s;
  int rc = check_desc(desc, &s, 0);
  if (rc) return rc;
  if (!q || !k || !v || !out) return LESSDEC_EINVAL;
  if (!aligned(q, 16) || !aligned(k, 16) || !aligned(v, 16) || !aligned(out, 16) ||
      !aligned(evicted_pos, 4))
    return LESSDEC_EINVAL;
  if (use_wpu(desc, s) && wpu_fusable(desc->batch, desc->heads, desc->head_dim, (int)s.C, desc->hidden, desc->rank)) {
    // feature maps and attention in one launch
    StepArgs a = state_args(desc, s);
    a.q = q; a.k = k; a.v = v; a.out = out; a.evicted_pos = evicted_pos; a.x_stride = x_stride;
    const Workspace w = carve(s, 0, desc->flags);
    float *parts = reinterpret_cast<float *>(static_cast<char *>(desc->workspace) + w.off_parts);
    a.mlp_parts = a.mlp_out = parts;
    MlpPartsArgs fm = parts_args(desc, q, k, parts);
    fm.x_stride = x_stride;
    return launch_step_wpu(a, desc->head_dim, (hipStream_t)hip_stream, &fm) == hipSuccess ? LESSDEC_OK : LESSDEC_EHIP;
  }
  if (gq_parts(desc, s) && x_stride == desc->head_dim &&
      gqs_fusable(desc->head_dim, (int)s.C, desc->hidden, desc->rank, (int)s.G)) {
    // several query heads per unit: feature maps and attention in one launch
    StepArgs a = state_args(desc, s);
    a.q = q; a.k = k; a.v = v; a.out = out; a.evicted_pos = evicted_pos; a.x_stride = x_stride;
    const Workspace w = carve(s, 0, desc->flags);
    float *parts = reinterpret_cast<float *>(static_cast<char *>(desc->workspace) + w.off_parts);
    a.mlp_parts = a.mlp_out = parts;
    MlpPartsArgs fm = parts_args(desc, q, k, parts);
    return launch_step_gqs(a, (int)s.G, desc->head_dim, (hipStream_t)hip_stream, &fm) == hipSuccess ? LESSDEC_OK
                                                                                                     : LESSDEC_EHIP;
  }
  rc = step_features_impl(desc, q, k, x_stride, hip_stream);
  if (rc) return rc;
  return step_attend_impl(desc, q, k, v, out, evicted_pos, x_stride, hip_stream);
}

}  // namespace

extern "C" {

int lessdec_step_features(const lessdec_desc *desc, const void *q, const void *k, void *hip_stream)
{
  return desc ? step_features_impl(desc, q, k, desc->head_dim, hip_stream) : LESSDEC_EINVAL;
}

int lessdec_step_attend(const lessdec_desc *desc, const void *q, const void *k, const void *v, void *out,
                        int32_t *evicted_pos, void *hip_stream)
{
  return desc ? step_attend_impl(desc, q, k, v, out, evicted_pos, desc->head_dim, hip_stream) : LESSDEC_EINVAL;
}

int lessdec_step(const lessdec_desc *desc, const void *q, const void *k, const void *v, void *out,
                 int32_t *evicted_pos, void *hip_stream)
{
  return desc ? step_impl(desc, q, k, v, out, evicted_pos, desc->head_dim, hip_stream) : LESSDEC_EINVAL;
}

int lessdec_step_launches(const lessdec_desc *desc)
{
  Shape s;
  if (!shape_ok(desc, &s)) return 0;
  if (gq_parts(desc, s) && gqs_fusable(desc->head_dim, (int)s.C, desc->hidden, desc->rank, (int)s.G)) return 1;
  if (s.G > 1)                                                              // feature maps, heads, (finishing launch)
    return !gqs_supported(desc->dtype, desc->head_dim, (int)s.C, desc->rank, (int)s.G) &&
                   gqa_head_blocks((long)s.U, (int)s.G) > 1 ? 3 : 2;
  if (use_wpu(desc, s))
    return wpu_fusable(desc->batch, desc->heads, desc->head_dim, (int)s.C, desc->hidden, desc->rank) ? 1 : 2;
  return 3;                                                                 // phi, psi, step
}

int lessdec_step_static(const lessdec_desc *desc, const void *q, const void *k, const void *v, void *out,
                        int32_t *evicted_pos, void *hip_stream)
{
  Shape s;
  if (!shape_ok(desc, &s)) return LESSDEC_EINVAL;
  if (carve(s, 0, desc->flags).total > (size_t)LESSDEC_STATIC_SCRATCH_BYTES) return LESSDEC_ESCRATCH;
  lessdec_desc d = *desc;
  void *addr = nullptr;
  const int rc = static_scratch(&addr);
  if (rc) return rc;
  d.workspace = addr;
  d.workspace_bytes = LESSDEC_STATIC_SCRATCH_BYTES;
  // always the two launches: the one-launch form of lessdec_step needs an exchange array that is
  // empty when the step starts, which a buffer shared by descriptors of any shape cannot promise
  if (!q || !k || !v || !out) return LESSDEC_EINVAL;
  if (!aligned(q, 16) || !aligned(k, 16) || !aligned(v, 16) || !aligned(out, 16) || !aligned(evicted_pos, 4))
    return LESSDEC_EINVAL;
  int rc2 = check_desc(&d, &s, 0);
  if (rc2) return rc2;
  rc2 = lessdec_step_features(&d, q, k, hip_stream);
  if (rc2) return rc2;
  return lessdec_step_attend(&d, q, k, v, out, evicted_pos, hip_stream);
}

int lessdec_prefill(const lessdec_desc *desc, const void *Q, const void *K, const void *V,
                    int32_t P, void *out, void *hip_stream)
{
  Shape s;
  if (P < 1) return LESSDEC_EINVAL;
  int rc = check_desc(desc, &s, (size_t)P);
  if (rc) return rc;
  if (!Q || !K || !V) return LESSDEC_EINVAL;
  if (!aligned(Q, 16) || !aligned(K, 16) || !aligned(V, 16) || !aligned(out, 16))
    return LESSDEC_EINVAL;
  const Workspace w = carve(s, (size_t)P, desc->flags);
  char *ws = static_cast<char *>(desc->workspace);
  // Lambda-masking taken through a prompt longer than the budget: the cache every token meets is
  // known beforehand, so all rows are computed at once (same results as the loop below)
  const bool masked = (desc->flags & LESSDEC_FLAG_PROMPT_STEPWISE) && (desc->flags & LESSDEC_FLAG_LAMBDA) &&
                      (size_t)P > s.C;
  if ((desc->flags & LESSDEC_FLAG_PROMPT_STEPWISE) && !masked) {
    // the generation loop over the prompt: token t's rows are staged as one step's q, k, v
    hipStream_t st = (hipStream_t)hip_stream;
    PromptRowsArgs r;
    r.Q = Q; r.K = K; r.V = V; r.out = out; r.P = P; r.U = (unsigned)s.U; r.D = desc->head_dim;
    r.dtype = desc->dtype; r.G = (int)s.G;
    const size_t part = s.U * s.G * s.D * sizeof(float);
    r.qs = ws + w.off_stage;
    r.ks = ws + w.off_stage + 1 * part;
    r.vs = ws + w.off_stage + 2 * part;
    r.outs = ws + w.off_stage + 3 * part;
    if (empty_exchange(desc, s, st) != hipSuccess) return LESSDEC_EHIP;
    if (launch_reset(desc, st) != hipSuccess) return LESSDEC_EHIP;
    if (use_wpu(desc, s) && out && (size_t)P * s.D < ((size_t)1 << 31)) {
      // the streaming path reads token t's rows where they lie in the prompt arrays and writes its
      // output row there: one step (one launch on large shapes) per token, nothing staged
      const size_t e = desc->dtype == LESSDEC_DTYPE_F16 ? 2 : 4;
      for (int32_t t = 0; t < P; ++t) {
        const size_t off = (size_t)t * s.D * e;
        rc = step_impl(desc, static_cast<const char *>(Q) + off, static_cast<const char *>(K) + off,
                       static_cast<const char *>(V) + off, static_cast<char *>(out) + off, nullptr, (int)(P * s.D),
                       hip_stream);
        if (rc) return rc;
      }
      return LESSDEC_OK;
    }
    for (int32_t t = 0; t < P; ++t) {
      if (launch_prompt_rows(r, t, (out && t > 0) ? t - 1 : -1, st) != hipSuccess) return LESSDEC_EHIP;
      if ((rc = lessdec_step_features(desc, r.qs, r.ks, hip_stream)) != LESSDEC_OK) return rc;
      if ((rc = lessdec_step_attend(desc, r.qs, r.ks, r.vs, r.outs, nullptr, hip_stream)) != LESSDEC_OK) return rc;
    }
    if (out && launch_prompt_rows(r, -1, P - 1, st) != hipSuccess) return LESSDEC_EHIP;
    return LESSDEC_OK;
  }
  PrefillArgs a;
  a.d = desc; a.Q = Q; a.K = K; a.V = V; a.P = P; a.out = out;
  a.lse = reinterpret_cast<double *>(ws + w.off_lse);
  a.colsum = reinterpret_cast<double *>(ws + w.off_colsum);
  a.slot_of = reinterpret_cast<int32_t *>(ws + w.off_slot);
  a.approx = reinterpret_cast<float *>(ws + w.off_approx);
  a.list = reinterpret_cast<int32_t *>(ws + w.off_list);
  a.count = reinterpret_cast<int32_t *>(ws + w.off_count);
  a.bound = reinterpret_cast<float *>(ws + w.off_bound);
  a.psi_all = reinterpret_cast<float *>(ws + w.off_psiall);
  a.phi_all = reinterpret_cast<float *>(ws + w.off_phiall);
  a.psimax = reinterpret_cast<float *>(ws + w.off_psimax);
  a.hpre = reinterpret_cast<float *>(ws + w.off_hpre);
  a.zpre = reinterpret_cast<float *>(ws + w.off_zpre);
  a.masked = masked ? 1 : 0;
  if (empty_exchange(desc, s, (hipStream_t)hip_stream) != hipSuccess) return LESSDEC_EHIP;
  return launch_prefill(a, (hipStream_t)hip_stream) == hipSuccess ? LESSDEC_OK : LESSDEC_EHIP;
}

const char *lessdec_strerror(int code)
{
  switch (code) {
    case LESSDEC_OK: return "ok";
    case LESSDEC_EINVAL: return "invalid argument (shape, NULL or misaligned pointer, unsupported size)";
    case LESSDEC_EWORKSPACE: return "workspace missing, misaligned or too small";
    case LESSDEC_EHIP: return "HIP launch failed";
    case LESSDEC_ESCRATCH: return "shape needs more scratch than the built-in buffer of lessdec_step_static holds";
    default: return "unknown lessdec error";
  }
}

int32_t lessdec_budget_tokens(double percent, int32_t max_len)
{
  if (!(percent >= 0.0) || max_len < 0) return 0;
  const double tokens = percent * (double)max_len / 100.0;
  const double half = floor(tokens * 0.5 + 1e-9);
  if (half > 1.0e9) return 0;
  return (int32_t)(2.0 * half);
}

}  // extern "C"
