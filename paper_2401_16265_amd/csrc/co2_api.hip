// C ABI of libco2 (see include/co2.h): host-side validation, workspace layout,
// kernel sequencing.  Nothing here allocates or synchronises; every call
// enqueues on the caller's stream and returns.  The only device state is the
// scratch array of co2_outer_step_static below.  (The optional buffer-set
// calls, the only ones that allocate, are in co2_buffers.hip.)
#include <cmath>
#include <cstdint>
#include <cstring>
#include <limits>
#include <mutex>

#include "co2.h"
#include "co2_launch.hpp"

// Scratch of co2_outer_step_static, the entry point for callers that cannot
// allocate: one copy per GPU, held from the moment the library's code object is
// loaded on that GPU until the process ends.  In host code this name is only a
// handle for hipGetSymbolAddress; the device address it stands for on a given
// GPU is looked up once per device (static_scratch_of) and only that address is
// ever handed to kernels.
static __device__ __align__(256) unsigned char scratch[CO2_STATIC_SCRATCH_BYTES];

namespace {

thread_local int g_last_hip_error = 0;

inline int fail_hip(hipError_t e) {
  g_last_hip_error = static_cast<int>(e);
  return CO2_EHIP;
}

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
inline bool aligned256(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 255u) == 0; }
inline size_t round256(size_t b) { return (b + 255u) & ~size_t(255u); }

// [p, p+bytes) ranges overlap?
inline bool overlaps(const void* a, size_t abytes, const void* b, size_t bbytes) {
  if (!a || !b) return false;
  const uintptr_t a0 = reinterpret_cast<uintptr_t>(a), b0 = reinterpret_cast<uintptr_t>(b);
  return a0 < b0 + bbytes && b0 < a0 + abytes;
}

inline bool table_ok(int64_t n, int32_t S, const int64_t* seg_off) {
  if (n < 1 || S < 1 || !seg_off) return false;
  if (seg_off[0] != 0 || seg_off[S] != n) return false;
  for (int32_t s = 0; s < S; ++s)
    if (seg_off[s + 1] < seg_off[s]) return false;
  return true;
}

// Workspace regions (all 256-byte aligned).  Slot arrays hold one 32-byte record
// per (tile, segment) pair, indexed tile + segment.
struct Workspace {
  co2::SlotRec* slots;     // records of the norm pass (kNormTile tiles), consumed by stage 2,
                           // then of the sweep (kSweepTile tiles), kept for the next round
  co2::SlotRec* adam_slots;  // records of the AdamW step norm (kAdamTile tiles)
  double* sub[2];          // [S*split] sub-sums of each segment's slots
  double* seg_sq;          // [2][S] per-segment sums
  float* inv;              // [S] 1/Lambda
  float* scale;            // [S] norm-rescale factor min(1, phi/||m_t||_s)
  int split;               // workgroups sharing one segment's slots
  size_t bytes;
};

// Large segments have their slots added by kSegSplit workgroups; tables with
// very many segments (per-coordinate readings) have short segments and use one.
inline int split_of(int32_t S) { return S <= 4096 ? co2::kSegSplit : 1; }

inline int64_t slots_of(int64_t n, int64_t tile, int32_t S) { return (n + tile - 1) / tile + S; }

inline Workspace layout(void* base, int64_t n, int32_t S) {
  Workspace w{};
  char* p = static_cast<char*>(base);
  size_t o = 0;
  auto take = [&](size_t bytes) {
    char* r = p ? p + o : nullptr;
    o += round256(bytes);
    return r;
  };
  // one region serves the norm pass and then the sweep: sized for the smaller tile
  constexpr int64_t kMinTile = co2::kSweepTile < co2::kNormTile ? co2::kSweepTile : co2::kNormTile;
  const size_t ss = sizeof(co2::SlotRec) * static_cast<size_t>(slots_of(n, kMinTile, S));
  const size_t sa = sizeof(co2::SlotRec) * static_cast<size_t>(slots_of(n, co2::kAdamTile, S));
  w.slots = reinterpret_cast<co2::SlotRec*>(take(ss));
  w.adam_slots = reinterpret_cast<co2::SlotRec*>(take(sa));
  w.split = split_of(S);
  const size_t sub = sizeof(double) * static_cast<size_t>(S) * static_cast<size_t>(w.split);
  w.sub[0] = reinterpret_cast<double*>(take(sub));
  w.sub[1] = reinterpret_cast<double*>(take(sub));
  w.seg_sq = reinterpret_cast<double*>(take(sizeof(double) * 2 * static_cast<size_t>(S)));
  w.inv = reinterpret_cast<float*>(take(sizeof(float) * static_cast<size_t>(S)));
  w.scale = reinterpret_cast<float*>(take(sizeof(float) * static_cast<size_t>(S)));
  w.bytes = o;
  return w;
}

// Longest segment of a table, in elements.
inline int64_t longest_segment(const co2_params* p) {
  int64_t longest = 0;
  for (int32_t s = 0; s < p->S; ++s) {
    const int64_t len = p->seg_off[s + 1] - p->seg_off[s];
    if (len > longest) longest = len;
  }
  return longest;
}

// Segments that span at most this many slots have them added by one workgroup,
// Lambda included: stage 2 is then one launch instead of two.
constexpr int64_t kDirectSlots = 4096;

// Stage 2 of the gap: slots -> (per-segment sub-sums ->) Lambda, 1/Lambda.
// `use_d`: the denominator is the norm of the own previous pseudo-gradient
// (column 1 of the slots); otherwise tau*first_step_norm, or none (Lambda = 1).
inline hipError_t enqueue_lambda(const Workspace& w, int64_t tile_elems, const co2_params* p,
                                 bool use_d, const float* first_step_norm, double numer_cap,
                                 float* lambda_out, hipStream_t st) {
  if (longest_segment(p) / tile_elems + 2 <= kDirectSlots)
    return co2::launch_lambda_direct(w.slots, p->seg_off_dev, p->S, tile_elems, use_d, first_step_norm,
                                     p->penalty_c, p->alpha, p->tau, numer_cap, w.seg_sq, w.inv,
                                     lambda_out, st);
  hipError_t e = co2::launch_slot_sums(w.slots, 0, use_d, p->seg_off_dev, p->S, tile_elems,
                                       w.split, w.sub[0], w.sub[1], st);
  if (e != hipSuccess) return e;
  return co2::launch_lambda_finish(w.sub[0], w.sub[1], use_d, p->S, w.split, first_step_norm,
                                   p->penalty_c, p->alpha, p->tau, numer_cap, w.seg_sq, w.inv,
                                   lambda_out, st);
}

inline hipError_t enqueue_totals(const Workspace& w, const co2::SlotRec* slots, int col,
                                 int64_t tile_elems, const int64_t* off_dev, int32_t S,
                                 double* out, hipStream_t st) {
  hipError_t e = co2::launch_slot_sums(slots, col, false, off_dev, S, tile_elems, w.split,
                                       w.sub[0], w.sub[1], st);
  if (e != hipSuccess) return e;
  return co2::launch_totals_finish(w.sub[0], S, w.split, out, st);
}

inline hipError_t enqueue_counts(const Workspace& w, const co2_params* p, hipStream_t st) {
  hipError_t e = co2::launch_slot_sums(w.slots, 2, false, p->seg_off_dev, p->S, co2::kSweepTile,
                                       w.split, w.sub[0], w.sub[1], st);
  if (e != hipSuccess) return e;
  return co2::launch_counts_finish(w.sub[0], p->S, w.split, p->clipped_out, st);
}

// Device address of `scratch` on the current GPU, resolved on the first call
// made while that GPU is current and kept for the life of the process.
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices] = {};

int static_scratch_of_current_device(void** out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return fail_hip(e);
  if (dev < 0 || dev >= kMaxDevices) return fail_hip(hipErrorInvalidDevice);
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* ptr = nullptr;
    e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return fail_hip(e);
    if (!ptr) return fail_hip(hipErrorInvalidSymbol);
    g_scratch_ptr[dev] = ptr;
  }
  *out = g_scratch_ptr[dev];
  return CO2_OK;
}

}  // namespace

namespace co2 {

void note_hip_error(hipError_t e) { g_last_hip_error = static_cast<int>(e); }

unsigned throttle_lds_bytes(int waves_per_cu) {
  if (waves_per_cu <= 0) return 0;
  if (waves_per_cu < 3) waves_per_cu = 3;           // a workgroup may reserve at most 64 KB
  unsigned b = static_cast<unsigned>(kLdsPerCu / waves_per_cu);
  b &= ~255u;
  return b > 65536u ? 65536u : b;
}

}  // namespace co2

extern "C" {

size_t co2_workspace_bytes(int64_t n, int32_t S, int32_t K) {
  if (n < 1 || S < 1 || K < 1 || K > CO2_MAX_K) return 0;
  return layout(nullptr, n, S).bytes;
}

const char* co2_strerror(int code) {
  switch (code) {
    case CO2_OK: return "ok";
    case CO2_EINVAL: return "invalid argument (NULL, out of range, misaligned or overlapping buffer)";
    case CO2_EWORKSPACE: return "workspace missing, misaligned or smaller than co2_workspace_bytes()";
    case CO2_EHIP: return "a HIP call (kernel launch or allocation) failed (see co2_last_hip_error())";
    case CO2_ESCRATCH: return "problem too large for the static scratch of co2_outer_step_static "
                              "(co2_workspace_bytes() exceeds CO2_STATIC_SCRATCH_BYTES)";
    default: return "unknown co2 error code";
  }
}

int co2_last_hip_error(void) { return g_last_hip_error; }

}  // extern "C"

namespace {

constexpr uint32_t kVariantFlags = CO2_FLAG_CURRENT_ROUND | CO2_FLAG_ANCHOR_PULL | CO2_FLAG_NORM_CLIP;
constexpr uint32_t kAllFlags = CO2_FLAG_CARRIED_NORMS | kVariantFlags;

// Shared by co2_outer_step (fp32 pseudo-gradient buffers), co2_outer_step_bf16 /
// co2_outer_step_f16 (`dtype`: the K buffers and delta_out hold 16-bit patterns)
// and co2_outer_step_static (`use_static`: the workspace is the library's own
// per-GPU scratch array; `workspace` and `workspace_bytes` are ignored).
int outer_step_impl(const co2_params* p, float* params, const float* anchor, float* anchor_out,
                    float* momentum, const void* const* deltas, void* delta_out, int dtype,
                    const float* first_step_norm, float* lambda_out, void* workspace,
                    size_t workspace_bytes, bool use_static, void* hip_stream) {
  // ---- validation (no side effects before it passes)
  if (!p) return CO2_EINVAL;
  if (!table_ok(p->n, p->S, p->seg_off) || !p->seg_off_dev) return CO2_EINVAL;
  if (use_static && layout(nullptr, p->n, p->S).bytes > CO2_STATIC_SCRATCH_BYTES) return CO2_ESCRATCH;
  if (p->K < 1 || p->K > CO2_MAX_K || p->tau < 1 || p->step < 0) return CO2_EINVAL;
  if (!std::isfinite(p->alpha)) return CO2_EINVAL;
  if (!(p->beta >= 0.0f && p->beta < 1.0f)) return CO2_EINVAL;
  if (!(p->clip_phi > 0.0f)) return CO2_EINVAL;                 // also rejects NaN
  if (!(p->penalty_c >= 0.0f) || !std::isfinite(p->penalty_c)) return CO2_EINVAL;
  if (p->flags & ~kAllFlags) return CO2_EINVAL;
  if (p->sweep_waves_per_cu < 0 || p->sweep_waves_per_cu > 32) return CO2_EINVAL;
  if (!anchor || !anchor_out || !momentum) return CO2_EINVAL;
  if ((params == nullptr) != (delta_out == nullptr)) return CO2_EINVAL;
  const bool current = (p->flags & CO2_FLAG_CURRENT_ROUND) != 0;
  const bool norm_clip = (p->flags & CO2_FLAG_NORM_CLIP) != 0;
  const bool pull_flag = (p->flags & CO2_FLAG_ANCHOR_PULL) != 0;
  if ((p->flags & kVariantFlags) && dtype != co2::kDeltaF32) return CO2_EINVAL;
  if (pull_flag && !(p->pull_rho > 0.0f && p->pull_rho <= 1.0f)) return CO2_EINVAL;
  if ((current || pull_flag) && !params) return CO2_EINVAL;     // both need the local parameters
  if (current && p->penalty_c != 0.0f && !first_step_norm) return CO2_EINVAL;
  if (norm_clip && p->clipped_out) return CO2_EINVAL;
  const bool first = p->step == 0 && !current;                   // stale order: round 0 forms delta_out only
  const bool carried = (p->flags & CO2_FLAG_CARRIED_NORMS) != 0;
  if (p->step == 0 && carried) return CO2_EINVAL;
  // The denominator of Eq. 3: first-step norms, else the own previous pseudo-gradient's
  // norm (stale order only), else none.
  const bool need_d0 = first_step_norm == nullptr && !current;
  // Carried sums of delta_out^2 exist only if the previous call formed delta_out.
  if (carried && need_d0 && !params) return CO2_EINVAL;
  const size_t nb = sizeof(float) * static_cast<size_t>(p->n);
  const size_t db = (dtype == co2::kDeltaF32 ? sizeof(float) : sizeof(uint16_t)) * static_cast<size_t>(p->n);
  const size_t sb = sizeof(float) * static_cast<size_t>(p->S);
  const size_t cb = sizeof(int64_t) * static_cast<size_t>(p->S);
  const size_t tb = sizeof(int64_t) * (static_cast<size_t>(p->S) + 1);
  const void* vec[5] = {params, anchor, momentum, delta_out, anchor_out == anchor ? nullptr : anchor_out};
  const size_t vecb[5] = {nb, nb, nb, db, nb};
  for (int i = 0; i < 5; ++i) {
    if (!aligned16(vec[i])) return CO2_EINVAL;
    for (int j = i + 1; j < 5; ++j)
      if (overlaps(vec[i], vecb[i], vec[j], vecb[j])) return CO2_EINVAL;
  }
  if (!aligned16(p->seg_off_dev) || !aligned16(first_step_norm) || !aligned16(lambda_out) ||
      !aligned16(p->clipped_out))
    return CO2_EINVAL;
  // The per-segment arrays: no output among them may touch anything else.
  const void* small[4] = {lambda_out, p->clipped_out, first_step_norm, p->seg_off_dev};
  const size_t smallb[4] = {sb, cb, sb, tb};
  for (int i = 0; i < 4; ++i) {
    for (int j = i + 1; j < 4; ++j)
      if ((i < 2 || j < 2) && overlaps(small[i], smallb[i], small[j], smallb[j])) return CO2_EINVAL;
    for (int v = 0; v < 5; ++v) {
      // the anchor is only read unless the update is in place
      const bool writes = i < 2 || v != 1 || anchor_out == anchor;
      if (writes && overlaps(small[i], smallb[i], vec[v], vecb[v])) return CO2_EINVAL;
    }
  }
  co2::DeltaPtrs dptr{};
  int nbuf = 0;                                                  // buffers the sweep reads
  if (!first) {
    if (!deltas && !(current && p->K == 1)) return CO2_EINVAL;
    for (int k = current ? 1 : 0; k < p->K; ++k) {
      const void* dk = deltas[k];
      if (!dk || !aligned16(dk)) return CO2_EINVAL;
      // inputs may repeat among themselves, but no output may touch them
      // (delta_out may BE deltas[0]: each coordinate's old value is read before the new one
      // is stored, by the same lane)
      const bool in_place_own = k == 0 && dk == delta_out;
      if (overlaps(dk, db, params, nb) || overlaps(dk, db, momentum, nb) ||
          (!in_place_own && overlaps(dk, db, delta_out, db)) || overlaps(dk, db, anchor_out, nb) ||
          overlaps(dk, db, lambda_out, sb) || overlaps(dk, db, p->clipped_out, cb))
        return CO2_EINVAL;
      dptr.p[nbuf++] = dk;
    }
  }
  Workspace w = layout(use_static ? nullptr : workspace, p->n, p->S);
  if (!use_static) {
    if (!workspace || !aligned256(workspace) || workspace_bytes < w.bytes) return CO2_EWORKSPACE;
    for (int i = 0; i < 5; ++i)
      if (overlaps(vec[i], vecb[i], workspace, w.bytes)) return CO2_EINVAL;
    for (int i = 0; i < 4; ++i)
      if (overlaps(small[i], smallb[i], workspace, w.bytes)) return CO2_EINVAL;
    for (int k = 0; k < nbuf; ++k)
      if (overlaps(dptr.p[k], db, workspace, w.bytes)) return CO2_EINVAL;
  } else {
    // Last step before the launches, after every argument check: the address of
    // this GPU's scratch array (no allocation; a table lookup after the first call).
    void* ptr = nullptr;
    const int rc = static_scratch_of_current_device(&ptr);
    if (rc != CO2_OK) return rc;
    w = layout(ptr, p->n, p->S);
  }

  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  const float inf = std::numeric_limits<float>::infinity();
  co2::SweepArgs g{};
  g.x = params; g.a_in = anchor; g.a_out = anchor_out; g.m = momentum; g.d = dptr;
  g.dout = delta_out; g.dtype = dtype; g.inv = w.inv; g.off_dev = p->seg_off_dev; g.S = p->S; g.n = p->n;
  g.alpha = p->alpha; g.beta = p->beta;
  // Under norm rescale the sweep clamps nothing and its slot sums are those of m' itself.
  g.phi = norm_clip ? inf : p->clip_phi;
  g.rK = static_cast<float>(1.0 / static_cast<double>(p->K));
  g.slots = w.slots;
  g.waves_per_cu = p->sweep_waves_per_cu;
  g.mode.own_current = current;
  g.mode.pull = pull_flag && p->pull_rho != 1.0f;
  g.mode.rho = p->pull_rho;
  g.mode.defer_iterate = norm_clip;
  const bool has_x = params != nullptr;
  hipError_t e;

  if (first) {
    if (p->ev_sweep_begin && (e = hipEventRecord(static_cast<hipEvent_t>(p->ev_sweep_begin), st)) != hipSuccess)
      return fail_hip(e);
    if ((e = co2::launch_first_round(has_x, g, st)) != hipSuccess) return fail_hip(e);
    if (p->ev_sweep_end && (e = hipEventRecord(static_cast<hipEvent_t>(p->ev_sweep_end), st)) != hipSuccess)
      return fail_hip(e);
    if (p->clipped_out && (e = enqueue_counts(w, p, st)) != hipSuccess) return fail_hip(e);
    return CO2_OK;
  }

  // ---- the two sums of squares of Eq. 3, then Lambda per segment
  const double numer_cap = norm_clip ? static_cast<double>(p->clip_phi)
                                     : std::numeric_limits<double>::infinity();
  if (carried) {
    e = enqueue_lambda(w, co2::kSweepTile, p, need_d0, first_step_norm, numer_cap, lambda_out, st);
  } else {
    e = co2::launch_sqnorm_partials(need_d0 ? 2 : 1, momentum, norm_clip ? 0.0f : p->clip_phi,
                                    need_d0 ? dptr.p[0] : nullptr, 0.0f, dtype, p->seg_off_dev,
                                    p->S, p->n, w.slots, st);
    if (e != hipSuccess) return fail_hip(e);
    e = enqueue_lambda(w, co2::kNormTile, p, need_d0, first_step_norm, numer_cap, lambda_out, st);
  }
  if (e != hipSuccess) return fail_hip(e);

  // ---- the fused sweep
  if (p->ev_sweep_begin && (e = hipEventRecord(static_cast<hipEvent_t>(p->ev_sweep_begin), st)) != hipSuccess)
    return fail_hip(e);
  if ((e = co2::launch_fused_sweep(nbuf, has_x, g, st)) != hipSuccess) return fail_hip(e);
  if (p->ev_sweep_end && (e = hipEventRecord(static_cast<hipEvent_t>(p->ev_sweep_end), st)) != hipSuccess)
    return fail_hip(e);
  if (norm_clip) {
    // ||m_t||_s from the sums the sweep just left -> scale -> the deferred outer iterate
    e = co2::launch_slot_sums(w.slots, 0, false, p->seg_off_dev, p->S, co2::kSweepTile, w.split,
                              w.sub[0], w.sub[1], st);
    if (e != hipSuccess) return fail_hip(e);
    if ((e = co2::launch_scale_finish(w.sub[0], p->S, w.split, p->clip_phi, w.scale, st)) != hipSuccess)
      return fail_hip(e);
    if ((e = co2::launch_apply_iterate(has_x, g, w.scale, st)) != hipSuccess) return fail_hip(e);
  }
  if (p->clipped_out && (e = enqueue_counts(w, p, st)) != hipSuccess) return fail_hip(e);
  return CO2_OK;
}

}  // namespace

extern "C" {

int co2_outer_step(const co2_params* p, float* params, const float* anchor, float* anchor_out,
                   float* momentum, const float* const* deltas, float* delta_out,
                   const float* first_step_norm, float* lambda_out, void* workspace,
                   size_t workspace_bytes, void* hip_stream) {
  return outer_step_impl(p, params, anchor, anchor_out, momentum,
                         reinterpret_cast<const void* const*>(deltas), delta_out, co2::kDeltaF32,
                         first_step_norm, lambda_out, workspace, workspace_bytes, false, hip_stream);
}

int co2_outer_step_static(const co2_params* p, float* params, const float* anchor,
                          float* anchor_out, float* momentum, const float* const* deltas,
                          float* delta_out, const float* first_step_norm, float* lambda_out,
                          void* hip_stream) {
  return outer_step_impl(p, params, anchor, anchor_out, momentum,
                         reinterpret_cast<const void* const*>(deltas), delta_out, co2::kDeltaF32,
                         first_step_norm, lambda_out, nullptr, 0, true, hip_stream);
}

int co2_outer_step_bf16(const co2_params* p, float* params, const float* anchor,
                        float* anchor_out, float* momentum, const uint16_t* const* deltas_bf16,
                        uint16_t* delta_out_bf16, const float* first_step_norm,
                        float* lambda_out, void* workspace, size_t workspace_bytes,
                        void* hip_stream) {
  return outer_step_impl(p, params, anchor, anchor_out, momentum,
                         reinterpret_cast<const void* const*>(deltas_bf16), delta_out_bf16,
                         co2::kDeltaBF16, first_step_norm, lambda_out, workspace, workspace_bytes, false,
                         hip_stream);
}

int co2_outer_step_f16(const co2_params* p, float* params, const float* anchor,
                       float* anchor_out, float* momentum, const uint16_t* const* deltas_f16,
                       uint16_t* delta_out_f16, const float* first_step_norm,
                       float* lambda_out, void* workspace, size_t workspace_bytes,
                       void* hip_stream) {
  return outer_step_impl(p, params, anchor, anchor_out, momentum,
                         reinterpret_cast<const void* const*>(deltas_f16), delta_out_f16,
                         co2::kDeltaF16, first_step_norm, lambda_out, workspace, workspace_bytes, false,
                         hip_stream);
}

int co2_pseudo_grad_norms(const co2_params* p, const float* const* bufs, int32_t nbuf,
                          const float* momentum, double* sqnorm_out, void* workspace,
                          size_t workspace_bytes, void* hip_stream) {
  if (!p) return CO2_EINVAL;
  if (!table_ok(p->n, p->S, p->seg_off) || !p->seg_off_dev || !aligned16(p->seg_off_dev))
    return CO2_EINVAL;
  if (nbuf < 0 || nbuf > CO2_MAX_NORM_BUFS || (nbuf > 0 && !bufs)) return CO2_EINVAL;
  if (nbuf == 0 && !momentum) return CO2_EINVAL;
  if (momentum && !(p->clip_phi > 0.0f)) return CO2_EINVAL;
  if (!sqnorm_out || !aligned16(sqnorm_out) || !aligned16(momentum)) return CO2_EINVAL;
  const size_t nb = sizeof(float) * static_cast<size_t>(p->n);
  const int rows = nbuf + (momentum ? 1 : 0);
  const size_t ob = sizeof(double) * static_cast<size_t>(rows) * static_cast<size_t>(p->S);
  const Workspace w = layout(workspace, p->n, p->S);
  if (!workspace || !aligned256(workspace) || workspace_bytes < w.bytes) return CO2_EWORKSPACE;
  if (overlaps(sqnorm_out, ob, workspace, w.bytes) || overlaps(sqnorm_out, ob, momentum, nb))
    return CO2_EINVAL;
  for (int i = 0; i < nbuf; ++i) {
    if (!bufs[i] || !aligned16(bufs[i]) || overlaps(bufs[i], nb, sqnorm_out, ob) ||
        overlaps(bufs[i], nb, workspace, w.bytes))
      return CO2_EINVAL;
  }
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  static_assert(co2::kAdamTile <= co2::kNormTile, "the AdamW slot region must hold the norm pass's slots");
  // Rows are reduced two at a time (two read streams per launch); launches on
  // one stream run in order, so the partial slots can be reused.
  for (int r = 0; r < rows; r += 2) {
    const bool pair = r + 1 < rows;
    const float* b0 = r < nbuf ? bufs[r] : momentum;
    const float phi0 = r < nbuf ? 0.0f : p->clip_phi;
    const float* b1 = pair ? (r + 1 < nbuf ? bufs[r + 1] : momentum) : nullptr;
    const float phi1 = pair ? (r + 1 < nbuf ? 0.0f : p->clip_phi) : 0.0f;
    // partials go to the AdamW slot region (large enough: its tiles are smaller), so
    // the sums an earlier sweep carried in w.slots for the next round stay intact
    hipError_t e = co2::launch_sqnorm_partials(pair ? 2 : 1, b0, phi0, b1, phi1, co2::kDeltaF32,
                                               p->seg_off_dev, p->S, p->n, w.adam_slots, st);
    if (e != hipSuccess) return fail_hip(e);
    e = enqueue_totals(w, w.adam_slots, 0, co2::kNormTile, p->seg_off_dev, p->S,
                       sqnorm_out + static_cast<size_t>(r) * p->S, st);
    if (e != hipSuccess) return fail_hip(e);
    if (pair) {
      e = enqueue_totals(w, w.adam_slots, 1, co2::kNormTile, p->seg_off_dev, p->S,
                         sqnorm_out + static_cast<size_t>(r + 1) * p->S, st);
      if (e != hipSuccess) return fail_hip(e);
    }
  }
  return CO2_OK;
}

int co2_inner_adamw(int64_t n, const float* p_in, float* p_out, const uint16_t* grad_bf16,
                    float* exp_avg, float* exp_avg_sq, float lr, float beta1, float beta2,
                    float eps, float weight_decay, int64_t adam_step, const float* anchor,
                    float* delta_out, const int64_t* seg_off, const int64_t* seg_off_dev,
                    int32_t S, double* step_sq_out, void* workspace, size_t workspace_bytes,
                    void* hip_stream) {
  if (n < 1 || !p_in || !grad_bf16 || !exp_avg || !exp_avg_sq) return CO2_EINVAL;
  if (!p_out && !delta_out) return CO2_EINVAL;       // p' must go somewhere
  if (adam_step < 1) return CO2_EINVAL;
  if (!std::isfinite(lr) || !(beta1 >= 0.0f && beta1 < 1.0f) || !(beta2 >= 0.0f && beta2 < 1.0f) ||
      !(eps >= 0.0f) || !std::isfinite(weight_decay))
    return CO2_EINVAL;
  if ((anchor == nullptr) != (delta_out == nullptr)) return CO2_EINVAL;
  const bool want_norm = step_sq_out != nullptr;
  if (want_norm != (seg_off_dev != nullptr) || want_norm != (seg_off != nullptr) ||
      want_norm != (S != 0))
    return CO2_EINVAL;
  if (want_norm && !table_ok(n, S, seg_off)) return CO2_EINVAL;
  const size_t nb = sizeof(float) * static_cast<size_t>(n);
  const void* outs[4] = {p_out, exp_avg, exp_avg_sq, delta_out};
  const size_t outb[4] = {nb, nb, nb, nb};
  const void* ins[3] = {grad_bf16, anchor, p_in == p_out ? nullptr : p_in};
  const size_t inb[3] = {nb / 2, nb, nb};
  for (int i = 0; i < 4; ++i) {
    if (!aligned16(outs[i])) return CO2_EINVAL;
    for (int j = i + 1; j < 4; ++j)
      if (overlaps(outs[i], outb[i], outs[j], outb[j])) return CO2_EINVAL;
    for (int j = 0; j < 3; ++j)
      if (overlaps(outs[i], outb[i], ins[j], inb[j])) return CO2_EINVAL;
  }
  if (!aligned16(p_in) || !aligned16(grad_bf16) || !aligned16(anchor) ||
      !aligned16(seg_off_dev) || !aligned16(step_sq_out))
    return CO2_EINVAL;
  Workspace w{};
  if (want_norm) {
    w = layout(workspace, n, S);
    if (!workspace || !aligned256(workspace) || workspace_bytes < w.bytes) return CO2_EWORKSPACE;
    for (int i = 0; i < 4; ++i)
      if (overlaps(outs[i], outb[i], workspace, w.bytes) ||
          overlaps(outs[i], outb[i], step_sq_out, sizeof(double) * static_cast<size_t>(S)))
        return CO2_EINVAL;
  }

  // Scalars of the step, evaluated once on the host in fp64 and rounded to fp32.
  const double bc1 = 1.0 - std::pow(static_cast<double>(beta1), static_cast<double>(adam_step));
  const double bc2 = 1.0 - std::pow(static_cast<double>(beta2), static_cast<double>(adam_step));
  co2::AdamArgs g{};
  g.n = n; g.p_in = p_in; g.p_out = p_out; g.grad = grad_bf16;
  g.exp_avg = exp_avg; g.exp_avg_sq = exp_avg_sq;
  g.beta1 = beta1; g.beta2 = beta2; g.omb1 = 1.0f - beta1; g.omb2 = 1.0f - beta2;
  g.decay = 1.0f - lr * weight_decay;
  g.step_size = static_cast<float>(static_cast<double>(lr) / bc1);
  g.sqrt_bc2 = static_cast<float>(std::sqrt(bc2));
  g.eps = eps;
  g.anchor = anchor; g.dout = delta_out;
  g.off_dev = seg_off_dev; g.S = S; g.slots = want_norm ? w.adam_slots : nullptr;

  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  hipError_t e = co2::launch_adamw(g, st);
  if (e != hipSuccess) return fail_hip(e);
  if (want_norm) {
    e = enqueue_totals(w, w.adam_slots, 0, co2::kAdamTile, seg_off_dev, S, step_sq_out, st);
    if (e != hipSuccess) return fail_hip(e);
  }
  return CO2_OK;
}

int co2_sqrt_to_f32(const double* sq, float* out, int32_t S, void* hip_stream) {
  if (!sq || !out || S < 1 || !aligned16(sq) || !aligned16(out)) return CO2_EINVAL;
  if (overlaps(sq, sizeof(double) * static_cast<size_t>(S), out, sizeof(float) * static_cast<size_t>(S)))
    return CO2_EINVAL;
  hipError_t e = co2::launch_sqrt_to_f32(sq, out, S, static_cast<hipStream_t>(hip_stream));
  return e == hipSuccess ? CO2_OK : fail_hip(e);
}

int co2_copy_f32(const float* src, float* dst, int64_t n, void* hip_stream) {
  if (!src || !dst || n < 1 || !aligned16(src) || !aligned16(dst)) return CO2_EINVAL;
  const size_t nb = sizeof(float) * static_cast<size_t>(n);
  if (overlaps(src, nb, dst, nb)) return CO2_EINVAL;
  hipError_t e = co2::launch_copy_f32(src, dst, n, static_cast<hipStream_t>(hip_stream));
  return e == hipSuccess ? CO2_OK : fail_hip(e);
}

}  // extern "C"
