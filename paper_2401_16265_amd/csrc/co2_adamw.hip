// Fused AdamW local update (CO2 paper, Algorithm 1, "LU" line with AdamW as the
// base optimizer; decoupled weight decay as in Loshchilov & Hutter), fp32 master
// weights and moments, bf16 gradients.  14 bytes read and 12 written per
// coordinate; optionally also forms the round's pseudo-gradient anchor - p'
// (the payload of the all-reduce launched after the last inner step; p' itself
// then need not be stored, since the next round restarts from the new anchor:
// p_out = NULL, 8 bytes written) and the
// per-segment sum of squares of the step p' - p_in (the first inner step's norm
// is the denominator of the staleness gap, Eq. 3).
#include "co2_device.hpp"
#include "co2_launch.hpp"

namespace co2 {

struct AdamScalars {
  float beta1, beta2, omb1, omb2, decay, step_size, sqrt_bc2, eps;
};

__device__ __forceinline__ float bf16_to_f32(uint32_t bits16) {
  return __uint_as_float(bits16 << 16);
}

// One coordinate; every fp32 operation rounded once, IEEE sqrt and division.
__device__ __forceinline__ float adamw_coord(float p, float g, float& m1, float& v,
                                             const AdamScalars& h) {
  const float t1 = h.beta1 * m1;
  const float t2 = h.omb1 * g;
  m1 = t1 + t2;
  const float t3 = h.beta2 * v;
  const float t4 = (h.omb2 * g) * g;
  v = t3 + t4;
  const float pd = p * h.decay;
  // sqrtf and '/' are IEEE-correct here (hipcc's default
  // -fhip-fp32-correctly-rounded-divide-sqrt); the __fsqrt_rn intrinsic is not.
  const float denom = sqrtf(v) / h.sqrt_bc2 + h.eps;
  const float upd = h.step_size * (m1 / denom);
  return pd - upd;
}

template <bool HAS_DOUT, bool HAS_NORM>
__global__ __launch_bounds__(kWave) void adamw_step(
    int64_t n, const float* p_in, float* p_out, const uint16_t* __restrict__ grad,
    float* __restrict__ exp_avg, float* __restrict__ exp_avg_sq, AdamScalars h,
    const float* __restrict__ anchor, float* __restrict__ dout,
    const int64_t* __restrict__ off, int S, SlotRec* __restrict__ slots) {
  constexpr int U = kAdamU;
  const int64_t tile = blockIdx.x;
  const int64_t base = tile * kAdamTile;
  const int lane = threadIdx.x;
  const bool full = base + kAdamTile <= n;

  // All loads of the tile first; the segment lookup overlaps with them.
  float4 vp[U], vm[U], vv[U], va[U];
  uint2 vg[U];
  if (full) {
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int64_t row = base + int64_t(u) * kWave * 4;
      vp[u] = ld4_stream(p_in + row, lane);
      const v2u gb = ld2_stream(grad + row, lane);
      vg[u] = make_uint2(gb.x, gb.y);
      vm[u] = ld4_stream(exp_avg + row, lane);
      vv[u] = ld4_stream(exp_avg_sq + row, lane);
      if (HAS_DOUT) va[u] = ld4_stream(anchor + row, lane);
    }
  }
  int s_lo = 0;
  bool one_segment = true;
  if (HAS_NORM) {
    s_lo = seg_of(off, S, base);
    one_segment = base + kAdamTile <= off[s_lo + 1];
  }

  if (full && one_segment) {
    double acc = 0.0;
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const float pc[4] = {vp[u].x, vp[u].y, vp[u].z, vp[u].w};
      float mc[4] = {vm[u].x, vm[u].y, vm[u].z, vm[u].w};
      float vc[4] = {vv[u].x, vv[u].y, vv[u].z, vv[u].w};
      const float gc[4] = {bf16_to_f32(vg[u].x & 0xFFFFu), bf16_to_f32(vg[u].x >> 16),
                           bf16_to_f32(vg[u].y & 0xFFFFu), bf16_to_f32(vg[u].y >> 16)};
      float po[4];
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        po[e] = adamw_coord(pc[e], gc[e], mc[e], vc[e], h);
        if (HAS_NORM) acc += sq(po[e] - pc[e]);
      }
      const int64_t jb = base + int64_t(u) * kWave * 4;      // first element of this 256-wide row
      constexpr int kRowBytes = kWave * 16;
      st4_stream(exp_avg + jb, kRowBytes, lane, make_float4(mc[0], mc[1], mc[2], mc[3]));
      st4_stream(exp_avg_sq + jb, kRowBytes, lane, make_float4(vc[0], vc[1], vc[2], vc[3]));
      if (p_out) st4_stream(p_out + jb, kRowBytes, lane, make_float4(po[0], po[1], po[2], po[3]));
      if (HAS_DOUT) {
        const float ac[4] = {va[u].x, va[u].y, va[u].z, va[u].w};
        st4_stream(dout + jb, kRowBytes, lane,
                   make_float4(ac[0] - po[0], ac[1] - po[1], ac[2] - po[2], ac[3] - po[3]));
      }
    }
    if (HAS_NORM) {
      const double t = wave_sum(acc);
      write_slot(slots, tile + s_lo, lane, t, 0.0, 0.0);
    }
    return;
  }

  // Boundary or ragged tile: one segment piece after the other.
  const int64_t end = (base + kAdamTile < n) ? base + kAdamTile : n;
  const int s_hi = HAS_NORM ? seg_of(off, S, end - 1) : 0;
  for (int s = s_lo; s <= s_hi; ++s) {
    int64_t lo = base, hi = end;
    if (HAS_NORM) {
      lo = off[s] > base ? off[s] : base;
      hi = off[s + 1] < end ? off[s + 1] : end;
    }
    if (lo >= hi) continue;
    double acc = 0.0;
    for (int64_t j = lo + lane; j < hi; j += kWave) {
      const float p = p_in[j];
      float m1 = exp_avg[j], v = exp_avg_sq[j];
      const float pn = adamw_coord(p, bf16_to_f32(grad[j]), m1, v, h);
      exp_avg[j] = m1;
      exp_avg_sq[j] = v;
      if (p_out) p_out[j] = pn;
      if (HAS_DOUT) dout[j] = anchor[j] - pn;
      if (HAS_NORM) acc += sq(pn - p);
    }
    if (HAS_NORM) {
      const double t = wave_sum(acc);
      write_slot(slots, tile + s, lane, t, 0.0, 0.0);
    }
  }
}

hipError_t launch_adamw(const AdamArgs& g, hipStream_t st) {
  const unsigned tiles = static_cast<unsigned>((g.n + kAdamTile - 1) / kAdamTile);
  const AdamScalars h{g.beta1, g.beta2, g.omb1, g.omb2, g.decay, g.step_size, g.sqrt_bc2, g.eps};
  const bool has_dout = g.dout != nullptr, has_norm = g.slots != nullptr;
  const unsigned lds = throttle_lds_bytes(!has_dout ? kAdamWavesPerCu : g.p_out ? kAdamWavesWithAnchor : kAdamWavesNoStore);
#define CO2_ADAM_LAUNCH(D, N)                                                              \
  hipLaunchKernelGGL((adamw_step<D, N>), dim3(tiles), dim3(kWave), lds, st, g.n, g.p_in,   \
                     g.p_out, g.grad, g.exp_avg, g.exp_avg_sq, h, g.anchor, g.dout,        \
                     g.off_dev, g.S, g.slots)
  if (has_dout && has_norm) CO2_ADAM_LAUNCH(true, true);
  else if (has_dout) CO2_ADAM_LAUNCH(true, false);
  else if (has_norm) CO2_ADAM_LAUNCH(false, true);
  else CO2_ADAM_LAUNCH(false, false);
#undef CO2_ADAM_LAUNCH
  return hipGetLastError();
}

}  // namespace co2
