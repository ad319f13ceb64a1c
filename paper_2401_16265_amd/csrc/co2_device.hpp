// Device-side helpers shared by the gfx950 kernels of libco2: launch geometry,
// wavefront (64-lane) reductions through DPP, segment lookup, streaming
// loads/stores.
//
// Geometry.  Every streaming kernel here runs ONE wavefront per workgroup over
// an aligned tile of the flat index space, one tile per workgroup, in dispatch
// order.  On MI355X a mixed read/write stream over many buffers is fastest when
// each compute unit keeps only about 56-64 KB of loads in flight (4-8
// wavefronts of 3+K 16-byte loads per lane): more resident wavefronts widen the
// window of DRAM pages touched at once and cost 10-15 % of HBM bandwidth.  The
// launch code therefore reserves dynamic LDS per workgroup purely to cap the
// number of resident wavefronts per compute unit (the kernels never touch it).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "co2.h"

namespace co2 {

constexpr int kWave = 64;                          // lanes per wavefront = threads per workgroup
constexpr int kSweepU = 1;                         // 16-byte vectors per lane and stream, fused sweep
constexpr int kNormU = 4;                          // ... norm pass
constexpr int kAdamU = 1;                          // ... AdamW step (two per lane cost 9-11 %: the step's
                                                   // IEEE square root and divisions keep a wavefront busy
                                                   // for about as long as its loads take, with nothing in flight)
constexpr int64_t kSweepTile = int64_t(kWave) * 4 * kSweepU;   // 256 elements
constexpr int64_t kNormSub = int64_t(kWave) * 4 * kNormU;      // 1024 elements read at once by the norm pass
constexpr int kNormSubs = 16;                      // such pieces per norm-pass tile (one record per tile:
                                                   // a record per 1024 elements cost the pass 5-8 %)
constexpr int64_t kNormTile = kNormSub * kNormSubs;            // 16384 elements
constexpr int64_t kAdamTile = int64_t(kWave) * 4 * kAdamU;     // 256 elements
constexpr int kLdsPerCu = 160 * 1024;              // gfx950 LDS per compute unit
constexpr int kReduceBlock = 256;                  // threads of the small reduction kernels
constexpr int kReduceWaves = kReduceBlock / kWave;
constexpr int kSegSplit = 32;                      // workgroups that share one segment's slots

// One 32-byte record per (tile, segment) slot, written with a single coalesced
// 32-byte store (8-byte partial stores cost a full 32-byte HBM write each).
//   v[0] sum of Clip(m,phi)^2 (or the only quantity of a one-column producer)
//   v[1] sum of d^2            v[2] count of clamped coordinates      v[3] unused
struct alignas(32) SlotRec {
  double v[4];
};

// Storage type of the pseudo-gradient buffers (the payload of the all-reduce):
// fp32, or bf16 / IEEE fp16 bit patterns for reduced-precision transport.
enum DeltaType : int { kDeltaF32 = 0, kDeltaBF16 = 1, kDeltaF16 = 2 };

// The workers' pseudo-gradient buffers that one sweep reads.
struct DeltaPtrs {
  const void* p[CO2_MAX_K];
};

// Section 3.3: Clip(chi, phi) = max{-phi, min{chi, phi}}.
__device__ __forceinline__ float clip_coord(float chi, float phi) {
  return fmaxf(-phi, fminf(chi, phi));
}

// Index s of the segment that holds flat index j, 0 <= j < off[S]:
// off[s] <= j < off[s+1].  Empty segments are skipped.
__device__ __forceinline__ int seg_of(const int64_t* __restrict__ off, int S, int64_t j) {
  int lo = 0, hi = S;                              // off[lo] <= j < off[hi]
  while (hi - lo > 1) {
    const int mid = (lo + hi) >> 1;
    if (off[mid] <= j) lo = mid; else hi = mid;
  }
  return lo;
}

// One DPP lane exchange of a double (two 32-bit halves).  Needs all 64 lanes
// of the wavefront active.
template <int CTRL>
__device__ __forceinline__ double dpp_move(double v) {
  int lo = __double2loint(v), hi = __double2hiint(v);
  lo = __builtin_amdgcn_update_dpp(0, lo, CTRL, 0xF, 0xF, false);
  hi = __builtin_amdgcn_update_dpp(0, hi, CTRL, 0xF, 0xF, false);
  return __hiloint2double(hi, lo);
}

__device__ __forceinline__ double read_lane(double v, int lane) {
  const int lo = __builtin_amdgcn_readlane(__double2loint(v), lane);
  const int hi = __builtin_amdgcn_readlane(__double2hiint(v), lane);
  return __hiloint2double(hi, lo);
}

// Sum over the 64 lanes of a wavefront, identical in every lane and for every
// run: a butterfly inside each row of 16 lanes (quad_perm [1,0,3,2], quad_perm
// [2,3,0,1], row_half_mirror, row_mirror), then the four row sums added in
// row order.
__device__ __forceinline__ double wave_sum(double v) {
  v += dpp_move<0xB1>(v);
  v += dpp_move<0x4E>(v);
  v += dpp_move<0x141>(v);
  v += dpp_move<0x140>(v);
  const double r0 = read_lane(v, 0), r1 = read_lane(v, 16);
  const double r2 = read_lane(v, 32), r3 = read_lane(v, 48);
  return ((r0 + r1) + r2) + r3;
}

// Tells the compiler that a value every lane holds identically IS wavefront-uniform
// (kept in scalar registers: scalar loads, no per-lane address handling), where its own
// analysis gives up (values carried around loops that also contain per-lane loops).
__device__ __forceinline__ int uniform(int v) { return __builtin_amdgcn_readfirstlane(v); }
__device__ __forceinline__ int64_t uniform(int64_t v) {
  const uint32_t lo = static_cast<uint32_t>(__builtin_amdgcn_readfirstlane(static_cast<int>(static_cast<uint64_t>(v))));
  const uint32_t hi = static_cast<uint32_t>(__builtin_amdgcn_readfirstlane(static_cast<int>(static_cast<uint64_t>(v) >> 32)));
  return static_cast<int64_t>((static_cast<uint64_t>(hi) << 32) | lo);
}

// Lanes 0..3 of the wavefront write one slot record; v0..v2 are wavefront-uniform.
__device__ __forceinline__ void write_slot(SlotRec* __restrict__ rec, int64_t slot, int lane,
                                           double v0, double v1, double v2) {
  if (lane < 4) {
    const double v = lane == 0 ? v0 : lane == 1 ? v1 : lane == 2 ? v2 : 0.0;
    reinterpret_cast<double*>(rec + slot)[lane] = v;
  }
}

// Sum over a kReduceBlock-thread workgroup (the small reduction kernels only);
// every thread must call it.  `lds` holds kReduceWaves doubles.
__device__ __forceinline__ double block_sum(double v, double* lds) {
  const double w = wave_sum(v);
  const int wave = threadIdx.x / kWave;
  __syncthreads();                                 // previous use of lds is over
  if ((threadIdx.x & (kWave - 1)) == 0) lds[wave] = w;
  __syncthreads();
  double t = lds[0];
#pragma unroll
  for (int i = 1; i < kReduceWaves; ++i) t += lds[i];
  return t;
}

// Streaming accesses: every element of every buffer is touched once per kernel,
// so loads and stores carry the non-temporal hint.
typedef unsigned v2u __attribute__((ext_vector_type(2)));

// Streaming stores of a whole tile row: buffer stores with the non-temporal and
// sc1 (write-through) cache-policy bits.  Written lines then leave the L2 in the
// order they were produced instead of lingering as dirty lines that are evicted
// later in scattered order, which is worth about 3 % of HBM bandwidth on a mixed
// read/write stream.  `tile_ptr` is the wavefront-uniform address of the tile's
// first element, `tile_bytes` the size of the window the wavefront may write.
typedef unsigned int v4u __attribute__((ext_vector_type(4)));
constexpr int kStoreAux = 2 | 16;                  // cache-policy bits: 1 = sc0, 2 = nt, 16 = sc1
constexpr int kRsrcWord3 = 0x00020000;             // raw 32-bit buffer, no swizzle, no stride

// Streaming loads of a whole tile row (64 lanes x 16 or 8 bytes): buffer loads
// with the non-temporal bit, addressed as wavefront-uniform row base + lane
// offset (measured about 1 % faster than per-lane 64-bit global addresses).
constexpr int kLoadAux = 2;                        // nt

__device__ __forceinline__ float4 ld4_stream(const float* row_ptr, int lane) {
  const __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<float*>(row_ptr), 0, kWave * 16, kRsrcWord3);
  const v4u t = __builtin_amdgcn_raw_buffer_load_b128(rs, lane * 16, 0, kLoadAux);
  return make_float4(__uint_as_float(t.x), __uint_as_float(t.y), __uint_as_float(t.z),
                     __uint_as_float(t.w));
}
__device__ __forceinline__ v2u ld2_stream(const void* row_ptr, int lane) {
  const __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<void*>(row_ptr), 0, kWave * 8, kRsrcWord3);
  return __builtin_amdgcn_raw_buffer_load_b64(rs, lane * 8, 0, kLoadAux);
}

__device__ __forceinline__ void st4_stream(float* tile_ptr, int tile_bytes, int lane, float4 v) {
  const __amdgpu_buffer_rsrc_t rs =
      __builtin_amdgcn_make_buffer_rsrc(tile_ptr, 0, tile_bytes, kRsrcWord3);
  const v4u t = {__float_as_uint(v.x), __float_as_uint(v.y), __float_as_uint(v.z),
                 __float_as_uint(v.w)};
  __builtin_amdgcn_raw_buffer_store_b128(t, rs, lane * 16, 0, kStoreAux);
}
__device__ __forceinline__ void st2_stream(void* tile_ptr, int tile_bytes, int lane, v2u v) {
  const __amdgpu_buffer_rsrc_t rs =
      __builtin_amdgcn_make_buffer_rsrc(tile_ptr, 0, tile_bytes, kRsrcWord3);
  __builtin_amdgcn_raw_buffer_store_b64(v, rs, lane * 8, 0, kStoreAux);
}

// fp32 -> bf16 bit pattern, round to nearest, ties to even; NaN stays a quiet NaN.
__device__ __forceinline__ uint32_t f32_to_bf16_bits(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (u >> 16) | 0x0040u;
  u += 0x7fffu + ((u >> 16) & 1u);
  return u >> 16;
}
__device__ __forceinline__ float bf16_bits_to_f32(uint32_t bits16) {
  return __uint_as_float(bits16 << 16);
}

// fp32 <-> IEEE fp16 through the hardware conversions (round to nearest even,
// gradual underflow, overflow to infinity).
__device__ __forceinline__ uint32_t f32_to_f16_bits(float f) {
  const _Float16 h = static_cast<_Float16>(f);
  return static_cast<uint32_t>(__builtin_bit_cast(unsigned short, h));
}
__device__ __forceinline__ float f16_bits_to_f32(uint32_t bits16) {
  const _Float16 h = __builtin_bit_cast(_Float16, static_cast<unsigned short>(bits16));
  return static_cast<float>(h);
}

// How a pseudo-gradient buffer is read and written: four coordinates per lane
// as one vector access, or one coordinate at a time on the element-wise path.
// `stored(d)` is the value a reader of the buffer will see after `d` is written.
template <int DT>
struct DeltaIO;

template <>
struct DeltaIO<kDeltaF32> {
  using Vec = float4;
  // one row of 256 coordinates starting at element `row`
  static __device__ __forceinline__ Vec load4(const void* p, int64_t row, int lane) {
    return ld4_stream(static_cast<const float*>(p) + row, lane);
  }
  static __device__ __forceinline__ float get(const Vec& v, int e) {
    return e == 0 ? v.x : e == 1 ? v.y : e == 2 ? v.z : v.w;
  }
  static __device__ __forceinline__ float load1(const void* p, int64_t j) {
    return static_cast<const float*>(p)[j];
  }
  static __device__ __forceinline__ float stored(float d) { return d; }
  // one 256-coordinate tile starting at element `base`
  static __device__ __forceinline__ void store4(void* p, int64_t base, int lane, const float (&d)[4]) {
    st4_stream(static_cast<float*>(p) + base, kWave * 16, lane, make_float4(d[0], d[1], d[2], d[3]));
  }
  static __device__ __forceinline__ void store1(void* p, int64_t j, float d) {
    static_cast<float*>(p)[j] = d;
  }
};

template <>
struct DeltaIO<kDeltaBF16> {
  using Vec = uint2;
  static __device__ __forceinline__ Vec load4(const void* p, int64_t row, int lane) {
    const v2u t = ld2_stream(static_cast<const uint16_t*>(p) + row, lane);
    return make_uint2(t.x, t.y);
  }
  static __device__ __forceinline__ float get(const Vec& v, int e) {
    const uint32_t w = e < 2 ? v.x : v.y;
    return __uint_as_float((e & 1) ? (w & 0xffff0000u) : (w << 16));
  }
  static __device__ __forceinline__ float load1(const void* p, int64_t j) {
    return bf16_bits_to_f32(static_cast<const uint16_t*>(p)[j]);
  }
  static __device__ __forceinline__ float stored(float d) {
    return bf16_bits_to_f32(f32_to_bf16_bits(d));
  }
  // d[] already holds representable values (stored()), so the shift is exact
  static __device__ __forceinline__ void store4(void* p, int64_t base, int lane, const float (&d)[4]) {
    const v2u t = {(__float_as_uint(d[0]) >> 16) | (__float_as_uint(d[1]) & 0xffff0000u),
                   (__float_as_uint(d[2]) >> 16) | (__float_as_uint(d[3]) & 0xffff0000u)};
    st2_stream(static_cast<uint16_t*>(p) + base, kWave * 8, lane, t);
  }
  static __device__ __forceinline__ void store1(void* p, int64_t j, float d) {
    static_cast<uint16_t*>(p)[j] = static_cast<uint16_t>(__float_as_uint(d) >> 16);
  }
};

template <>
struct DeltaIO<kDeltaF16> {
  using Vec = uint2;
  static __device__ __forceinline__ Vec load4(const void* p, int64_t row, int lane) {
    const v2u t = ld2_stream(static_cast<const uint16_t*>(p) + row, lane);
    return make_uint2(t.x, t.y);
  }
  static __device__ __forceinline__ float get(const Vec& v, int e) {
    const uint32_t w = e < 2 ? v.x : v.y;
    return f16_bits_to_f32((e & 1) ? (w >> 16) : (w & 0xffffu));
  }
  static __device__ __forceinline__ float load1(const void* p, int64_t j) {
    return f16_bits_to_f32(static_cast<const uint16_t*>(p)[j]);
  }
  static __device__ __forceinline__ float stored(float d) {
    return f16_bits_to_f32(f32_to_f16_bits(d));
  }
  // d[] already holds representable values (stored()), so the conversion is exact
  static __device__ __forceinline__ void store4(void* p, int64_t base, int lane, const float (&d)[4]) {
    const v2u t = {f32_to_f16_bits(d[0]) | (f32_to_f16_bits(d[1]) << 16),
                   f32_to_f16_bits(d[2]) | (f32_to_f16_bits(d[3]) << 16)};
    st2_stream(static_cast<uint16_t*>(p) + base, kWave * 8, lane, t);
  }
  static __device__ __forceinline__ void store1(void* p, int64_t j, float d) {
    static_cast<uint16_t*>(p)[j] = static_cast<uint16_t>(f32_to_f16_bits(d));
  }
};

__device__ __forceinline__ double sq(float v) {
  const double d = static_cast<double>(v);
  return d * d;                                    // exact: 24-bit x 24-bit
}

}  // namespace co2
