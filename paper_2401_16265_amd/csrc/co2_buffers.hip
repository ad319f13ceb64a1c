// co2_buffer_set: device buffers for the flat vectors of the update, placed for
// the sweep (see include/co2_layout.h).  Host code only: HIP virtual-memory-management
// calls, no kernels.
//
// The sweep reads element e of every buffer at the same time.  With ordinary
// allocations the K + 4 buffers lie gigabytes apart and the sweep's duration
// depends on which physical pages the driver happened to hand out (measured:
// up to 10 % between otherwise identical allocations).  Here the physical
// memory is obtained in P pieces per buffer and in PIECE-MAJOR order -- piece 0
// of every buffer, then piece 1 of every buffer, ... -- and each buffer's
// pieces are mapped back to back into one contiguous virtual range, so the
// buffers stay ordinary flat vectors while the parts of them that are in flight
// together are neighbours in device memory.
#include <cstdint>
#include <cstdlib>
#include <new>
#include <vector>

#include "co2_layout.h"
#include "co2_launch.hpp"

struct co2_buffer_set {
  std::vector<hipMemGenericAllocationHandle_t> handles;   // created so far
  std::vector<char*> va;                                   // reserved range per buffer
  std::vector<size_t> va_bytes;
  std::vector<size_t> piece;                               // piece size of each buffer
  std::vector<size_t> mapped;                              // pieces mapped at the start of each range
};

namespace {

constexpr size_t kAlign = size_t(2) << 20;                 // piece sizes are multiples of 2 MiB
// Default piece size.  Measured with the 1.3B-parameter sweep (5.4 GB buffers, K = 8, 12 and 16): sets
// with 64 MiB pieces were fast every time, 32 MiB nearly as good, 128 MiB consistently 5 % slower and
// 256 MiB .. 2 GiB anything in between.
constexpr size_t kTargetPiece = size_t(64) << 20;
constexpr size_t kSkew = 4096;                             // buffer i starts i * kSkew into its range

inline size_t round_up(size_t b, size_t a) { return (b + a - 1) / a * a; }

int release(co2_buffer_set* s) {
  hipError_t first = hipSuccess;
  auto keep = [&](hipError_t e) { if (e != hipSuccess && first == hipSuccess) first = e; };
  for (size_t i = 0; i < s->va.size(); ++i) {
    if (!s->va[i]) continue;
    for (size_t j = 0; j < s->mapped[i]; ++j) keep(hipMemUnmap(s->va[i] + s->piece[i] * j, s->piece[i]));
    keep(hipMemAddressFree(s->va[i], s->va_bytes[i]));
  }
  for (auto h : s->handles) keep(hipMemRelease(h));
  delete s;
  if (first != hipSuccess) {
    (void)hipGetLastError();
    co2::note_hip_error(first);
    return CO2_EHIP;
  }
  return CO2_OK;
}

}  // namespace

extern "C" {

int co2_buffer_set_create(int32_t count, const size_t* bytes, size_t piece_bytes, void** bufs_out,
                          co2_buffer_set** set_out) {
  if (count < 1 || count > CO2_MAX_BUFFER_SET || !bytes || !bufs_out || !set_out) return CO2_EINVAL;
  size_t largest = 0;
  for (int32_t i = 0; i < count; ++i) {
    if (bytes[i] == 0) return CO2_EINVAL;
    if (bytes[i] > largest) largest = bytes[i];
  }
  if (piece_bytes == 0) piece_bytes = kTargetPiece;
  if (piece_bytes % kAlign != 0) return CO2_EINVAL;

  int device = 0;
  hipError_t e = hipGetDevice(&device);
  if (e != hipSuccess) { co2::note_hip_error(e); return CO2_EHIP; }
  hipMemAllocationProp prop{};
  prop.type = hipMemAllocationTypePinned;
  prop.location.type = hipMemLocationTypeDevice;
  prop.location.id = device;
  size_t gran = 0;
  e = hipMemGetAllocationGranularity(&gran, &prop, hipMemAllocationGranularityRecommended);
  if (e != hipSuccess) { (void)hipGetLastError(); co2::note_hip_error(e); return CO2_EHIP; }
  const size_t align = round_up(kAlign, gran ? gran : 1);

  // Every buffer is cut into the same number of pieces, so that piece j of each
  // covers the same element range whatever the element size.
  const size_t P = (largest + size_t(count) * kSkew + piece_bytes - 1) / piece_bytes;
  co2_buffer_set* s = new (std::nothrow) co2_buffer_set;
  if (!s) return CO2_EINVAL;
  try {
    s->va.assign(count, nullptr);
    s->va_bytes.assign(count, 0);
    s->piece.assign(count, 0);
    s->mapped.assign(count, 0);
    s->handles.reserve(static_cast<size_t>(count) * P);
  } catch (...) { delete s; return CO2_EINVAL; }

  auto fail = [&](hipError_t err) {
    (void)hipGetLastError();
    (void)release(s);
    co2::note_hip_error(err);
    return CO2_EHIP;
  };

  for (int32_t i = 0; i < count; ++i) {
    s->piece[i] = round_up((bytes[i] + size_t(i) * kSkew + P - 1) / P, align);
    s->va_bytes[i] = s->piece[i] * P;
    void* p = nullptr;
    e = hipMemAddressReserve(&p, s->va_bytes[i], align, nullptr, 0);
    if (e != hipSuccess) return fail(e);
    s->va[i] = static_cast<char*>(p);
  }
  hipMemAccessDesc acc{};
  acc.location = prop.location;
  acc.flags = hipMemAccessFlagsProtReadWrite;
  for (size_t j = 0; j < P; ++j) {
    for (int32_t i = 0; i < count; ++i) {
      hipMemGenericAllocationHandle_t h;
      e = hipMemCreate(&h, s->piece[i], &prop, 0);
      if (e != hipSuccess) return fail(e);
      s->handles.push_back(h);
      e = hipMemMap(s->va[i] + s->piece[i] * j, s->piece[i], 0, h, 0);
      if (e != hipSuccess) return fail(e);
      s->mapped[i] = j + 1;
    }
  }
  for (int32_t i = 0; i < count; ++i) {
    e = hipMemSetAccess(s->va[i], s->va_bytes[i], &acc, 1);
    if (e != hipSuccess) return fail(e);
  }
  for (int32_t i = 0; i < count; ++i) bufs_out[i] = s->va[i] + size_t(i) * kSkew;
  *set_out = s;
  return CO2_OK;
}

int co2_buffer_set_destroy(co2_buffer_set* set) {
  if (!set) return CO2_EINVAL;
  return release(set);
}

}  // extern "C"
