// Small host-side helpers that linfusion.hip shares with the library's other translation units.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace lfh {

// LINFUSION_OK when the current device is a gfx950, else LINFUSION_ERR_DEVICE (cached per device)
int check_device();
// `dflt`, unless tuning is switched on (LINFUSION_TUNE=1 at first use, or linfusion_set_tuning) and the
// environment holds a positive integer under `name`
int env_int(const char* name, int dflt);
// compute units of the current device (256 while no device is visible)
int num_cu();

// Element strides {batch, head, token} of a [B, H, N, d] view with contiguous channels (null = dense).
// check_strides: LINFUSION_OK when the kernels can address the view (non-negative, token rows 16-byte aligned,
// index widths); `written` additionally requires that no two rows share memory.  span_bytes: bytes from the
// first to one past the last element the view touches.
int check_strides(const long long s[3], int B, int H, long long N, int d, size_t esz, bool written);
size_t span_bytes(const long long s[3], int B, int H, long long N, int d, size_t esz);

// true when the byte ranges [a, a + na) and [b, b + nb) share a byte
inline bool overlaps(const void* a, size_t na, const void* b, size_t nb) {
  const uintptr_t x = (uintptr_t)a, y = (uintptr_t)b;
  return x < y + nb && y < x + na;
}

// Workgroups may use up to 160 KiB of LDS on this device; above 64 KiB the kernel has to be told (per kernel; cheap).
template <typename KernelT>
inline bool allow_lds(KernelT kernel, int bytes) {
  if (bytes <= 65536) return true;
  if (hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize, bytes) !=
      hipSuccess) {
    (void)hipGetLastError();
    return false;
  }
  return true;
}

}  // namespace lfh
