// Error strings, version, and the device-side weight copies of a re-plan (Sec. 4.3 / 5: the
// state transfers that move expert replicas to their new slots).
#include "lz_common.h"

extern "C" const char* lz_strerror(int32_t code) {
  switch (code) {
    case LZ_OK: return "ok";
    case LZ_EINVAL: return "invalid argument";
    case LZ_ESHAPE: return "shape outside the supported limits";
    case LZ_EWORKSPACE: return "workspace missing, misaligned or too small";
    case LZ_EUNRECOVERABLE: return "an expert has no replica on any surviving rank";
    case LZ_EINFEASIBLE: return "fewer replica slots than experts";
    case LZ_EHIP: return "HIP runtime error";
    default: return "unknown error";
  }
}

extern "C" int32_t lz_version(void) { return 100; }

extern "C" int32_t lz_apply_transfers(const lz_transfer* xfers, int32_t n, const void* w1_old,
                                      const void* w2_old, int32_t S_old, void* w1_new, void* w2_new,
                                      int32_t S_new, const lz_shape* shape, void* stream) {
  if (!lz::shape_ok(shape)) return LZ_ESHAPE;
  if (n < 0 || S_old < 1 || S_new < 1) return LZ_EINVAL;
  if (n == 0) return LZ_OK;
  if (!xfers || !w1_old || !w2_old || !w1_new || !w2_new) return LZ_EINVAL;
  const size_t eb = lz::elem_bytes(shape->dtype);
  const size_t w1_bytes = (size_t)shape->ffn * (shape->act == LZ_SWIGLU ? 2 : 1) * shape->d * eb;
  const size_t w2_bytes = (size_t)shape->d * shape->ffn * eb;
  for (int i = 0; i < n; ++i)
    if (xfers[i].dst_slot < 0 || xfers[i].dst_slot >= S_new || xfers[i].src_slot < 0 ||
        xfers[i].src_slot >= S_old)
      return LZ_EINVAL;
  hipStream_t st = (hipStream_t)stream;
  for (int i = 0; i < n; ++i) {
    const size_t d = (size_t)xfers[i].dst_slot, s = (size_t)xfers[i].src_slot;
    if (hipMemcpyAsync((char*)w1_new + d * w1_bytes, (const char*)w1_old + s * w1_bytes, w1_bytes,
                       hipMemcpyDeviceToDevice, st) != hipSuccess)
      return LZ_EHIP;
    if (hipMemcpyAsync((char*)w2_new + d * w2_bytes, (const char*)w2_old + s * w2_bytes, w2_bytes,
                       hipMemcpyDeviceToDevice, st) != hipSuccess)
      return LZ_EHIP;
  }
  return LZ_OK;
}
