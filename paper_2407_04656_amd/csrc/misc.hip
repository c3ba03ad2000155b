// Error strings, version, the one-time conversion of expert weights into the library's
// input-major layout, and the device-side weight copies of a re-plan (Sec. 4.3 / 5: the state
// transfers that move expert replicas to their new slots).
#include "lz_common.h"

namespace {

// dst[s][c][r] = src[s][r][c]: 32 x 32 tiles through LDS, both sides coalesced, any sizes
template <typename Elem>
__global__ __launch_bounds__(256) void transpose_kernel(const Elem* __restrict__ src, int rows, int cols,
                                                        Elem* __restrict__ dst) {
  __shared__ Elem tile[32][33];
  const size_t base = (size_t)blockIdx.z * rows * cols;
  const int r0 = blockIdx.y * 32, c0 = blockIdx.x * 32;
  const int tx = threadIdx.x % 32, ty = threadIdx.x / 32;  // 32 x 8 threads
  for (int i = ty; i < 32; i += 8)
    if (r0 + i < rows && c0 + tx < cols) tile[i][tx] = src[base + (size_t)(r0 + i) * cols + c0 + tx];
  __syncthreads();
  for (int i = ty; i < 32; i += 8)
    if (c0 + i < cols && r0 + tx < rows) dst[base + (size_t)(c0 + i) * rows + r0 + tx] = tile[tx][i];
}

}  // namespace

extern "C" int32_t lz_pack_weights(const void* w, int32_t S, int32_t rows, int32_t cols, int32_t dtype,
                                   void* packed, void* stream) {
  if (S < 0 || rows < 1 || cols < 1 || (dtype != LZ_F32 && dtype != LZ_BF16)) return LZ_ESHAPE;
  if (S > 65535 || (rows + 31) / 32 > 65535) return LZ_ESHAPE;
  if (S == 0) return LZ_OK;
  if (!w || !packed || w == packed) return LZ_EINVAL;
  const dim3 grid((cols + 31) / 32, (rows + 31) / 32, S);
  if (dtype == LZ_F32)
    hipLaunchKernelGGL(transpose_kernel<float>, grid, dim3(256), 0, (hipStream_t)stream, (const float*)w, rows, cols,
                       (float*)packed);
  else
    hipLaunchKernelGGL(transpose_kernel<uint16_t>, grid, dim3(256), 0, (hipStream_t)stream, (const uint16_t*)w,
                       rows, cols, (uint16_t*)packed);
  return lz::launch_status();
}

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
