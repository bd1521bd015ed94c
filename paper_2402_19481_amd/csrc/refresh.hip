// Stale-buffer refresh (Section 4, Displaced patch parallelism): the patch's
// fresh rows replace its region of the full-shape buffer.  A pure HBM copy:
// 16 bytes per lane, four independent loads in flight per lane, grid-stride.
#include "kernels.h"

namespace df {

__global__ __launch_bounds__(256) void copy_rows_vec16(char* __restrict__ dst, const char* __restrict__ src,
                                                       long long row_vecs, long long dst_stride, long long src_stride) {
  const long long row = blockIdx.y;
  const u32x4* s = reinterpret_cast<const u32x4*>(src + row * src_stride);
  u32x4* d = reinterpret_cast<u32x4*>(dst + row * dst_stride);
  const long long step = (long long)gridDim.x * blockDim.x;
  long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  for (; i + 3 * step < row_vecs; i += 4 * step) {
    u32x4 a = __builtin_nontemporal_load(s + i);
    u32x4 b = __builtin_nontemporal_load(s + i + step);
    u32x4 c = __builtin_nontemporal_load(s + i + 2 * step);
    u32x4 e = __builtin_nontemporal_load(s + i + 3 * step);
    __builtin_nontemporal_store(a, d + i);
    __builtin_nontemporal_store(b, d + i + step);
    __builtin_nontemporal_store(c, d + i + 2 * step);
    __builtin_nontemporal_store(e, d + i + 3 * step);
  }
  for (; i < row_vecs; i += step) d[i] = s[i];
}

// many short rows: one lane per 16-byte vector of the flattened (row, vector) index space
__global__ __launch_bounds__(256) void copy_rows_flat16(char* __restrict__ dst, const char* __restrict__ src,
                                                        long long rows, int row_vecs, long long dst_stride,
                                                        long long src_stride) {
  const long long total = rows * row_vecs;
  const long long step = (long long)gridDim.x * blockDim.x;
  for (long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += step) {
    const long long r = i / row_vecs;
    const int v = (int)(i - r * row_vecs);
    const u32x4 t = *reinterpret_cast<const u32x4*>(src + r * src_stride + (long long)v * 16);
    *reinterpret_cast<u32x4*>(dst + r * dst_stride + (long long)v * 16) = t;
  }
}

__global__ __launch_bounds__(256) void copy_rows_bytes(char* __restrict__ dst, const char* __restrict__ src,
                                                       long long row_bytes, long long dst_stride, long long src_stride) {
  const long long row = blockIdx.y;
  const char* s = src + row * src_stride;
  char* d = dst + row * dst_stride;
  const long long step = (long long)gridDim.x * blockDim.x;
  for (long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x; i < row_bytes; i += step) d[i] = s[i];
}

// Copies `rows` rows of row_bytes each; row r goes from src + r*src_stride to dst + r*dst_stride.
int launch_copy_rows(void* dst, const void* src, long long rows, long long row_bytes, long long dst_stride,
                     long long src_stride, hipStream_t st) {
  if (rows <= 0 || row_bytes <= 0) return DF_OK;
  // contiguous rows collapse into one long row so the grid is sized by bytes, not by row count
  if (rows > 1 && dst_stride == row_bytes && src_stride == row_bytes) {
    row_bytes *= rows;
    rows = 1;
  }
  const bool vec = ((uintptr_t)dst % 16 == 0) && ((uintptr_t)src % 16 == 0) && (row_bytes % 16 == 0) &&
                   (dst_stride % 16 == 0) && (src_stride % 16 == 0);
  if (vec && rows > 8 && row_bytes <= (1 << 20)) {
    const long long total = rows * (row_bytes / 16);
    long long blocks = (total + 255) / 256;
    if (blocks > 4096) blocks = 4096;
    hipLaunchKernelGGL(copy_rows_flat16, dim3((unsigned)blocks), dim3(256), 0, st, (char*)dst, (const char*)src, rows,
                       (int)(row_bytes / 16), dst_stride, src_stride);
  } else if (vec) {
    if (rows > 65535) return DF_ESHAPE;
    long long v = row_bytes / 16;
    // 2048 blocks of 256 lanes cover the 256 compute units eight times over; each lane moves 64 B per trip
    long long blocks = (v + 256 * 4 - 1) / (256 * 4);
    long long cap = 2048 / (rows < 2048 ? rows : 2048);
    if (cap < 1) cap = 1;
    if (blocks > cap) blocks = cap;
    if (blocks < 1) blocks = 1;
    hipLaunchKernelGGL(copy_rows_vec16, dim3((unsigned)blocks, (unsigned)rows), dim3(256), 0, st, (char*)dst,
                       (const char*)src, v, dst_stride, src_stride);
  } else {
    if (rows > 65535) return DF_ESHAPE;
    long long blocks = (row_bytes + 255) / 256;
    if (blocks > 1024) blocks = 1024;
    hipLaunchKernelGGL(copy_rows_bytes, dim3((unsigned)blocks, (unsigned)rows), dim3(256), 0, st, (char*)dst,
                       (const char*)src, row_bytes, dst_stride, src_stride);
  }
  DF_LAUNCH_CHECK();
  return DF_OK;
}

}  // namespace df
