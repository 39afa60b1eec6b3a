// Measurement kernels (see include/pipad_ceilings.h): a streaming read and a row gather with the
// access shape of the aggregation kernel, to state what the memory system delivers for the two
// kinds of traffic the aggregation consists of.
#include "pipad_ceilings.h"
#include "pipad_internal.h"

#ifndef PIPAD_STREAM_BLOCKS
#define PIPAD_STREAM_BLOCKS 2048  // workgroups of the streaming kernels: eight per CU
#endif

namespace pipad {
namespace {

constexpr int kGatherPerBlock = 4096;      // index entries per workgroup (1024 per wave)
constexpr size_t kSinkFloats = (size_t)1 << 22;

__global__ __launch_bounds__(kBlock) void k_stream_read(const float4 *src, size_t n16, float *sink) {
  float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
  const size_t stride = (size_t)gridDim.x * kBlock;
  size_t i = (size_t)blockIdx.x * kBlock + threadIdx.x;
  // four independent loads in flight per lane
  for (; i + 3 * stride < n16; i += 4 * stride) {
    const float4 a = src[i], b = src[i + stride], c = src[i + 2 * stride], d = src[i + 3 * stride];
    acc.x += a.x + b.x + c.x + d.x;
    acc.y += a.y + b.y + c.y + d.y;
    acc.z += a.z + b.z + c.z + d.z;
    acc.w += a.w + b.w + c.w + d.w;
  }
  for (; i < n16; i += stride) {
    const float4 a = src[i];
    acc.x += a.x; acc.y += a.y; acc.z += a.z; acc.w += a.w;
  }
  float s = acc.x + acc.y + acc.z + acc.w;
  for (int m = kWave >> 1; m >= 1; m >>= 1) s += __shfl_xor(s, m, kWave);
  if (threadIdx.x % kWave == 0) sink[(size_t)(blockIdx.x * kWavesPerBlock + threadIdx.x / kWave) % kSinkFloats] = s;
}

// Plain copy, 16 bytes per lane, four loads in flight: its memory traffic is known exactly (bytes
// read = bytes written = the argument), which is what hardware traffic counters are scaled by.
__global__ __launch_bounds__(kBlock) void k_stream_copy(const float4 *src, float4 *dst, size_t n16) {
  const size_t stride = (size_t)gridDim.x * kBlock;
  size_t i = (size_t)blockIdx.x * kBlock + threadIdx.x;
  for (; i + 3 * stride < n16; i += 4 * stride) {
    const float4 a = src[i], b = src[i + stride], c = src[i + 2 * stride], d = src[i + 3 * stride];
    dst[i] = a;
    dst[i + stride] = b;
    dst[i + 2 * stride] = c;
    dst[i + 3 * stride] = d;
  }
  for (; i < n16; i += stride) dst[i] = src[i];
}

// A wave owns 1024 consecutive index entries; its 64 / LS lane teams take entries team, team +
// nteams, ... of every 64-entry chunk, four gathers in flight per lane, exactly like the wave-wide
// walk of the aggregation kernel (indices staged through LDS as 32-bit byte offsets).
template <int LS_LOG2>
__global__ __launch_bounds__(kBlock) void k_gather(const float *table, uint32_t rows,
                                                    uint32_t row_bytes, const int32_t *index,
                                                    int64_t count, int32_t classes, float *sink) {
  __shared__ uint32_t off[kWavesPerBlock][kWave];
  constexpr int LS = 1 << LS_LOG2, NT = kWave >> LS_LOG2;
  const int lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;
  const int fl = lane & (LS - 1), team = lane >> LS_LOG2;
  int64_t chunk = blockIdx.x;
  if (classes > 1) {
    const int64_t per_class = count / classes / kGatherPerBlock;
    chunk = (int64_t)(blockIdx.x % classes) * per_class + blockIdx.x / classes;
  }
  const int64_t first = chunk * kGatherPerBlock + (int64_t)wave * (kGatherPerBlock / kWavesPerBlock);
  const char *base = reinterpret_cast<const char *>(table) + fl * 16;
  float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
  int32_t next = index[first + lane];
  for (int c = 0; c < kGatherPerBlock / kWavesPerBlock / kWave; ++c) {
    off[wave][lane] = min((uint32_t)next, rows - 1u) * row_bytes;  // never past the table
    if (c + 1 < kGatherPerBlock / kWavesPerBlock / kWave) next = index[first + (c + 1) * kWave + lane];
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    for (int e0 = 0; e0 < kWave; e0 += NT * 4) {
      uint32_t o[4];
      float4 x[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) o[u] = off[wave][e0 + u * NT + team];
#pragma unroll
      for (int u = 0; u < 4; ++u) x[u] = *reinterpret_cast<const float4 *>(base + o[u]);
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        acc.x += x[u].x; acc.y += x[u].y; acc.z += x[u].z; acc.w += x[u].w;
      }
    }
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
  }
  if (fl == 0 && team == 0)
    sink[(size_t)(blockIdx.x * kWavesPerBlock + wave) % kSinkFloats] = acc.x + acc.y + acc.z + acc.w;
}

}  // namespace
}  // namespace pipad

extern "C" {

size_t pipad_ceiling_sink_floats(void) { return pipad::kSinkFloats; }

int pipad_ceiling_stream_read(const float *src, size_t bytes, float *sink, void *stream) {
  if (!src || !sink || bytes % 16 != 0 || (reinterpret_cast<uintptr_t>(src) & 15u))
    return PIPAD_ERR_INVALID_ARG;
  if (bytes == 0) return PIPAD_OK;
  const size_t n16 = bytes / 16;
  const unsigned blocks =
      (unsigned)std::min<size_t>(PIPAD_STREAM_BLOCKS, (n16 + pipad::kBlock - 1) / pipad::kBlock);
  hipLaunchKernelGGL(pipad::k_stream_read, dim3(blocks), dim3(pipad::kBlock), 0,
                     static_cast<hipStream_t>(stream), reinterpret_cast<const float4 *>(src), n16, sink);
  PIPAD_HIP(hipGetLastError());
  return PIPAD_OK;
}

int pipad_ceiling_stream_copy(const float *src, float *dst, size_t bytes, void *stream) {
  const uintptr_t a = reinterpret_cast<uintptr_t>(src), b = reinterpret_cast<uintptr_t>(dst);
  if (!src || !dst || bytes % 16 != 0 || ((a | b) & 15u)) return PIPAD_ERR_INVALID_ARG;
  if (a < b + bytes && b < a + bytes) return PIPAD_ERR_INVALID_ARG;  // overlapping
  if (bytes == 0) return PIPAD_OK;
  const size_t n16 = bytes / 16;
  const unsigned blocks =
      (unsigned)std::min<size_t>(PIPAD_STREAM_BLOCKS, (n16 + pipad::kBlock - 1) / pipad::kBlock);
  hipLaunchKernelGGL(pipad::k_stream_copy, dim3(blocks), dim3(pipad::kBlock), 0,
                     static_cast<hipStream_t>(stream), reinterpret_cast<const float4 *>(src),
                     reinterpret_cast<float4 *>(dst), n16);
  PIPAD_HIP(hipGetLastError());
  return PIPAD_OK;
}

int pipad_ceiling_gather(const float *table, int64_t rows, int32_t row_floats, int64_t stride_floats,
                         const int32_t *index, int64_t count, int32_t xcd_classes, float *sink,
                         void *stream) {
  if (!table || !index || !sink || rows < 1 || count < 0 || stride_floats < row_floats ||
      stride_floats % 4 != 0 || (reinterpret_cast<uintptr_t>(table) & 15u))
    return PIPAD_ERR_INVALID_ARG;
  if (row_floats != 16 && row_floats != 32 && row_floats != 64) return PIPAD_ERR_INVALID_ARG;
  if (xcd_classes != 0 && xcd_classes != pipad::kClasses) return PIPAD_ERR_INVALID_ARG;
  const int64_t unit = (int64_t)pipad::kGatherPerBlock * (xcd_classes ? xcd_classes : 1);
  if (count % unit != 0) return PIPAD_ERR_INVALID_ARG;
  if (rows * stride_floats * 4 >= ((int64_t)1 << 32)) return PIPAD_ERR_TOO_LARGE;
  const int64_t blocks = count / pipad::kGatherPerBlock;
  if (blocks >= ((int64_t)1 << 31)) return PIPAD_ERR_TOO_LARGE;
  if (blocks == 0) return PIPAD_OK;
  const uint32_t row_bytes = (uint32_t)stride_floats * 4u;
  hipStream_t st = static_cast<hipStream_t>(stream);
  const dim3 grid((unsigned)blocks), block(pipad::kBlock);
  if (row_floats == 64)
    hipLaunchKernelGGL(pipad::k_gather<4>, grid, block, 0, st, table, (uint32_t)rows, row_bytes, index, count, xcd_classes, sink);
  else if (row_floats == 32)
    hipLaunchKernelGGL(pipad::k_gather<3>, grid, block, 0, st, table, (uint32_t)rows, row_bytes, index, count, xcd_classes, sink);
  else
    hipLaunchKernelGGL(pipad::k_gather<2>, grid, block, 0, st, table, (uint32_t)rows, row_bytes, index, count, xcd_classes, sink);
  PIPAD_HIP(hipGetLastError());
  return PIPAD_OK;
}

}  // extern "C"
