// Device-side fill of a synthetic KV cache: the same integer recipe as gen/cases.py
// (splitmix64 counters -> Irwin-Hall(12) normal -> one fp32 bias add -> optional bf16 / fp16 / E4M3 RNE),
// so the device cache holds exactly the bits the CPU regenerates row by row.
// Input generation only: nothing of the attention method is computed here.
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace {

__device__ __forceinline__ uint64_t mix64(uint64_t x) {
  x ^= x >> 30;
  x *= 0xBF58476D1CE4E5B9ull;
  x ^= x >> 27;
  x *= 0x94D049BB133111EBull;
  x ^= x >> 31;
  return x;
}

__device__ __forceinline__ float normal12(uint64_t key, uint64_t e) {
  const uint64_t PHI = 0x9E3779B97F4A7C15ull;
  uint64_t ha = mix64(key + (2 * e) * PHI), hb = mix64(key + (2 * e + 1) * PHI);
  int acc = 0;
#pragma unroll
  for (int i = 0; i < 6; ++i) {
    acc += (int)((ha >> (10 * i)) & 1023u);
    acc += (int)((hb >> (10 * i)) & 1023u);
  }
  return (float)(acc - 6138) * (1.0f / 1024.0f);
}

__device__ __forceinline__ uint16_t bf16_rne(float x) {
  uint32_t u = __float_as_uint(x);
  u += 0x7FFFu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}

// fp32 -> OCP FP8 E4M3, round to nearest even, saturating at 448: the recipe of f32_to_e4m3_bits in cases.py.
__device__ __forceinline__ uint32_t e4m3_rne(float x) {
  const uint32_t sign = (__float_as_uint(x) >> 24) & 0x80u;
  const float a = fabsf(x);
  uint32_t bits;
  if (a < 0.015625f) {                                  // below 2^-6: a multiple of 2^-9
    bits = (uint32_t)rintf(a * 512.0f);
  } else {
    uint32_t u = __float_as_uint(a);
    u += 0x7FFFFu + ((u >> 20) & 1u);
    const int e = (int)(u >> 23) - 127 + 7;
    const uint32_t m = (u >> 20) & 7u;
    bits = (e > 15 || (e == 15 && m == 7u)) ? 0x7Eu : (((uint32_t)e << 3) | m);
  }
  return bits | sign;
}

// One thread per 8 channels of one row.  grid.x covers rows*16, grid.y = B*Hkv.
__global__ __launch_bounds__(256) void k_fill(void* __restrict__ out, int format, int Hkv, int Lcap, int n_hot,
                                              const uint64_t* __restrict__ keys, const int32_t* __restrict__ row_end,
                                              const int32_t* __restrict__ recent_start,
                                              const int32_t* __restrict__ hot_pos, const float* __restrict__ bias) {
  const int bg = blockIdx.y, b = bg / Hkv;
  const int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x;
  const int row = (int)(t >> 4), c0 = (int)(t & 15) * 8;
  if (row >= Lcap) return;
  float x[8];
  if (row < row_end[b]) {
    const uint64_t key = keys[bg];
#pragma unroll
    for (int c = 0; c < 8; ++c) x[c] = normal12(key, (uint64_t)row * 128u + (uint64_t)(c0 + c));
    if (bias) {
      int cls = 0;
      for (int i = 0; i < n_hot; ++i) cls = (hot_pos[(int64_t)bg * n_hot + i] == row) ? 2 : cls;
      if (row >= recent_start[b]) cls = 3;
      if (row < 4) cls = 1;
      const float* bp = bias + ((int64_t)bg * 4 + cls) * 128 + c0;
#pragma unroll
      for (int c = 0; c < 8; ++c) x[c] = x[c] + bp[c];
    }
  } else {
#pragma unroll
    for (int c = 0; c < 8; ++c) x[c] = 0.f;
  }
  const int64_t o = ((int64_t)bg * Lcap + row) * 128 + c0;
  if (format == 2) {
    uint2 w;
    w.x = e4m3_rne(x[0]) | (e4m3_rne(x[1]) << 8) | (e4m3_rne(x[2]) << 16) | (e4m3_rne(x[3]) << 24);
    w.y = e4m3_rne(x[4]) | (e4m3_rne(x[5]) << 8) | (e4m3_rne(x[6]) << 16) | (e4m3_rne(x[7]) << 24);
    *reinterpret_cast<uint2*>((uint8_t*)out + o) = w;
  } else if (format == 3) {
    union {
      _Float16 h[8];
      uint4 w;
    } u;
#pragma unroll
    for (int c = 0; c < 8; ++c) u.h[c] = (_Float16)x[c];      // round to nearest even
    *reinterpret_cast<uint4*>((uint16_t*)out + o) = u.w;
  } else if (format == 1) {
    uint4 w;
    w.x = bf16_rne(x[0]) | ((uint32_t)bf16_rne(x[1]) << 16);
    w.y = bf16_rne(x[2]) | ((uint32_t)bf16_rne(x[3]) << 16);
    w.z = bf16_rne(x[4]) | ((uint32_t)bf16_rne(x[5]) << 16);
    w.w = bf16_rne(x[6]) | ((uint32_t)bf16_rne(x[7]) << 16);
    *reinterpret_cast<uint4*>((uint16_t*)out + o) = w;
  } else {
    float4* p = reinterpret_cast<float4*>((float*)out + o);
    p[0] = make_float4(x[0], x[1], x[2], x[3]);
    p[1] = make_float4(x[4], x[5], x[6], x[7]);
  }
}

}  // namespace

// All pointers are device pointers.  out is [B, Hkv, Lcap, 128] contiguous; format 0 = fp32, 1 = bf16,
// 2 = OCP FP8 E4M3, 3 = fp16.
// bias == NULL fills a value tensor (no structure).  Returns the hipError_t of the launch.
extern "C" __attribute__((visibility("default"))) int gen_fill_kv(
    void* out, int format, int B, int Hkv, int Lcap, int n_hot, const uint64_t* keys, const int32_t* row_end,
    const int32_t* recent_start, const int32_t* hot_pos, const float* bias, void* stream) {
  if (!out || !keys || !row_end || B < 1 || Hkv < 1 || Lcap < 1 || format < 0 || format > 3)
    return (int)hipErrorInvalidValue;
  if (bias && (!recent_start || (n_hot > 0 && !hot_pos))) return (int)hipErrorInvalidValue;
  dim3 grid((unsigned)(((int64_t)Lcap * 16 + 255) / 256), (unsigned)(B * Hkv));
  hipLaunchKernelGGL(k_fill, grid, dim3(256), 0, (hipStream_t)stream, out, format, Hkv, Lcap, n_hot, keys, row_end,
                     recent_start, hot_pos, bias);
  return (int)hipGetLastError();
}
