// Gate projection: logits[t,e] = sum_h hidden[t,h] * w_gate[e,h]  (the paper's
// "gate function", applied before Algorithm 1; Introduction / Method,
// "Integration with MoE Forward Pass").
//
// bf16 path (gfx950): one workgroup of 4 wavefronts per tile of 64 tokens.  The
// contraction axis is cut into chunks of 64 values dealt round-robin to the 4
// waves, so at any moment a workgroup reads 512 contiguous bytes of every token
// row.  Operands go from memory straight into MFMA layout: in the
// 32x32x16 bf16 MFMA a lane owns one row (expert, A operand) or column (token, B
// operand) and 8 consecutive contraction slots, and both operands use the same
// slot -> h mapping, so each lane simply reads 4 x 16 bytes (64 contiguous bytes)
// of its row per chunk.  Accumulation is fp32.  The 4 partial tiles meet in LDS
// and are added in the fixed order ((w0 + w1) + w2) + w3, which keeps the logits
// bit-reproducible from run to run.
#include "laser_internal.h"

namespace laser {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;

constexpr int kGateWaves = 4;
constexpr int kPartStride = 68;  // floats per token row of a partial tile (64 + 4 pad)
constexpr int kGateLdsBytes = kGateWaves * kTile * kPartStride * 4;

template <int EB>  // 32-expert blocks: 1 (E <= 32) or 2 (E <= 64)
__global__ __launch_bounds__(256) void gate_bf16_kernel(const uint16_t* __restrict__ hidden,
                                                        const uint16_t* __restrict__ w,
                                                        int T, int H, int E,
                                                        float* __restrict__ logits) {
  extern __shared__ __align__(16) float part[];  // [4][64][kPartStride]
  const int tile = blockIdx.x;
  const int wave = threadIdx.x >> 6;
  const int lane = threadIdx.x & 63;
  const int n = lane & 31;      // row (expert) / column (token) inside a 32-block
  const int half = lane >> 5;   // which 32-value half of the 64-value chunk

  f32x16 acc[EB][2];
#pragma unroll
  for (int eb = 0; eb < EB; ++eb)
#pragma unroll
    for (int tb = 0; tb < 2; ++tb)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[eb][tb][r] = 0.0f;

  const uint16_t* hrow[2];
  bool hlive[2];
#pragma unroll
  for (int tb = 0; tb < 2; ++tb) {
    const int tok = tile * kTile + tb * 32 + n;
    hlive[tb] = tok < T;
    hrow[tb] = hidden + (size_t)(hlive[tb] ? tok : 0) * H;
  }
  const uint16_t* wrow[EB];
  bool wlive[EB];
#pragma unroll
  for (int eb = 0; eb < EB; ++eb) {
    const int ex = eb * 32 + n;
    wlive[eb] = ex < E;
    wrow[eb] = w + (size_t)(wlive[eb] ? ex : 0) * H;
  }

  const int nchunks = (H + 63) >> 6;
  const uint4 zero4 = make_uint4(0, 0, 0, 0);
  for (int ch = wave; ch < nchunks; ch += kGateWaves) {
    const int kbase = ch * 64 + half * 32;
    uint4 b[2][4], a[EB][4];
#pragma unroll
    for (int s = 0; s < 4; ++s) {
      const int kk = kbase + s * 8;
      const bool kin = kk < H;  // H % 8 == 0: a 16-byte piece is wholly inside or outside
#pragma unroll
      for (int tb = 0; tb < 2; ++tb)
        b[tb][s] = (kin && hlive[tb]) ? *reinterpret_cast<const uint4*>(hrow[tb] + kk) : zero4;
#pragma unroll
      for (int eb = 0; eb < EB; ++eb)
        a[eb][s] = (kin && wlive[eb]) ? *reinterpret_cast<const uint4*>(wrow[eb] + kk) : zero4;
    }
#pragma unroll
    for (int s = 0; s < 4; ++s)
#pragma unroll
      for (int eb = 0; eb < EB; ++eb)
#pragma unroll
        for (int tb = 0; tb < 2; ++tb)
          acc[eb][tb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
              __builtin_bit_cast(bf16x8, a[eb][s]), __builtin_bit_cast(bf16x8, b[tb][s]),
              acc[eb][tb], 0, 0, 0);
  }

  // Accumulator layout of the 32x32 MFMA: register r of lane l holds
  // row 8*(r/4) + 4*(l/32) + r%4 (expert) of column l%32 (token).
  float* mine = part + (size_t)wave * kTile * kPartStride;
#pragma unroll
  for (int eb = 0; eb < EB; ++eb)
#pragma unroll
    for (int tb = 0; tb < 2; ++tb)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        float4 v = make_float4(acc[eb][tb][4 * g], acc[eb][tb][4 * g + 1],
                               acc[eb][tb][4 * g + 2], acc[eb][tb][4 * g + 3]);
        *reinterpret_cast<float4*>(mine + (tb * 32 + n) * kPartStride + eb * 32 + 8 * g +
                                   4 * half) = v;
      }
  __syncthreads();

  const int total = kTile * E;
  for (int idx = threadIdx.x; idx < total; idx += 256) {
    const int tok = idx / E;
    const int e = idx - tok * E;
    const int o = tok * kPartStride + e;
    float v = part[o] + part[kTile * kPartStride + o];
    v = v + part[2 * kTile * kPartStride + o];
    v = v + part[3 * kTile * kPartStride + o];
    const int t = tile * kTile + tok;
    if (t < T) logits[(size_t)t * E + e] = v;
  }
}

hipError_t launch_gate_bf16(const void* hidden, const void* w, int T, int H, int E,
                            float* logits, hipStream_t s) {
  static bool attr_set = false;
  if (!attr_set) {
    hipError_t e1 = hipFuncSetAttribute(reinterpret_cast<const void*>(&gate_bf16_kernel<1>),
                                        hipFuncAttributeMaxDynamicSharedMemorySize, kGateLdsBytes);
    hipError_t e2 = hipFuncSetAttribute(reinterpret_cast<const void*>(&gate_bf16_kernel<2>),
                                        hipFuncAttributeMaxDynamicSharedMemorySize, kGateLdsBytes);
    if (e1 != hipSuccess) return e1;
    if (e2 != hipSuccess) return e2;
    attr_set = true;
  }
  const int ntiles = (T + kTile - 1) / kTile;
  if (ntiles == 0) return hipSuccess;
  const uint16_t* h16 = static_cast<const uint16_t*>(hidden);
  const uint16_t* w16 = static_cast<const uint16_t*>(w);
  if (E <= 32)
    hipLaunchKernelGGL(gate_bf16_kernel<1>, dim3(ntiles), dim3(256), kGateLdsBytes, s, h16, w16,
                       T, H, E, logits);
  else
    hipLaunchKernelGGL(gate_bf16_kernel<2>, dim3(ntiles), dim3(256), kGateLdsBytes, s, h16, w16,
                       T, H, E, logits);
  return hipGetLastError();
}

// fp32 path: one thread per (token, expert) dot product, float4 loads, fused
// multiply-add accumulation in h order.  Meant for small fp32 problems.
__global__ __launch_bounds__(256) void gate_f32_kernel(const float* __restrict__ hidden,
                                                       const float* __restrict__ w, int T, int H,
                                                       int E, float* __restrict__ logits) {
  const long long idx = (long long)blockIdx.x * 256 + threadIdx.x;
  if (idx >= (long long)T * E) return;
  const int t = (int)(idx / E);
  const int e = (int)(idx - (long long)t * E);
  const float4* h4 = reinterpret_cast<const float4*>(hidden + (size_t)t * H);
  const float4* w4 = reinterpret_cast<const float4*>(w + (size_t)e * H);
  float acc = 0.0f;
  for (int i = 0; i < (H >> 2); ++i) {
    const float4 x = h4[i], y = w4[i];
    acc = __builtin_fmaf(x.x, y.x, acc);
    acc = __builtin_fmaf(x.y, y.y, acc);
    acc = __builtin_fmaf(x.z, y.z, acc);
    acc = __builtin_fmaf(x.w, y.w, acc);
  }
  logits[idx] = acc;
}

hipError_t launch_gate_f32(const float* hidden, const float* w, int T, int H, int E,
                           float* logits, hipStream_t s) {
  const long long total = (long long)T * E;
  if (total == 0) return hipSuccess;
  const unsigned blocks = (unsigned)((total + 255) / 256);
  hipLaunchKernelGGL(gate_f32_kernel, dim3(blocks), dim3(256), 0, s, hidden, w, T, H, E, logits);
  return hipGetLastError();
}

}  // namespace laser
