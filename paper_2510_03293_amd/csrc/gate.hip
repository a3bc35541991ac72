// Gate projection: logits[t,e] = sum_h hidden[t,h] * w_gate[e,h]  (the paper's
// "gate function", applied before Algorithm 1; Introduction / Method,
// "Integration with MoE Forward Pass").
//
// bf16 path (gfx950): one workgroup of 4 wavefronts per tile of 64 tokens.  The
// contraction axis is cut into chunks of 64 values dealt round-robin to the 4
// waves, so at any moment a workgroup reads 512 contiguous bytes of every token
// row.  Operands go from memory straight into MFMA layout.  The 16x16x32 bf16 MFMA
// is used because of how its operands sit in the wave: lane l owns row (expert, A
// operand) or column (token, B operand) l%16 and the 8 contraction slots
// 8*(l/16)..+7, and both operands use the same slot -> h mapping.  One 16-byte
// load per lane then covers 16 rows x 64 contiguous bytes, which the memory
// pipeline handles as 16 half cache lines per instruction (the 32x32 shapes spread
// a load over 32 rows x 2 separate 16-byte pieces and run at a quarter of the
// rate).  Accumulation is fp32.  The 4 partial tiles meet in LDS and are added in
// the fixed order ((w0 + w1) + w2) + w3, which keeps the logits bit-reproducible.
#include "laser_internal.h"

namespace laser {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef const __attribute__((address_space(1))) u32x4* global_u4_ptr;

constexpr int kGateWaves = 4;
constexpr int kPartStride = 68;  // floats per token row of a partial tile (64 + 4 pad)
constexpr int kGateLdsBytes = kGateWaves * kTile * kPartStride * 4;

// 16-byte load from global memory (explicit address space: plain global_load, which
// only counts on vmcnt, so MFMAs can start while later loads are still in flight).
__device__ __forceinline__ u32x4 load_global_16(const uint16_t* p) {
  return *(global_u4_ptr)(p);
}

// Loads one 64-value chunk of the operands in MFMA layout: 2 k-steps x (EB expert
// blocks of W + 4 token blocks of hidden), 16 bytes per lane and piece.  Rows are
// clamped to valid ones by the caller, so every load is unconditional.  The
// scheduling barriers keep the compiler from sinking a chunk's loads down to their
// first use, which would undo the prefetch.
#define GATE_LOAD_CHUNK(A, B, KOFF)                                              \
  _Pragma("unroll") for (int s_ = 0; s_ < 2; ++s_) {                             \
    _Pragma("unroll") for (int tb_ = 0; tb_ < 4; ++tb_)                          \
        B[tb_][s_] = load_global_16(hrow[tb_] + (KOFF) + s_ * 32);               \
    _Pragma("unroll") for (int eb_ = 0; eb_ < EB; ++eb_)                         \
        A[eb_][s_] = load_global_16(wrow[eb_] + (KOFF) + s_ * 32);               \
  }                                                                              \
  __builtin_amdgcn_sched_barrier(0);

#define GATE_MFMA_CHUNK(A, B)                                                    \
  _Pragma("unroll") for (int s_ = 0; s_ < 2; ++s_)                               \
    _Pragma("unroll") for (int eb_ = 0; eb_ < EB; ++eb_)                         \
      _Pragma("unroll") for (int tb_ = 0; tb_ < 4; ++tb_)                        \
        acc[eb_][tb_] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(                 \
            __builtin_bit_cast(bf16x8, A[eb_][s_]), __builtin_bit_cast(bf16x8, B[tb_][s_]), \
            acc[eb_][tb_], 0, 0, 0);                                             \
  __builtin_amdgcn_sched_barrier(0);

template <int EB>  // 16-expert blocks: 1 (E <= 16), 2 (E <= 32) or 4 (E <= 64)
__global__ __launch_bounds__(256) void gate_bf16_kernel(const uint16_t* __restrict__ hidden,
                                                        const uint16_t* __restrict__ w,
                                                        int T, int H, int E,
                                                        float* __restrict__ logits) {
  extern __shared__ __align__(16) float part[];  // [4][64][kPartStride]
  const int tile = blockIdx.x;
  const int wave = threadIdx.x >> 6;
  const int lane = threadIdx.x & 63;
  const int n = lane & 15;       // row (expert) / column (token) inside a 16-block
  const int kgrp = lane >> 4;    // which 8-value group of a 32-value k-step

  f32x4 acc[EB][4];
#pragma unroll
  for (int eb = 0; eb < EB; ++eb)
#pragma unroll
    for (int tb = 0; tb < 4; ++tb)
#pragma unroll
      for (int r = 0; r < 4; ++r) acc[eb][tb][r] = 0.0f;

  // Rows past the end (tokens >= T, experts >= E) are clamped to the last valid
  // row: their products land in accumulator entries that are never written out.
  const uint16_t* hrow[4];
#pragma unroll
  for (int tb = 0; tb < 4; ++tb)
    hrow[tb] = hidden + (size_t)min(tile * kTile + tb * 16 + n, T - 1) * H + kgrp * 8;
  const uint16_t* wrow[EB];
#pragma unroll
  for (int eb = 0; eb < EB; ++eb) wrow[eb] = w + (size_t)min(eb * 16 + n, E - 1) * H + kgrp * 8;

  // Full chunks, two in flight per wave: the loads of chunk i+1 are issued before
  // the MFMAs of chunk i, so a workgroup keeps 64 KiB of operand reads outstanding.
  // The wave index is made wave-uniform so that the loop is plain scalar control
  // flow and the compiler's wait counts inside the body stay exact.
  const int nfull = H >> 6;
  const int wave_u = __builtin_amdgcn_readfirstlane(wave);
  const int nmine = (nfull - wave_u + kGateWaves - 1) / kGateWaves;  // chunks wave, wave+4, ...
  const int cstride = kGateWaves * 64;
  u32x4 a0[EB][2], b0[4][2], a1[EB][2], b1[4][2];
  int koff = wave_u * 64;  // element offset of the chunk held in (a0, b0)
  int i = 0;
  if (nmine > 0) { GATE_LOAD_CHUNK(a0, b0, koff) }
  while (i + 2 < nmine) {  // straight-line body: waits are exact
    GATE_LOAD_CHUNK(a1, b1, koff + cstride)
    GATE_MFMA_CHUNK(a0, b0)
    GATE_LOAD_CHUNK(a0, b0, koff + 2 * cstride)
    GATE_MFMA_CHUNK(a1, b1)
    koff += 2 * cstride;
    i += 2;
  }
  if (i + 1 < nmine) {
    GATE_LOAD_CHUNK(a1, b1, koff + cstride)
    GATE_MFMA_CHUNK(a0, b0)
    GATE_MFMA_CHUNK(a1, b1)
  } else if (i < nmine) {
    GATE_MFMA_CHUNK(a0, b0)
  }
  // Ragged tail of the contraction axis (H % 64 != 0), taken by one wave: pieces
  // past H are read from the start of the row instead and replaced by zeros.
  if ((H & 63) != 0 && wave_u == (nfull & 3)) {
    const u32x4 zero4 = {0u, 0u, 0u, 0u};
#pragma unroll
    for (int s = 0; s < 2; ++s) {
      const int kk = nfull * 64 + s * 32 + kgrp * 8;  // H % 8 == 0: a piece is all in or all out
      const bool kin = kk < H;
      const int off = kin ? nfull * 64 + s * 32 : -kgrp * 8;
#pragma unroll
      for (int tb = 0; tb < 4; ++tb) {
        const u32x4 v = load_global_16(hrow[tb] + off);
        b0[tb][s] = kin ? v : zero4;
      }
#pragma unroll
      for (int eb = 0; eb < EB; ++eb) {
        const u32x4 v = load_global_16(wrow[eb] + off);
        a0[eb][s] = kin ? v : zero4;
      }
    }
    GATE_MFMA_CHUNK(a0, b0)
  }

  // Accumulator layout of the 16x16 MFMA: register r of lane l holds
  // row 4*(l/16) + r (expert) of column l%16 (token).
  float* mine = part + (size_t)wave * kTile * kPartStride;
#pragma unroll
  for (int eb = 0; eb < EB; ++eb)
#pragma unroll
    for (int tb = 0; tb < 4; ++tb) {
      float4 v = make_float4(acc[eb][tb][0], acc[eb][tb][1], acc[eb][tb][2], acc[eb][tb][3]);
      *reinterpret_cast<float4*>(mine + (tb * 16 + n) * kPartStride + eb * 16 + 4 * kgrp) = v;
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
    hipError_t e4 = hipFuncSetAttribute(reinterpret_cast<const void*>(&gate_bf16_kernel<4>),
                                        hipFuncAttributeMaxDynamicSharedMemorySize, kGateLdsBytes);
    if (e1 != hipSuccess) return e1;
    if (e2 != hipSuccess) return e2;
    if (e4 != hipSuccess) return e4;
    attr_set = true;
  }
  const int ntiles = (T + kTile - 1) / kTile;
  if (ntiles == 0) return hipSuccess;
  const uint16_t* h16 = static_cast<const uint16_t*>(hidden);
  const uint16_t* w16 = static_cast<const uint16_t*>(w);
  if (E <= 16)
    hipLaunchKernelGGL(gate_bf16_kernel<1>, dim3(ntiles), dim3(256), kGateLdsBytes, s, h16, w16,
                       T, H, E, logits);
  else if (E <= 32)
    hipLaunchKernelGGL(gate_bf16_kernel<2>, dim3(ntiles), dim3(256), kGateLdsBytes, s, h16, w16,
                       T, H, E, logits);
  else
    hipLaunchKernelGGL(gate_bf16_kernel<4>, dim3(ntiles), dim3(256), kGateLdsBytes, s, h16, w16,
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
