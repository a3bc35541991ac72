// Gate projection: logits[t,e] = sum_h hidden[t,h] * w_gate[e,h]  (the paper's
// "gate function", applied before Algorithm 1; Introduction / Method,
// "Integration with MoE Forward Pass"), followed in the same kernel by the
// per-token analysis, so the logits never travel through HBM unless asked for.
//
// bf16 path (gfx950): one workgroup of 4 wavefronts per tile of 64 tokens.  The
// contraction axis is cut into chunks of 64 values dealt round-robin to the 4
// waves, so at any moment a workgroup reads 512 contiguous bytes of every token
// row; each wave owns its chunks from load to MFMA and needs no barrier until the
// end.
//
// Memory -> registers: 16-byte loads with 8 consecutive lanes on one row, i.e. 8
// rows x 128 contiguous bytes per instruction.  The vector memory pipeline runs at
// full rate only when each group of 4 consecutive lanes reads 64 contiguous bytes;
// loading straight into MFMA layout (consecutive lanes on different rows) runs at a
// quarter of it, which for this kernel costs more than the HBM stream itself.
// Registers -> LDS -> registers: the wave parks the chunk in a private LDS strip
// (rows padded to 144 bytes) and reads it back in the layout of the 16x16x32 bf16
// MFMA (lane l: row/column l%16, contraction slots 8*(l/16)..+7); both operands use
// the same slot -> h mapping.  Two chunks are in flight in registers while a third
// is being multiplied.  Accumulation is fp32.  The 4 partial tiles meet in LDS and
// are added in the fixed order ((w0 + w1) + w2) + w3 (bit-reproducible logits).
#include "analyse.h"
#include "laser_internal.h"

namespace laser {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef const __attribute__((address_space(1))) u32x4* global_u4_ptr;
typedef __attribute__((address_space(3))) u32x4* lds_u4_ptr;

constexpr int kGateWaves = 4;
constexpr int kPartStride = 68;   // floats per token row of a partial tile (64 + 4 pad)
constexpr int kRowBytes = 144;    // staged row: 128 bytes of a chunk + 16 bytes pad
constexpr int kStripBytes = 2 * kTile * kRowBytes;  // per wave: hidden rows, then W rows
constexpr int kPartBytes = kGateWaves * kTile * kPartStride * 4;
constexpr int kGateLdsBytes =
    kPartBytes > kGateWaves * kStripBytes ? kPartBytes : kGateWaves * kStripBytes;

__device__ __forceinline__ u32x4 load_global_16(const uint16_t* p) {
  return *(global_u4_ptr)(p);
}

// G: global -> registers, one chunk (8 loads of hidden rows, 2*EB of W rows).
#define GATE_G(R, KOFF)                                                          \
  _Pragma("unroll") for (int q_ = 0; q_ < 8; ++q_)                               \
      R.h[q_] = load_global_16(hsrc[q_] + (KOFF));                               \
  _Pragma("unroll") for (int q_ = 0; q_ < 2 * EB; ++q_)                          \
      R.w[q_] = load_global_16(wsrc[q_] + (KOFF));                               \
  __builtin_amdgcn_sched_barrier(0);

// S: registers -> the wave's LDS strip.
#define GATE_S(R)                                                                \
  _Pragma("unroll") for (int q_ = 0; q_ < 8; ++q_)                               \
      *(lds_u4_ptr)(st_wr + q_ * 8 * kRowBytes) = R.h[q_];                       \
  _Pragma("unroll") for (int q_ = 0; q_ < 2 * EB; ++q_)                          \
      *(lds_u4_ptr)(st_wr + kTile * kRowBytes + q_ * 8 * kRowBytes) = R.w[q_];   \
  __builtin_amdgcn_sched_barrier(0);

// M: LDS strip -> MFMA operands -> accumulate, two k-steps of 32.
#define GATE_M()                                                                 \
  _Pragma("unroll") for (int s_ = 0; s_ < 2; ++s_) {                             \
    u32x4 b_[4], a_[EB];                                                         \
    _Pragma("unroll") for (int tb_ = 0; tb_ < 4; ++tb_)                          \
        b_[tb_] = *(lds_u4_ptr)(st_rd + tb_ * 16 * kRowBytes + s_ * 64);         \
    _Pragma("unroll") for (int eb_ = 0; eb_ < EB; ++eb_)                         \
        a_[eb_] = *(lds_u4_ptr)(st_rd + kTile * kRowBytes + eb_ * 16 * kRowBytes + s_ * 64); \
    _Pragma("unroll") for (int eb_ = 0; eb_ < EB; ++eb_)                         \
      _Pragma("unroll") for (int tb_ = 0; tb_ < 4; ++tb_)                        \
        acc[eb_][tb_] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(                 \
            __builtin_bit_cast(bf16x8, a_[eb_]), __builtin_bit_cast(bf16x8, b_[tb_]), \
            acc[eb_][tb_], 0, 0, 0);                                             \
  }                                                                              \
  __builtin_amdgcn_sched_barrier(0);

template <int EB>
struct GateRegs {
  u32x4 h[8];
  u32x4 w[2 * EB];
};

// EB: 16-expert blocks, 1 (E <= 16), 2 (E <= 32) or 4 (E <= 64).  NE: experts per
// lane of the per-token analysis that follows in the same kernel (padded E / 4).
template <int EB, int NE>
__global__ __launch_bounds__(256) void gate_analyse_bf16_kernel(
    const uint16_t* __restrict__ hidden, const uint16_t* __restrict__ w, int H, const RouteArgs a,
    const Workspace ws, int32_t* __restrict__ expert_ids, float* __restrict__ weights,
    float* __restrict__ logits_out) {
  extern __shared__ __align__(16) unsigned char gate_lds[];
  __shared__ unsigned long long mask64[64];
  __shared__ unsigned long long flex_lds;
  const int T = a.T, E = a.E;
  const int tile = blockIdx.x;
  const int wave = threadIdx.x >> 6;
  const int lane = threadIdx.x & 63;
  const int wave_u = __builtin_amdgcn_readfirstlane(wave);

  f32x4 acc[EB][4];
#pragma unroll
  for (int eb = 0; eb < EB; ++eb)
#pragma unroll
    for (int tb = 0; tb < 4; ++tb)
#pragma unroll
      for (int r = 0; r < 4; ++r) acc[eb][tb][r] = 0.0f;

  // Load side: lane l of load q takes piece l%8 (16 bytes) of row 8q + l/8.  Rows past
  // the end (tokens >= T, experts >= E) are clamped to the last valid row: their
  // products land in accumulator entries that are never used.
  const int lrow = lane >> 3, lpiece = lane & 7;
  const uint16_t* hsrc[8];
#pragma unroll
  for (int q = 0; q < 8; ++q)
    hsrc[q] = hidden + (size_t)min(tile * kTile + q * 8 + lrow, T - 1) * H + lpiece * 8;
  const uint16_t* wsrc[2 * EB];
#pragma unroll
  for (int q = 0; q < 2 * EB; ++q) wsrc[q] = w + (size_t)min(q * 8 + lrow, E - 1) * H + lpiece * 8;
  // LDS side: the strip of this wave; write position of (row l/8, piece l%8), read
  // position of (row l%16, slot group l/16).
  unsigned char* strip = gate_lds + wave_u * kStripBytes;
  unsigned char* st_wr = strip + lrow * kRowBytes + lpiece * 16;
  unsigned char* st_rd = strip + (lane & 15) * kRowBytes + (lane >> 4) * 16;

  const int nfull = H >> 6;
  const int nmine = (nfull - wave_u + kGateWaves - 1) / kGateWaves;  // chunks wave, wave+4, ...
  // Every tile starts its walk over the contraction axis at a different chunk, so
  // that the workgroups running at the same time do not all read the same column
  // range of their rows (which would land on the same memory channels).
  const int lim = nfull * 64;
  const int cstride = kGateWaves * 64;
  int koff = nfull > 0 ? ((tile * 5 + wave_u) % nfull) * 64 : 0;
  auto step = [&](int k) { k += cstride; return k >= lim ? k - lim : k; };  // nfull >= 4 when used

  // Software pipeline over this wave's chunks c0, c1, ...: while chunk i is
  // multiplied out of LDS, chunks i+1 and i+2 are in flight in ra / rb.
  GateRegs<EB> ra, rb;
  if (nmine > 0) {
    GATE_G(ra, koff)
    GATE_S(ra)                       // chunk 0 staged
    if (nmine > 1) { koff = step(koff); GATE_G(ra, koff) }   // chunk 1 in ra
    int i = 0;
    while (i + 3 < nmine) {          // straight-line body, two chunks per trip
      koff = step(koff);
      GATE_G(rb, koff)               // chunk i+2
      GATE_M()                       // chunk i
      GATE_S(ra)                     // chunk i+1 staged
      koff = step(koff);
      GATE_G(ra, koff)               // chunk i+3
      GATE_M()                       // chunk i+1
      GATE_S(rb)                     // chunk i+2 staged
      i += 2;
    }
    // here: chunk i staged, chunk i+1 (if any) in ra; at most 3 chunks left
    if (i + 2 < nmine) {
      koff = step(koff);
      GATE_G(rb, koff)               // chunk i+2, the last one
      GATE_M()
      GATE_S(ra)
      GATE_M()
      GATE_S(rb)
      GATE_M()
    } else if (i + 1 < nmine) {
      GATE_M()
      GATE_S(ra)
      GATE_M()
    } else {
      GATE_M()
    }
  }
  // Ragged tail of the contraction axis (H % 64 != 0), taken by one wave: pieces
  // past H are read from the start of the row instead and replaced by zeros.
  if ((H & 63) != 0 && wave_u == (nfull & 3)) {
    const u32x4 zero4 = {0u, 0u, 0u, 0u};
    const bool kin = nfull * 64 + lpiece * 8 < H;  // H % 8 == 0: a piece is all in or all out
    const int off = kin ? nfull * 64 : -lpiece * 8;
#pragma unroll
    for (int q = 0; q < 8; ++q) {
      const u32x4 v = load_global_16(hsrc[q] + off);
      ra.h[q] = kin ? v : zero4;
    }
#pragma unroll
    for (int q = 0; q < 2 * EB; ++q) {
      const u32x4 v = load_global_16(wsrc[q] + off);
      ra.w[q] = kin ? v : zero4;
    }
    GATE_S(ra)
    GATE_M()
  }
  __syncthreads();  // all strips are dead: the partial tiles reuse the space

  // Accumulator layout of the 16x16 MFMA: register r of lane l holds
  // row 4*(l/16) + r (expert) of column l%16 (token).
  float* part = reinterpret_cast<float*>(gate_lds);  // [4][64][kPartStride]
  float* mine = part + (size_t)wave * kTile * kPartStride;
  const int n = lane & 15, kgrp = lane >> 4;
#pragma unroll
  for (int eb = 0; eb < EB; ++eb)
#pragma unroll
    for (int tb = 0; tb < 4; ++tb) {
      float4 v = make_float4(acc[eb][tb][0], acc[eb][tb][1], acc[eb][tb][2], acc[eb][tb][3]);
      *reinterpret_cast<float4*>(mine + (tb * 16 + n) * kPartStride + eb * 16 + 4 * kgrp) = v;
    }
  __syncthreads();

  // The four partial tiles are summed on the fly by the analysis.
  analyse_tile<NE, kGateWaves>(part, kPartStride, mask64, &flex_lds, tile, a, ws, expert_ids,
                               weights, logits_out);
}

template <int EB, int NE>
static hipError_t launch_one(const void* hidden, const void* w, int H, const RouteArgs& a,
                             const Workspace& ws, int32_t* expert_ids, float* weights,
                             float* logits_out, hipStream_t s) {
  static bool attr_set = false;
  const void* fn = reinterpret_cast<const void*>(&gate_analyse_bf16_kernel<EB, NE>);
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, kGateLdsBytes);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  hipLaunchKernelGGL((gate_analyse_bf16_kernel<EB, NE>), dim3(a.ntiles), dim3(256), kGateLdsBytes, s,
                     static_cast<const uint16_t*>(hidden), static_cast<const uint16_t*>(w), H, a, ws,
                     expert_ids, weights, logits_out);
  return hipGetLastError();
}

hipError_t launch_gate_analyse_bf16(const void* hidden, const void* w, int H, const RouteArgs& a,
                                    const Workspace& ws, int32_t* expert_ids, float* weights,
                                    float* logits_out, hipStream_t s) {
  if (a.ntiles == 0) return hipSuccess;
  switch (a.EP) {
    case 8: return launch_one<1, 2>(hidden, w, H, a, ws, expert_ids, weights, logits_out, s);
    case 16: return launch_one<1, 4>(hidden, w, H, a, ws, expert_ids, weights, logits_out, s);
    case 32: return launch_one<2, 8>(hidden, w, H, a, ws, expert_ids, weights, logits_out, s);
    default: return launch_one<4, 16>(hidden, w, H, a, ws, expert_ids, weights, logits_out, s);
  }
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
