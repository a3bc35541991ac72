// What the bf16 gate kernels share: the tile geometry in LDS and the four steps a
// wavefront takes per chunk of the contraction axis (see gate.hip for the design).
#pragma once

#include "analyse.h"
#include "laser_internal.h"

namespace laser {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef const __attribute__((address_space(1))) u32x4* global_u4_ptr;
typedef __attribute__((address_space(3))) u32x4* lds_u4_ptr;

constexpr int kGateWaves = 8;
constexpr int kGateThreads = kGateWaves * 64;
constexpr int kPartStride = 72;   // floats per token row of a partial tile (64 + 8 pad)
constexpr int kRowBytes = 144;    // staged row: 128 bytes of a chunk + 16 bytes pad
constexpr int kStripBytes = 2 * kTile * kRowBytes;  // per wave: hidden rows, then W rows
constexpr int kPartBytes = kGateWaves * kTile * kPartStride * 4;
constexpr int kGateLdsBytes =
    kPartBytes > kGateWaves * kStripBytes ? kPartBytes : kGateWaves * kStripBytes;

__device__ __forceinline__ u32x4 load_global_16(const unsigned char* p) {
  return *(global_u4_ptr)(p);
}
__device__ __forceinline__ u32x4 load_global_16_stream(const unsigned char* p) {
  return __builtin_nontemporal_load((global_u4_ptr)(p));
}

// GH / GW: global -> registers, the hidden rows (8 loads) or the W rows (2*EB loads)
// of one chunk.  The scheduling barriers keep the compiler from sinking the loads
// down to their first use, which would undo the prefetch.
#define GATE_GH(RH, KBYTES)                                                      \
  _Pragma("unroll") for (int q_ = 0; q_ < 8; ++q_)                               \
      RH[q_] = load_global_16_stream(hbase + hoff[q_] + (KBYTES));                      \
  __builtin_amdgcn_sched_barrier(0);
#define GATE_GW(RW, KBYTES)                                                      \
  _Pragma("unroll") for (int q_ = 0; q_ < 2 * EB; ++q_)                          \
      RW[q_] = load_global_16(wbase + woff[q_] + (KBYTES));                      \
  __builtin_amdgcn_sched_barrier(0);

// S: registers -> the wave's LDS strip.
#define GATE_S(RH, RW)                                                           \
  _Pragma("unroll") for (int q_ = 0; q_ < 8; ++q_)                               \
      *(lds_u4_ptr)(st_wr + q_ * 8 * kRowBytes) = RH[q_];                        \
  _Pragma("unroll") for (int q_ = 0; q_ < 2 * EB; ++q_)                          \
      *(lds_u4_ptr)(st_wr + kTile * kRowBytes + q_ * 8 * kRowBytes) = RW[q_];    \
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
    __builtin_amdgcn_sched_barrier(0);                                           \
  }

// EB: 16-expert blocks, 1 (E <= 16), 2 (E <= 32) or 4 (E <= 64).  NE: experts per
// lane of the per-token analysis that follows in the same kernel (padded E / 8).
// NM: chunks per wave when H == 512 * NM (the main loop is then written out with
// deeper prefetch), 0 for any other H.  STATS: the analysis also writes the per-token
// statistics.  BATCH: blockIdx.y is the problem of a batched call (a kernel of its own:

}  // namespace laser
