// Gate projection: logits[t,e] = sum_h hidden[t,h] * w_gate[e,h]  (the paper's
// "gate function", applied before Algorithm 1; Introduction / Method,
// "Integration with MoE Forward Pass"), followed in the same kernel by the
// per-token analysis, so the logits never travel through HBM unless asked for.
//
// bf16 path (gfx950): one workgroup of 8 wavefronts per tile of 64 tokens.  The
// contraction axis is cut into chunks of 64 values dealt round-robin to the 8
// waves; each wave owns its chunks from load to MFMA and needs no barrier until the
// end.  Eight waves (two per SIMD, at most 256 registers each) rather than four
// with deeper per-wave prefetch, because a lone wavefront issues a vector
// instruction only every ~8 cycles on this part: the analysis that follows runs
// twice as fast with a second wave to fill the gaps.  Each wave keeps two 16 KiB
// chunks in flight (256 KiB per CU).
//
// Memory -> registers: 16-byte loads with 8 consecutive lanes on one row, i.e. 8
// rows x 128 contiguous bytes per instruction.  The vector memory pipeline runs at
// full rate only when each group of 4 consecutive lanes reads 64 contiguous bytes;
// loading straight into MFMA layout (consecutive lanes on different rows) runs at a
// quarter of it, which for this kernel costs more than the HBM stream itself.
// Registers -> LDS -> registers: the wave parks the chunk in a private LDS strip
// (rows padded to 144 bytes) and reads it back in the layout of the 16x16x32 bf16
// MFMA (lane l: row/column l%16, contraction slots 8*(l/16)..+7); both operands use
// the same slot -> h mapping.  While chunk i is multiplied out of LDS, chunks i+1 and
// i+2 are in flight in registers.  Accumulation is fp32.  The 8 partial tiles meet in LDS
// and are added in a fixed order (bit-reproducible logits).
#include "gate_tile.h"

namespace laser {

// the longer prologue would delay the first loads of the single-problem kernel).
template <int EB, int NE, int NM, bool STATS, bool BATCH>
__global__ __launch_bounds__(kGateThreads) void gate_analyse_bf16_kernel(
    const uint16_t* __restrict__ hidden, const uint16_t* __restrict__ w, int H, const RouteArgs a0,
    const Workspace ws0, int32_t* __restrict__ expert_ids, float* __restrict__ weights,
    float* __restrict__ logits_out, size_t logits_stride) {
  extern __shared__ __align__(16) unsigned char gate_lds[];
  __shared__ unsigned long long mask64[64];
  __shared__ unsigned long long flex_lds;
  const int prob = BATCH ? blockIdx.y : 0;
  RouteArgs a = BATCH ? problem_args(a0, prob) : a0;
  const Workspace ws = BATCH ? problem_workspace(ws0, (size_t)prob * a0.ws_stride) : ws0;
  if (STATS && a.pool_in_ws) a.st_pool = ws.pool;
  if (BATCH) {
    hidden += (size_t)prob * a.T * H;
    w += (size_t)prob * a.E * H;
    expert_ids += (size_t)prob * a.T * a.k;
    weights += (size_t)prob * a.T * a.k;
    logits_out = logits_out != nullptr ? logits_out + (size_t)prob * logits_stride : nullptr;
  }
  const int T = a.T, E = a.E;
  // Workgroups go to the eight XCDs in turn; an XCD then works on one contiguous eighth
  // of the tiles (measured: up to 1.4 % on the kernel, nothing lost anywhere).
  const int per_xcd = (int)gridDim.x >> 3;
  const int tile = ((int)gridDim.x & 7) == 0 ? ((int)blockIdx.x & 7) * per_xcd + ((int)blockIdx.x >> 3)
                                            : (int)blockIdx.x;
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
  // products land in accumulator entries that are never used.  Addresses are a
  // wave-uniform base plus a 32-bit byte offset per lane.
  const int lrow = lane >> 3, lpiece = lane & 7;
  const size_t row_bytes = (size_t)H * 2;
  const unsigned char* hbase = reinterpret_cast<const unsigned char*>(hidden) + (size_t)tile * kTile * row_bytes;
  const unsigned char* wbase = reinterpret_cast<const unsigned char*>(w);
  const int last_row = T - 1 - tile * kTile;  // >= 0
  unsigned hoff[8], woff[2 * EB];
#pragma unroll
  for (int q = 0; q < 8; ++q) hoff[q] = (unsigned)(min(q * 8 + lrow, last_row) * row_bytes) + lpiece * 16;
#pragma unroll
  for (int q = 0; q < 2 * EB; ++q) woff[q] = (unsigned)(min(q * 8 + lrow, E - 1) * row_bytes) + lpiece * 16;
  // LDS side: the strip of this wave; write position of (row l/8, piece l%8), read
  // position of (row l%16, slot group l/16).
  unsigned char* strip = gate_lds + wave_u * kStripBytes;
  unsigned char* st_wr = strip + lrow * kRowBytes + lpiece * 16;
  unsigned char* st_rd = strip + (lane & 15) * kRowBytes + (lane >> 4) * 16;

  const int nfull = NM > 0 ? 8 * NM : H >> 6;  // (a constant when the loop is written out: no division below)
  const int nmine = (nfull - wave_u + kGateWaves - 1) / kGateWaves;  // chunks wave, wave+8, ...
  // Every tile starts its walk over the contraction axis at a different chunk, so
  // that the workgroups running at the same time do not all read the same column
  // range of their rows (which would land on the same memory channels).
  const int lim = nfull * 128;          // bytes of the full chunks of a row
  const int cstride = kGateWaves * 128;
  int koff = nfull > 0 ? ((tile * 5 + wave_u) % nfull) * 128 : 0;
  auto step = [&](int k) { k += cstride; return k >= lim ? k - lim : k; };  // nfull >= 8 when used

  u32x4 rh[8], rw[2 * EB];
  if constexpr (NM > 0) {
    // Exactly NM chunks per wave (H == 512 * NM), written out straight.  In flight
    // while chunk i is multiplied: the hidden rows of chunks i+1 and i+2 (from HBM;
    // register sets rh, rh2 in turn) and the W rows of chunk i+1 (from L2).  Loads
    // complete in issue order, so W(i+1) is issued before hidden(i+2).
    u32x4 rh2[8];
    int kw = koff;
    GATE_GH(rh, koff)
    GATE_GW(rw, kw)
    koff = step(koff);
    GATE_GH(rh2, koff)
#pragma unroll
    for (int i = 0; i < NM; ++i) {
      if (i % 2 == 0) {
        GATE_S(rh, rw)
      } else {
        GATE_S(rh2, rw)
      }
      if (i + 1 < NM) {
        kw = step(kw);
        GATE_GW(rw, kw)
      }
      if (i + 2 < NM) {
        koff = step(koff);
        if (i % 2 == 0) {
          GATE_GH(rh, koff)
        } else {
          GATE_GH(rh2, koff)
        }
      }
      GATE_M()
    }
  } else if (nmine > 0) {
    // any H: one chunk in flight per wave
    GATE_GH(rh, koff)
    GATE_GW(rw, koff)
    for (int i = 0; i + 1 < nmine; ++i) {
      GATE_S(rh, rw)      // chunk i staged (waits for its loads)
      koff = step(koff);
      GATE_GH(rh, koff)   // chunk i+1 in flight ...
      GATE_GW(rw, koff)
      GATE_M()            // ... while chunk i is multiplied
    }
    GATE_S(rh, rw)
    GATE_M()
  }
  // Ragged tail of the contraction axis (H % 64 != 0), taken by one wave: pieces
  // past H are read from the start of the row instead and replaced by zeros.
  if (NM == 0 && (H & 63) != 0 && wave_u == (nfull & (kGateWaves - 1))) {
    const u32x4 zero4 = {0u, 0u, 0u, 0u};
    const bool kin = nfull * 64 + lpiece * 8 < H;  // H % 8 == 0: a piece is all in or all out
    const int off = kin ? nfull * 128 : -lpiece * 16;
#pragma unroll
    for (int q = 0; q < 8; ++q) {
      const u32x4 v = load_global_16(hbase + hoff[q] + off);
      rh[q] = kin ? v : zero4;
    }
#pragma unroll
    for (int q = 0; q < 2 * EB; ++q) {
      const u32x4 v = load_global_16(wbase + woff[q] + off);
      rw[q] = kin ? v : zero4;
    }
    GATE_S(rh, rw)
    GATE_M()
  }
  __syncthreads();  // all strips are dead: the partial tiles reuse the space

  // Accumulator layout of the 16x16 MFMA: register r of lane l holds
  // row 4*(l/16) + r (expert) of column l%16 (token).
  float* part = reinterpret_cast<float*>(gate_lds);  // [8][64][kPartStride]
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

  // The eight partial tiles are summed on the fly by the analysis.
  analyse_tile<NE, kGateWaves, STATS>(part, kPartStride, mask64, &flex_lds, tile, a, ws, expert_ids,
                                      weights, logits_out);
}

template <int EB, int NE, int NM, bool STATS, bool BATCH>
static hipError_t launch_nmb(const void* hidden, const void* w, int H, const RouteArgs& a,
                             const Workspace& ws, int32_t* expert_ids, float* weights,
                             float* logits_out, size_t logits_stride, hipStream_t s) {
  static LdsAttr allowed;
  const void* fn = reinterpret_cast<const void*>(&gate_analyse_bf16_kernel<EB, NE, NM, STATS, BATCH>);
  const hipError_t e = allow_dynamic_lds(fn, kGateLdsBytes, allowed);
  if (e != hipSuccess) return e;
  clear_stale_error();
  hipLaunchKernelGGL((gate_analyse_bf16_kernel<EB, NE, NM, STATS, BATCH>), dim3(a.ntiles, a.nbatch), dim3(kGateThreads), kGateLdsBytes, s,
                     static_cast<const uint16_t*>(hidden), static_cast<const uint16_t*>(w), H, a, ws,
                     expert_ids, weights, logits_out, logits_stride);
  return hipGetLastError();
}

template <int EB, int NE, int NM, bool STATS>
static hipError_t launch_nm(const void* hidden, const void* w, int H, const RouteArgs& a,
                            const Workspace& ws, int32_t* expert_ids, float* weights,
                            float* logits_out, size_t logits_stride, hipStream_t s) {
  if (a.nbatch > 1)
    return launch_nmb<EB, NE, NM, STATS, true>(hidden, w, H, a, ws, expert_ids, weights, logits_out,
                                               logits_stride, s);
  return launch_nmb<EB, NE, NM, STATS, false>(hidden, w, H, a, ws, expert_ids, weights, logits_out,
                                              logits_stride, s);
}

template <int EB, int NE>
static hipError_t launch_one(const void* hidden, const void* w, int H, const RouteArgs& a,
                             const Workspace& ws, int32_t* expert_ids, float* weights,
                             float* logits_out, size_t logits_stride, hipStream_t s) {
  if (wants_stats(a)) {
    if (H == 2048) return launch_nm<EB, NE, 4, true>(hidden, w, H, a, ws, expert_ids, weights, logits_out, logits_stride, s);
    if (H == 4096) return launch_nm<EB, NE, 8, true>(hidden, w, H, a, ws, expert_ids, weights, logits_out, logits_stride, s);
    return launch_nm<EB, NE, 0, true>(hidden, w, H, a, ws, expert_ids, weights, logits_out, logits_stride, s);
  }
  if (H == 2048) return launch_nm<EB, NE, 4, false>(hidden, w, H, a, ws, expert_ids, weights, logits_out, logits_stride, s);
  if (H == 4096) return launch_nm<EB, NE, 8, false>(hidden, w, H, a, ws, expert_ids, weights, logits_out, logits_stride, s);
  return launch_nm<EB, NE, 0, false>(hidden, w, H, a, ws, expert_ids, weights, logits_out, logits_stride, s);
}

hipError_t launch_gate_analyse_bf16(const void* hidden, const void* w, int H, const RouteArgs& a,
                                    const Workspace& ws, int32_t* expert_ids, float* weights,
                                    float* logits_out, size_t logits_stride, hipStream_t s) {
  if (a.ntiles == 0) return hipSuccess;
  if (a.nseg > 0) return launch_gate_pipeline_bf16(hidden, w, H, a, ws, expert_ids, weights, logits_out, s);
  if (a.split > 0) return launch_gate_split_bf16(hidden, w, H, a, ws, expert_ids, weights, logits_out, s);
  switch (a.EP) {
    case 8: return launch_one<1, 1>(hidden, w, H, a, ws, expert_ids, weights, logits_out, logits_stride, s);
    case 16: return launch_one<1, 2>(hidden, w, H, a, ws, expert_ids, weights, logits_out, logits_stride, s);
    case 32: return launch_one<2, 4>(hidden, w, H, a, ws, expert_ids, weights, logits_out, logits_stride, s);
    default: return launch_one<4, 8>(hidden, w, H, a, ws, expert_ids, weights, logits_out, logits_stride, s);
  }
}

// fp32 path: one thread per (token, expert) dot product, float4 loads, fused
// multiply-add accumulation in h order.  Meant for small fp32 problems.
__global__ __launch_bounds__(256) void gate_f32_kernel(const float* __restrict__ hidden,
                                                       const float* __restrict__ w, int T, int H,
                                                       int E, float* __restrict__ logits,
                                                       size_t logits_stride) {
  hidden += (size_t)blockIdx.y * T * H;
  w += (size_t)blockIdx.y * E * H;
  logits += (size_t)blockIdx.y * logits_stride;
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

hipError_t launch_gate_f32(const float* hidden, const float* w, int T, int H, int E, int nbatch,
                           float* logits, size_t logits_stride, hipStream_t s) {
  const long long total = (long long)T * E;
  if (total == 0) return hipSuccess;
  const unsigned blocks = (unsigned)((total + 255) / 256);
  clear_stale_error();
  hipLaunchKernelGGL(gate_f32_kernel, dim3(blocks, nbatch), dim3(256), 0, s, hidden, w, T, H, E, logits,
                     logits_stride);
  return hipGetLastError();
}

}  // namespace laser
