// The bf16 gate projection and analysis of small calls: the contraction axis of a tile
// cut over several workgroups (see the comment above the kernel).
#include <atomic>

#include "gate_tile.h"

namespace laser {

// ---- small calls (fewer tiles than an eighth of the compute units) -------------------
//
// In gate_analyse_bf16_kernel one workgroup streams the 64 rows of its tile and all of W
// through one compute unit; with a handful of tiles the rest of the chip idles while that
// unit pulls its half megabyte at what one unit can pull.  Here the eight wavefront roles
// of that kernel -- role r owns the chunks r, r + 8, ... of the contraction axis, from
// load to MFMA, in the same order -- go to `split` workgroups of 8 / split roles each.
// Every workgroup leaves its roles' partial tiles in the workspace (stored write-through)
// and, all stores acknowledged, counts itself into the tile's counter; the workgroup that
// finds the count complete fetches the eight partial tiles (agent-scope loads), and goes on
// exactly as the other kernel does: the analysis adds the same eight partial tiles in the
// same order, so the logits, and with them everything else, are bit for bit those of a
// call that is not split.  Nobody waits for anybody.
//
// The counters must be zero before the first workgroup arrives and the caller's workspace
// holds whatever it held, so they live in the library's own memory: an array that is part
// of the code object (zero when it is loaded) of which every workspace address gets a slice
// on first sight.  The last workgroup of a tile sets the tile's counter back to zero.  Calls
// that share a workspace must not overlap anyway, so a slice has one user at a time.
template <int EB, int NE, bool STATS>
__global__ __launch_bounds__(kGateThreads) void gate_split_bf16_kernel(
    const uint16_t* __restrict__ hidden, const uint16_t* __restrict__ w, int H, const RouteArgs a0,
    const Workspace ws, int32_t* __restrict__ expert_ids, float* __restrict__ weights,
    float* __restrict__ logits_out) {
  extern __shared__ __align__(16) unsigned char gate_lds[];
  __shared__ unsigned long long mask64[64];
  __shared__ unsigned long long flex_lds;
  __shared__ int sh_last;
  RouteArgs a = a0;
  if (STATS && a.pool_in_ws) a.st_pool = ws.pool;
  const int T = a.T, E = a.E;
  const int split = a.split;  // workgroups per tile
  constexpr int nroles = 1;   // wavefront roles of a workgroup (the launcher sees to split == kGateWaves)
  // (the workgroups of a tile are ntiles apart in the grid)
  const int tile = (int)blockIdx.x % a.ntiles;
  const int role = (int)blockIdx.x / a.ntiles;
  const int part_of_tile = role;
  const int wave = threadIdx.x >> 6;
  const int lane = threadIdx.x & 63;
  const int wave_u = __builtin_amdgcn_readfirstlane(wave);

  // The role's chunks are those of wave `role` of the unsplit kernel, in its order:
  // chunk i is (start + 8 i) mod nfull.  Here wave v of the workgroup loads and stages
  // chunk v + 8 r in round r, so that all chunks of a round are in flight at once (a role
  // of the projection shapes with 2048 or 4096 columns is one round); then every wave
  // multiplies the round's chunks, in the role's order, into its own 16x16 blocks of the
  // partial tile: block (eb, tb) accumulates exactly the products it accumulates in the
  // unsplit kernel, in the same order, whoever runs the instructions.
  constexpr int kBlocks = EB * 4;                 // 16x16 blocks of the partial tile
  constexpr int kMine = (kBlocks + kGateWaves - 1) / kGateWaves;  // per wave: blocks wave, wave + 8
  f32x4 acc[kMine];
#pragma unroll
  for (int m = 0; m < kMine; ++m)
#pragma unroll
    for (int r = 0; r < 4; ++r) acc[m][r] = 0.0f;

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
  unsigned char* st_wr = gate_lds + wave_u * kStripBytes + lrow * kRowBytes + lpiece * 16;
  const unsigned rd_lane = (lane & 15) * kRowBytes + (lane >> 4) * 16;

  const int nfull = H >> 6;
  const int nmine = (nfull - role + kGateWaves - 1) / kGateWaves;  // full chunks of the role
  const int start = nfull > 0 ? (tile * 5 + role) % nfull : 0;
  // the ragged end of the contraction axis (H % 64 != 0) goes, as in the unsplit kernel, to
  // one role, after its full chunks: pieces past H are read from the start of the row
  // instead and replaced by zeros
  const bool ragged = (H & 63) != 0 && role == (nfull & (kGateWaves - 1));
  const int nitems = nmine + (ragged ? 1 : 0);
  const u32x4 zero4 = {0u, 0u, 0u, 0u};

  u32x4 rh[8], rw[2 * EB];
  auto load_item = [&](int i) {  // chunk i of the role, or (i == nmine) the ragged end
    if (i < nmine) {
      const int koff = ((start + kGateWaves * i) % nfull) * 128;
      GATE_GH(rh, koff)
      GATE_GW(rw, koff)
    } else {
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
    }
  };
  if (wave_u < nitems) load_item(wave_u);
  for (int r0 = 0; r0 < nitems; r0 += kGateWaves) {
    if (r0 + wave_u < nitems) {
      GATE_S(rh, rw)  // (waits for the loads)
    }
    __syncthreads();
    // the next round's loads travel while this round is multiplied
    if (r0 + kGateWaves + wave_u < nitems) load_item(r0 + kGateWaves + wave_u);
    const int nround = min(kGateWaves, nitems - r0);
    // chunk j of the round, from strip j
    auto multiply = [&](int j) {
      const unsigned char* st_rd = gate_lds + j * kStripBytes + rd_lane;
#pragma unroll
      for (int s_ = 0; s_ < 2; ++s_) {
#pragma unroll
        for (int m = 0; m < kMine; ++m) {
          const int blk = wave_u + m * kGateWaves;  // block (eb, tb) = (blk / 4, blk % 4)
          if (blk < kBlocks) {
            const u32x4 b_ = *(lds_u4_ptr)(st_rd + (blk & 3) * 16 * kRowBytes + s_ * 64);
            const u32x4 a_ = *(lds_u4_ptr)(st_rd + kTile * kRowBytes + (blk >> 2) * 16 * kRowBytes + s_ * 64);
            acc[m] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a_),
                                                             __builtin_bit_cast(bf16x8, b_), acc[m], 0, 0, 0);
          }
        }
      }
    };
    // (written out for the usual round sizes, so that the operand reads of a chunk do not
    // wait for the products of the chunk before)
    if (nround == 4) {
#pragma unroll
      for (int j = 0; j < 4; ++j) multiply(j);
    } else if (nround == 8) {
#pragma unroll
      for (int j = 0; j < 8; ++j) multiply(j);
    } else {
      for (int j = 0; j < nround; ++j) multiply(j);
    }
    __syncthreads();  // the strips are free again (after the last round: dead, the partial tile reuses the space)
  }
  if (nitems == 0) __syncthreads();

  float* part = reinterpret_cast<float*>(gate_lds);  // [roles][64][kPartStride]
  {
    const int n = lane & 15, kgrp = lane >> 4;
#pragma unroll
    for (int m = 0; m < kMine; ++m) {
      const int blk = wave_u + m * kGateWaves;
      if (blk < kBlocks) {
        const int eb = blk >> 2, tb = blk & 3;
        const float4 v = make_float4(acc[m][0], acc[m][1], acc[m][2], acc[m][3]);
        *reinterpret_cast<float4*>(part + (tb * 16 + n) * kPartStride + eb * 16 + 4 * kgrp) = v;
      }
    }
  }
  __syncthreads();

  // ---- this workgroup's partial tiles -> workspace, 64 x 64 floats per role ------------
  // (element j of a role's tile, 8 bytes: row j / 32, columns 2 (j % 32) and the next)
  constexpr int kPairs = kTile * 64 / 2;  // 8-byte elements per partial tile
  auto lds_pair = [&](int r, int jj) {
    return reinterpret_cast<unsigned long long*>(part + ((size_t)r * kTile + (jj >> 5)) * kPartStride + 2 * (jj & 31));
  };
  unsigned long long* const tile_parts =
      reinterpret_cast<unsigned long long*>(ws.split_part) + (size_t)tile * kGateWaves * kPairs;
  {
    unsigned long long* dst = tile_parts + (size_t)part_of_tile * nroles * kPairs;
    for (int j = threadIdx.x; j < nroles * kPairs; j += kGateThreads)
      __hip_atomic_store(dst + j, *lds_pair(j / kPairs, j % kPairs), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // every store acknowledged ...
  __syncthreads();                                   // ... by every wavefront
  if (threadIdx.x == 0) {
    int32_t* counter = a.split_cnt + tile;
    const int before = __hip_atomic_fetch_add(counter, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    const int last = before == split - 1;
    if (last) __hip_atomic_store(counter, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);  // for the next call
    sh_last = last;
  }
  __syncthreads();
  if (sh_last == 0) return;

  // ---- the last workgroup of the tile: all eight partial tiles -> LDS, then the analysis ----
  // Wave w fetches the tile of role w: 16 loads of 16 bytes per lane, 1 KiB per instruction
  // (with 8-byte loads the fetch took twice as long: the memory pipeline takes a wave's
  // instruction every 16 cycles whatever its width).  Agent-scope loads of 16 bytes exist
  // only as instructions, so they are written out, all of them and the wait for them in one
  // block: the compiler takes an output of a block as valid when the block ends.
  {
    const unsigned char* src = reinterpret_cast<const unsigned char*>(tile_parts) + (size_t)wave * (kPairs * 8) + lane * 16;
    const unsigned char *s0 = src, *s1 = src + 4096, *s2 = src + 8192, *s3 = src + 12288;
    u32x4 v[16];
    asm volatile(
        "global_load_dwordx4 %0, %16, off sc1\n\t"
        "global_load_dwordx4 %1, %16, off offset:1024 sc1\n\t"
        "global_load_dwordx4 %2, %16, off offset:2048 sc1\n\t"
        "global_load_dwordx4 %3, %16, off offset:3072 sc1\n\t"
        "global_load_dwordx4 %4, %17, off sc1\n\t"
        "global_load_dwordx4 %5, %17, off offset:1024 sc1\n\t"
        "global_load_dwordx4 %6, %17, off offset:2048 sc1\n\t"
        "global_load_dwordx4 %7, %17, off offset:3072 sc1\n\t"
        "global_load_dwordx4 %8, %18, off sc1\n\t"
        "global_load_dwordx4 %9, %18, off offset:1024 sc1\n\t"
        "global_load_dwordx4 %10, %18, off offset:2048 sc1\n\t"
        "global_load_dwordx4 %11, %18, off offset:3072 sc1\n\t"
        "global_load_dwordx4 %12, %19, off sc1\n\t"
        "global_load_dwordx4 %13, %19, off offset:1024 sc1\n\t"
        "global_load_dwordx4 %14, %19, off offset:2048 sc1\n\t"
        "global_load_dwordx4 %15, %19, off offset:3072 sc1\n\t"
        "s_waitcnt vmcnt(0)"
        : "=&v"(v[0]), "=&v"(v[1]), "=&v"(v[2]), "=&v"(v[3]), "=&v"(v[4]), "=&v"(v[5]), "=&v"(v[6]), "=&v"(v[7]),
          "=&v"(v[8]), "=&v"(v[9]), "=&v"(v[10]), "=&v"(v[11]), "=&v"(v[12]), "=&v"(v[13]), "=&v"(v[14]),
          "=&v"(v[15])
        : "v"(s0), "v"(s1), "v"(s2), "v"(s3)
        : "memory");
    // bytes 1024 u + 16 lane of the tile = row 4 u + lane / 16, columns 4 (lane % 16) ...
#pragma unroll
    for (int u = 0; u < 16; ++u)
      *reinterpret_cast<u32x4*>(part + ((size_t)wave * kTile + 4 * u + (lane >> 4)) * kPartStride + 4 * (lane & 15)) = v[u];
  }
  __syncthreads();
  analyse_tile<NE, kGateWaves, STATS>(part, kPartStride, mask64, &flex_lds, tile, a, ws, expert_ids, weights,
                                      logits_out);
}

// ---- the counters ---------------------------------------------------------------------
constexpr int kSplitSlices = 1024;
static __device__ int32_t split_counters[kSplitSlices * kSplitMaxTiles];

struct SplitTable {
  std::atomic<uintptr_t> key[kSplitSlices];  // workspace address that owns the slice, 0: free
  std::atomic<int32_t*> base;                // the array's address on this device
};
static SplitTable g_split[kMaxDevices];

int32_t* split_counters_for(const void* workspace) {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
  SplitTable& t = g_split[dev];
  int32_t* base = t.base.load(std::memory_order_acquire);
  if (base == nullptr) {
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(split_counters)) != hipSuccess || p == nullptr) {
      (void)hipGetLastError();
      return nullptr;
    }
    base = static_cast<int32_t*>(p);
    t.base.store(base, std::memory_order_release);
  }
  const uintptr_t k = reinterpret_cast<uintptr_t>(workspace);
  const unsigned h = (unsigned)((k >> 8) * 0x9E3779B1u);
  for (int probe = 0; probe < 64; ++probe) {
    const unsigned i = (h + (unsigned)probe) % kSplitSlices;
    uintptr_t cur = t.key[i].load(std::memory_order_acquire);
    if (cur == 0) {
      if (t.key[i].compare_exchange_strong(cur, k, std::memory_order_acq_rel)) cur = k;
      // (on failure `cur` holds what another thread put there)
    }
    if (cur == k) return base + (size_t)i * kSplitMaxTiles;
  }
  return nullptr;  // the table is crowded: the call runs without the split
}

template <int EB, int NE, bool STATS>
static hipError_t launch_split(const void* hidden, const void* w, int H, const RouteArgs& a, const Workspace& ws,
                               int32_t* expert_ids, float* weights, float* logits_out, hipStream_t s) {
  static LdsAttr allowed;
  const void* fn = reinterpret_cast<const void*>(&gate_split_bf16_kernel<EB, NE, STATS>);
  const hipError_t e = allow_dynamic_lds(fn, kGateLdsBytes, allowed);
  if (e != hipSuccess) return e;
  if (a.split != kGateWaves) return hipErrorInvalidValue;  // (one wavefront role per workgroup)
  clear_stale_error();
  hipLaunchKernelGGL((gate_split_bf16_kernel<EB, NE, STATS>), dim3(a.ntiles * a.split), dim3(kGateThreads),
                     kGateLdsBytes, s, static_cast<const uint16_t*>(hidden), static_cast<const uint16_t*>(w), H, a, ws,
                     expert_ids, weights, logits_out);
  return hipGetLastError();
}

template <int EB, int NE>
static hipError_t launch_split_one(const void* hidden, const void* w, int H, const RouteArgs& a, const Workspace& ws,
                                   int32_t* expert_ids, float* weights, float* logits_out, hipStream_t s) {
  if (wants_stats(a)) return launch_split<EB, NE, true>(hidden, w, H, a, ws, expert_ids, weights, logits_out, s);
  return launch_split<EB, NE, false>(hidden, w, H, a, ws, expert_ids, weights, logits_out, s);
}

hipError_t launch_gate_split_bf16(const void* hidden, const void* w, int H, const RouteArgs& a, const Workspace& ws,
                                  int32_t* expert_ids, float* weights, float* logits_out, hipStream_t s) {
  switch (a.EP) {
    case 8: return launch_split_one<1, 1>(hidden, w, H, a, ws, expert_ids, weights, logits_out, s);
    case 16: return launch_split_one<1, 2>(hidden, w, H, a, ws, expert_ids, weights, logits_out, s);
    case 32: return launch_split_one<2, 4>(hidden, w, H, a, ws, expert_ids, weights, logits_out, s);
    default: return launch_split_one<4, 8>(hidden, w, H, a, ws, expert_ids, weights, logits_out, s);
  }
}

}  // namespace laser
