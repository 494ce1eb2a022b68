// Shared pieces of the MFMA decode kernels (bf16 latent caches, d_cb = 128, d_r = 64): tile geometry,
// the LDS swizzle, wait-count helpers and the direct-to-LDS load.  Included inside namespace mlra's
// anonymous namespace of each kernel file.
#pragma once

#include "mlra_internal.h"

namespace mlra {
namespace mfma_tile {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(4))) short short4v;
typedef __attribute__((ext_vector_type(8))) short short8v;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;

constexpr int kDcb = 128, kDr = 64, kTile = 64, kHeadsWG = 128;
constexpr int kLatBytes = kTile * kDcb * 2;   // 16 KiB
constexpr int kRopeBytes = kTile * kDr * 2;   //  8 KiB
constexpr int kStageBytes = kLatBytes + kRopeBytes;
constexpr int kLoadsPerTile = 6;              // direct-to-LDS loads each thread issues per tile
constexpr int kZPitch = kDcb + 4;             // floats per head row of the epilogue buffer
constexpr float kNegBig = -1.0e30f;
constexpr float kLazy = 8.0f;                 // log2 headroom before the running max is refreshed

struct MfmaParams {
  const bf16_t* latent;
  const bf16_t* rope;
  const int32_t* page_table;
  const int32_t* seq_lens;
  const int32_t* seq_order;   // sequence ids in dispatch order, or null for 0, 1, 2, ...
  const int32_t* chunk_tab;   // per-sequence chunk length, or null for the uniform `chunk`
  const int32_t* unit_tab;    // active (sequence, chunk) pairs, sequence * 1024 + chunk, then -1 (with chunk_tab)
  const bf16_t* q_abs;
  const bf16_t* q_rope;
  float* part_z;
  float* part_ml;
  int page_size, max_pages, n_blocks, h, n_splits, chunk, batch;
  int groups;                 // head groups (Eq. (6)): block b serves the h heads of group b / (n_blocks / groups);
                              // q_rope holds groups * h heads.  1 = every block serves every head (Eq. (5))
  float scale_log2;
  int rows_bf16;              // 1: part_z receives each chunk's partial as z / l rounded to bf16, [..][chunk][head][channels]
                              // (what the MFMA epilogue merges); 0: fp32 partials, not normalised (generic merge, MLA)
};

// LDS has 64 four-byte banks; a 128-bit read is served 16 lanes at a time and a 64-bit transpose read
// 32 lanes at a time.  16-byte chunk c of latent token row t (256 bytes = one sweep of the banks) is
// stored at chunk position c ^ lat_swz(t): sixteen consecutive tokens put one logical chunk on sixteen
// different bank groups (score reads), and four consecutive tokens put a run of four chunks on four
// different quarters of the banks (transpose reads).  RoPE rows are 128 bytes, so two rows make one
// sweep and the row pair index is what permutes the eight chunks.
__device__ __forceinline__ int lat_swz(int t) { return ((t & 3) << 2) | ((t >> 2) & 3); }
__device__ __forceinline__ int rope_swz(int t) { return (t >> 1) & 7; }

template <int N>
__device__ __forceinline__ void wait_vmcnt() {
  static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit field");
  // gfx9 encoding: vmcnt[3:0] | expcnt[6:4] | lgkmcnt[11:8] | vmcnt[5:4] << 14 ; leave the others unbounded
  __builtin_amdgcn_s_waitcnt((N & 0xF) | (0x7 << 4) | (0xF << 8) | ((N >> 4) << 14));
}

// same, and also waits for every LDS / scalar-memory operation of this wave (lgkmcnt = 0)
template <int N>
__device__ __forceinline__ void wait_vm_lgkm() {
  static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit field");
  __builtin_amdgcn_s_waitcnt((N & 0xF) | (0x7 << 4) | (0x0 << 8) | ((N >> 4) << 14));
}

// Direct-to-LDS load: lane i's 16 bytes at (sbase + voff_i + OFF) land at LDS byte address
// m0 + OFF + 16 i (the instruction offset moves both sides).  Written as inline asm so that the
// compiler's wait-count insertion does not tie later LDS reads to these loads (it would drain all of
// them before every transpose read); completion is tracked by the explicit wait_vmcnt + barrier pairs
// below.  m0 is not otherwise used in this kernel.
__device__ __forceinline__ void set_m0(unsigned v) { asm volatile("s_mov_b32 m0, %0\n\ts_nop 0" : : "s"(v) : "memory"); }
template <int OFF>
__device__ __forceinline__ void lds_dma16(const void* sbase, unsigned voff) {
  asm volatile("global_load_lds_dwordx4 %0, %1 offset:%2" : : "v"(voff), "s"(sbase), "n"(OFF) : "memory");
}

__device__ __forceinline__ short4v lds_tr16(const __attribute__((address_space(3))) unsigned char* p) {
  return __builtin_amdgcn_ds_read_tr16_b64_v4i16((short4v __attribute__((address_space(3)))*)p);
}

}  // namespace mfma_tile
}  // namespace mlra
