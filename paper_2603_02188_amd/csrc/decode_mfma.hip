// MFMA decode kernel for bf16 latent caches with d_cb = 128, d_r = 64 (Step 2 of the absorbed decode,
// Eq. (1), applied to one latent block; the block loop of Eq. (5) is the grid's y dimension).
//
// One workgroup (4 wavefronts) owns one (context chunk, latent block, 128 query heads, sequence).
//   * Tiles of 64 tokens [C_b | K^RoPE] stream HBM -> LDS with direct-to-LDS loads, kStages deep.
//     The same LDS tile is the key (for the scores) and the value (for PV): V = C_b.
//   * Wave (hw, tw) owns heads [64 hw, 64 hw + 64) and tokens [32 tw, 32 tw + 32) of every tile.
//   * Scores are computed transposed, S^T = K Q^T (tokens x heads), so that in the MFMA accumulator
//     layout a lane owns one head column and the softmax row reductions are in-register plus one
//     lane^32 exchange.  P^T (bf16) is then already laid out as the B operand of
//     Z^T += V^T P^T (channels x heads); V^T comes from the row-major tile through LDS transpose reads.
//   * Running max is updated lazily (only when it grows by more than 2^8), which is exact: the
//     partial (m, l, z) stays self-consistent and the merge kernel normalises.
#include "mlra_internal.h"

namespace mlra {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
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
  const bf16_t* q_abs;
  const bf16_t* q_rope;
  float* part_z;
  float* part_ml;
  int page_size, max_pages, n_blocks, h, n_splits, chunk;
  float scale_log2;
};

// 16-byte chunk c of token row t is stored at chunk position c ^ swz(t & 7) of its row: eight
// consecutive tokens spread one logical chunk over all 32 banks (128-bit score reads), and four
// consecutive tokens spread a pair of chunks over all banks (64-bit transpose reads).
__device__ __forceinline__ int swz(int t) { return ((t & 3) << 1) | ((t >> 2) & 1); }

template <int N>
__device__ __forceinline__ void wait_vmcnt() {
  static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit field");
  // gfx9 encoding: vmcnt[3:0] | expcnt[6:4] | lgkmcnt[11:8] | vmcnt[5:4] << 14 ; leave the others unbounded
  __builtin_amdgcn_s_waitcnt((N & 0xF) | (0x7 << 4) | (0xF << 8) | ((N >> 4) << 14));
}

// Direct-to-LDS load: lane i's 16 bytes at (sbase + voff_i) land at LDS byte address m0_base + 16 i.
// Written as inline asm so that the compiler's wait-count insertion does not tie later LDS reads to
// these loads (it would drain all of them before every transpose read); completion is tracked by the
// explicit wait_vmcnt + barrier pairs below.  m0 is not otherwise used in this kernel.
__device__ __forceinline__ void lds_dma16(const void* sbase, unsigned voff, unsigned m0_base) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
               :
               : "s"(m0_base), "v"(voff), "s"(sbase)
               : "memory");
}

__device__ __forceinline__ short4v lds_tr16(const void* p) {
  return __builtin_amdgcn_ds_read_tr16_b64_v4i16((short4v __attribute__((address_space(3)))*)p);
}

template <int STAGES>
__global__ __launch_bounds__(256) void decode_mfma_kernel(MfmaParams p) {
  extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
  const int split = blockIdx.x;
  const int n_hg = (p.h + kHeadsWG - 1) / kHeadsWG;
  const int blk = blockIdx.y / n_hg, hgrp = blockIdx.y % n_hg;
  const int seq = blockIdx.z;
  const int n = p.seq_lens[seq];
  const int t0 = split * p.chunk;
  if (t0 >= n) return;
  const int t1 = min(n, t0 + p.chunk);
  const int ntiles = (t1 - t0 + kTile - 1) / kTile;
  const int nvalid_last = t1 - t0 - (ntiles - 1) * kTile;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int hw = wave & 1, tw = wave >> 1, g = lane >> 5, c32 = lane & 31;

  // ---- absorbed + RoPE queries as MFMA B operands, resident in registers for the whole chunk ----
  bf16x8 qreg[2][12];
#pragma unroll
  for (int nt = 0; nt < 2; ++nt) {
    const int head = min(hgrp * kHeadsWG + hw * 64 + nt * 32 + c32, p.h - 1);
    const bf16_t* qa = p.q_abs + (((size_t)seq * p.n_blocks + blk) * p.h + head) * kDcb + g * 8;
    const bf16_t* qr = p.q_rope + ((size_t)seq * p.h + head) * kDr + g * 8;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) qreg[nt][ks] = *(const bf16x8*)(qa + ks * 16);
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) qreg[nt][8 + ks] = *(const bf16x8*)(qr + ks * 16);
  }
  // Pin the queries into accumulation registers: MFMA reads its B operand from there directly, which
  // leaves the architectural VGPRs to the per-tile working set.
#pragma unroll
  for (int nt = 0; nt < 2; ++nt)
#pragma unroll
    for (int ks = 0; ks < 12; ++ks) asm volatile("" : "+a"(qreg[nt][ks]));

  // ---- page ids of up to 64 tiles ahead, one per lane ----
  const int32_t* pt_row = p.page_table + (size_t)seq * p.max_pages;
  auto load_page_ids = [&](int tile_base) {
    const int idx = min((t0 + (tile_base + lane) * kTile) / p.page_size, p.max_pages - 1);
    return pt_row[idx];
  };
  int pid_vec = load_page_ids(0);
  int pid_next = 0;

  // per-lane constants of the tile loads: row within the tile and byte offset within the row
  int lat_t[4], lat_off[4], rope_t[2], rope_off[2];
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    const int P = (wave * 4 + q) * 64 + lane;
    lat_t[q] = P >> 4;
    lat_off[q] = ((P & 15) ^ swz((P >> 4) & 7)) << 4;
  }
#pragma unroll
  for (int q = 0; q < 2; ++q) {
    const int P = (wave * 2 + q) * 64 + lane;
    rope_t[q] = P >> 3;
    rope_off[q] = ((P & 7) ^ swz((P >> 3) & 7)) << 4;
  }
  const unsigned lds_base = (unsigned)(size_t)(__attribute__((address_space(3))) unsigned char*)smem;
  const unsigned wave_u = __builtin_amdgcn_readfirstlane(wave);

  auto issue_tile = [&](int jj) {
    if ((jj & 63) == 32) pid_next = load_page_ids(jj + 32);
    if ((jj & 63) == 0 && jj > 0) pid_vec = pid_next;
    const int page = __builtin_amdgcn_readlane(pid_vec, jj & 63);
    const int tok0 = t0 + jj * kTile;
    const int slot0 = tok0 % p.page_size;
    const int last = min(kTile, t1 - tok0) - 1;   // rows past the chunk re-read its last row (finite, weight 0)
    const char* lat_base =
        (const char*)p.latent + ((((size_t)page * p.n_blocks + blk) * p.page_size + slot0) * kDcb) * 2;
    const char* rope_base = (const char*)p.rope + (((size_t)page * p.page_size + slot0) * kDr) * 2;
    const unsigned stage = lds_base + (jj % STAGES) * kStageBytes;
#pragma unroll
    for (int q = 0; q < 4; ++q)
      lds_dma16(lat_base, min(lat_t[q], last) * (kDcb * 2) + lat_off[q], stage + (wave_u * 4 + q) * 1024);
#pragma unroll
    for (int q = 0; q < 2; ++q)
      lds_dma16(rope_base, min(rope_t[q], last) * (kDr * 2) + rope_off[q],
                stage + kLatBytes + (wave_u * 2 + q) * 1024);
  };

  // ---- per-lane LDS read offsets ----
  const int s_tok = tw * 32 + c32;
  const int s_f = swz(s_tok & 7);
  int pv_off[2][4];
  {
    const int k = (lane & 15) >> 2, seg = lane & 3, hb = (lane >> 4) & 1;
#pragma unroll
    for (int s = 0; s < 2; ++s) {
      const int ta = tw * 32 + 16 * s + 4 * g + k;
      const int f = swz(ta & 7);
#pragma unroll
      for (int mt = 0; mt < 4; ++mt) {
        const int cc = 4 * mt + 2 * hb + (seg >> 1);
        pv_off[s][mt] = ta * (kDcb * 2) + ((cc ^ f) << 4) + ((seg & 1) << 3);
      }
    }
  }

  float m_run[2] = {kNegBig, kNegBig}, l_run[2] = {0.f, 0.f};
  f32x16 zacc[4][2];
#pragma unroll
  for (int mt = 0; mt < 4; ++mt)
#pragma unroll
    for (int nt = 0; nt < 2; ++nt)
#pragma unroll
      for (int i = 0; i < 16; ++i) zacc[mt][nt][i] = 0.f;

  const float sc = p.scale_log2;

  // online softmax of one 32-token x 32-head score tile (accumulator layout: this lane owns head
  // column c32 of head tile nt and 16 of the 32 tokens); returns P^T as the two B operands of PV
  auto softmax = [&](int nt, bool tail, f32x16& s, bf16x8 (&pb)[2]) {
    if (tail) {
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int tok = tw * 32 + (r >> 2) * 8 + g * 4 + (r & 3);
        if (tok >= nvalid_last) s[r] = -INFINITY;
      }
    }
    float mx = s[0];
#pragma unroll
    for (int r = 1; r < 16; ++r) mx = fmaxf(mx, s[r]);
    mx = fmaxf(mx, __shfl_xor(mx, 32));
    const float cand = mx * sc;
    const bool need = cand > m_run[nt] + kLazy;
    if (__any(need)) {
      const float m_new = need ? cand : m_run[nt];
      const float alpha = __builtin_amdgcn_exp2f(m_run[nt] - m_new);
#pragma unroll
      for (int mt = 0; mt < 4; ++mt)
#pragma unroll
        for (int i = 0; i < 16; ++i) zacc[mt][nt][i] *= alpha;
      l_run[nt] *= alpha;
      m_run[nt] = m_new;
    }
    const float neg_m = -m_run[nt];
    float lsum = 0.f;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const float pr = __builtin_amdgcn_exp2f(__builtin_fmaf(s[r], sc, neg_m));
      lsum += pr;
      pb[r >> 3][r & 7] = (__bf16)pr;
    }
    l_run[nt] += lsum;
  };

  // ---- main loop: loads run STAGES-1 tiles ahead of the tile being consumed ----
  for (int jj = 0; jj < STAGES - 1 && jj < ntiles; ++jj) issue_tile(jj);

  for (int j = 0; j < ntiles; ++j) {
    if (j + STAGES - 2 <= ntiles - 1) wait_vmcnt<kLoadsPerTile * (STAGES - 2)>(); else wait_vmcnt<0>();
    __builtin_amdgcn_s_barrier();   // tile j landed for every wave; everyone is done with tile j-1
    if (j + STAGES - 1 < ntiles) issue_tile(j + STAGES - 1);

    const unsigned char* lat = smem + (j % STAGES) * kStageBytes;
    const unsigned char* rope = lat + kLatBytes;
    const bool tail = (j == ntiles - 1) && (nvalid_last < kTile);

    // key operands (this wave's 32 token rows, all 192 channels) and transposed value operands
    bf16x8 ka[12], va[2][4];
#pragma unroll
    for (int ks = 0; ks < 8; ++ks)
      ka[ks] = *(const bf16x8*)(lat + s_tok * (kDcb * 2) + (((2 * ks + g) ^ s_f) << 4));
#pragma unroll
    for (int ks = 0; ks < 4; ++ks)
      ka[8 + ks] = *(const bf16x8*)(rope + s_tok * (kDr * 2) + (((2 * ks + g) ^ s_f) << 4));
#pragma unroll
    for (int ss = 0; ss < 2; ++ss)
#pragma unroll
      for (int mt = 0; mt < 4; ++mt) {
        const short4v lo = lds_tr16(lat + pv_off[ss][mt]);
        const short4v hi = lds_tr16(lat + pv_off[ss][mt] + 8 * (kDcb * 2));
        va[ss][mt] = __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
      }

    f32x16 s0, s1;
#pragma unroll
    for (int i = 0; i < 16; ++i) { s0[i] = 0.f; s1[i] = 0.f; }
#pragma unroll
    for (int ks = 0; ks < 12; ++ks) s0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka[ks], qreg[0][ks], s0, 0, 0, 0);
#pragma unroll
    for (int ks = 0; ks < 12; ++ks) s1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka[ks], qreg[1][ks], s1, 0, 0, 0);

    bf16x8 pb0[2], pb1[2];
    softmax(0, tail, s0, pb0);
#pragma unroll
    for (int ss = 0; ss < 2; ++ss)
#pragma unroll
      for (int mt = 0; mt < 4; ++mt)
        zacc[mt][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(va[ss][mt], pb0[ss], zacc[mt][0], 0, 0, 0);
    softmax(1, tail, s1, pb1);
#pragma unroll
    for (int ss = 0; ss < 2; ++ss)
#pragma unroll
      for (int mt = 0; mt < 4; ++mt)
        zacc[mt][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(va[ss][mt], pb1[ss], zacc[mt][1], 0, 0, 0);
  }

  // ---- merge the two token halves of each head half through LDS, write the chunk's partial ----
#pragma unroll
  for (int nt = 0; nt < 2; ++nt) l_run[nt] += __shfl_xor(l_run[nt], 32);
  __builtin_amdgcn_s_barrier();     // every wave is past its last tile read: the stages can be reused
  float* mbuf = (float*)smem;                 // [4 waves][64 heads]
  float* lbuf = mbuf + 256;
  float* zbuf = (float*)(smem + 2048);        // [128 heads][kZPitch]
  if (g == 0) {
#pragma unroll
    for (int nt = 0; nt < 2; ++nt) {
      mbuf[wave * 64 + nt * 32 + c32] = m_run[nt];
      lbuf[wave * 64 + nt * 32 + c32] = l_run[nt];
    }
  }
  __syncthreads();
  float m_out[2], l_out[2];
#pragma unroll
  for (int nt = 0; nt < 2; ++nt) {
    const float mp = mbuf[(wave ^ 2) * 64 + nt * 32 + c32];
    const float lp = lbuf[(wave ^ 2) * 64 + nt * 32 + c32];
    const float ms = fmaxf(m_run[nt], mp);
    const float w_own = __builtin_amdgcn_exp2f(m_run[nt] - ms);
    const float w_par = __builtin_amdgcn_exp2f(mp - ms);
    m_out[nt] = ms;
    l_out[nt] = l_run[nt] * w_own + lp * w_par;
#pragma unroll
    for (int mt = 0; mt < 4; ++mt)
#pragma unroll
      for (int i = 0; i < 16; ++i) zacc[mt][nt][i] *= w_own;
  }
  auto zrow = [&](int nt, int mt, int r4) {
    return zbuf + (hw * 64 + nt * 32 + c32) * kZPitch + mt * 32 + r4 * 8 + g * 4;
  };
  if (tw == 1) {
#pragma unroll
    for (int nt = 0; nt < 2; ++nt)
#pragma unroll
      for (int mt = 0; mt < 4; ++mt)
#pragma unroll
        for (int r4 = 0; r4 < 4; ++r4) {
          f32x4 v = {zacc[mt][nt][r4 * 4], zacc[mt][nt][r4 * 4 + 1], zacc[mt][nt][r4 * 4 + 2],
                     zacc[mt][nt][r4 * 4 + 3]};
          *(f32x4*)zrow(nt, mt, r4) = v;
        }
  }
  __syncthreads();
  if (tw == 0) {
#pragma unroll
    for (int nt = 0; nt < 2; ++nt)
#pragma unroll
      for (int mt = 0; mt < 4; ++mt)
#pragma unroll
        for (int r4 = 0; r4 < 4; ++r4) {
          f32x4 v = *(f32x4*)zrow(nt, mt, r4);
          v[0] += zacc[mt][nt][r4 * 4];
          v[1] += zacc[mt][nt][r4 * 4 + 1];
          v[2] += zacc[mt][nt][r4 * 4 + 2];
          v[3] += zacc[mt][nt][r4 * 4 + 3];
          *(f32x4*)zrow(nt, mt, r4) = v;
        }
  }
  __syncthreads();
  const size_t unit = ((size_t)seq * p.n_blocks + blk) * p.n_splits + split;
  const int head_base = hgrp * kHeadsWG;
  for (int idx = tid; idx < kHeadsWG * (kDcb / 4); idx += 256) {
    const int hl = idx / (kDcb / 4), f4 = idx % (kDcb / 4);
    if (head_base + hl < p.h)
      *(f32x4*)(p.part_z + (unit * p.h + head_base + hl) * kDcb + f4 * 4) = *(const f32x4*)(zbuf + hl * kZPitch + f4 * 4);
  }
  if (tw == 0 && g == 0) {
#pragma unroll
    for (int nt = 0; nt < 2; ++nt) {
      const int head = head_base + hw * 64 + nt * 32 + c32;
      if (head < p.h) {
        p.part_ml[(unit * p.h + head) * 2 + 0] = m_out[nt];
        p.part_ml[(unit * p.h + head) * 2 + 1] = l_out[nt];
      }
    }
  }
}

constexpr int kStages = 4;

}  // namespace

bool decode_mfma_supported(const DecodeArgs& a) {
  return a.dtype == MLRA_BF16 && a.d_cb == kDcb && a.d_r == kDr && a.page_size % kTile == 0 &&
         a.plan.chunk_tokens % kTile == 0;
}

int launch_decode_mfma(const DecodeArgs& a) {
  static bool configured = false;
  const int lds = kStages * kStageBytes;
  if (!configured) {
    if (hipFuncSetAttribute((const void*)decode_mfma_kernel<kStages>, hipFuncAttributeMaxDynamicSharedMemorySize,
                            lds) != hipSuccess)
      return MLRA_ERR_LAUNCH;
    configured = true;
  }
  MfmaParams p;
  p.latent = (const bf16_t*)a.latent;
  p.rope = (const bf16_t*)a.rope;
  p.page_table = a.page_table;
  p.seq_lens = a.seq_lens;
  p.q_abs = (const bf16_t*)a.q_abs;
  p.q_rope = (const bf16_t*)a.q_rope;
  p.part_z = a.part_z;
  p.part_ml = a.part_ml;
  p.page_size = a.page_size;
  p.max_pages = a.max_pages;
  p.n_blocks = a.n_blocks;
  p.h = a.h;
  p.n_splits = a.plan.n_splits;
  p.chunk = a.plan.chunk_tokens;
  p.scale_log2 = a.softmax_scale * 1.4426950408889634f;
  const int n_hg = (a.h + kHeadsWG - 1) / kHeadsWG;
  dim3 grid(a.plan.n_splits, a.n_blocks * n_hg, a.batch);
  decode_mfma_kernel<kStages><<<grid, 256, lds, a.stream>>>(p);
  return check_launch();
}

}  // namespace mlra
