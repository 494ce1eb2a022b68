// Split-role MFMA decode kernel for bf16 latent caches with d_cb = 128, d_r = 64 (Step 2 of the absorbed
// decode, Eq. (1), applied to one latent block; the block loop of Eq. (5) is spread over workgroups).
//
// One workgroup = 8 wavefronts = 4 pairs; pair (hw, tw) owns heads [64 hw, 64 hw + 64) and tokens
// [32 tw, 32 tw + 32) of every 64-token tile [C_b | K^RoPE].  The two waves of a pair sit on the same
// SIMD and split the work by role, so that neither needs more than half of the register file and the
// SIMD always has a second instruction stream to issue from:
//   * the score wave keeps the absorbed + RoPE queries (96 registers), computes S^T = K Q^T, the column
//     maxima, P^T = 2^(tau' S^T - m) and the row sums, and hands P^T (bf16, already in the layout of an
//     MFMA B operand) to its partner through LDS;
//   * the value wave keeps the Z accumulators (128 registers), issues the direct-to-LDS tile loads,
//     and computes Z^T += V^T P^T one tile behind, with V^T from LDS transpose reads of the same tile.
// One workgroup barrier per tile orders everything: tile j+2 has landed, P^T of tile j is complete,
// and the stage of tile j-1 and the P^T buffer of tile j-1 are free.  When a running maximum has to be
// refreshed (lazily, see decode_mfma.hip) the score wave passes the rescale factors and a flag along
// with P^T.
#include "mfma_tile.h"

namespace mlra {
namespace {

using namespace mfma_tile;

constexpr int kSStages = 5;
constexpr int kSLoadsPerTile = 6;                        // per value wave (4 of them share a tile)
constexpr int kPPairBytes = 4 * 64 * 16;                 // P^T of one pair and tile: 4 operands x 64 lanes x 16 B
constexpr int kPBufBytes = 4 * kPPairBytes;              // all four pairs
constexpr int kPOff = kSStages * kStageBytes;            // two P^T buffers (tile parity)
constexpr int kAlphaOff = kPOff + 2 * kPBufBytes;        // rescale factors [parity][pair][64 heads]
constexpr int kFlagOff = kAlphaOff + 2 * 4 * 64 * 4;     // rescale flags   [parity][pair]
constexpr int kMlOff = kFlagOff + 64;                    // final (m, l) of the score waves [pair][2][64]
constexpr int kSplitLdsBytes = kMlOff + 4 * 2 * 64 * 4;  // 159,808 bytes

typedef const __attribute__((address_space(3))) bf16x8* lds_bf16x8_ptr;
typedef __attribute__((address_space(3))) bf16x8* lds_bf16x8_wptr;
typedef const __attribute__((address_space(3))) unsigned char* lds_byte_ptr;

__device__ __forceinline__ void swap_halves(float& a, float& b) {
  // exchanges the upper half of a with the lower half of b
  asm volatile("s_nop 1\n\tv_permlane32_swap_b32 %0, %1\n\ts_nop 1" : "+v"(a), "+v"(b));
}

__global__ __launch_bounds__(512) void decode_split_kernel(MfmaParams p) {
  extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
  // Workgroup -> (sequence, chunk, block, head group): the members of one (sequence, chunk) family get
  // ids 8 apart so that they share an XCD and its L2 (see decode_mfma.hip).
  const int n_hg = (p.h + kHeadsWG - 1) / kHeadsWG;
  const int fam = p.n_blocks * n_hg;
  const int n_units = p.n_splits * p.batch;
  const int full_units = n_units & ~7;
  int wg = blockIdx.x, su, member;
  if (wg < full_units * fam) {
    const int r = wg >> 3;
    member = r % fam;
    su = (r / fam) * 8 + (wg & 7);
  } else {
    wg -= full_units * fam;
    su = full_units + wg / fam;
    member = wg % fam;
  }
  const int split = su % p.n_splits, seq = su / p.n_splits;
  const int blk = member / n_hg, hgrp = member % n_hg;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int role = __builtin_amdgcn_readfirstlane(wave >> 2);   // 0: scores + softmax, 1: loads + PV
  const int pw = wave & 3, hw = pw & 1, tw = pw >> 1, g = lane >> 5, c32 = lane & 31;
  const unsigned pw_u = __builtin_amdgcn_readfirstlane(pw);
  const int t0 = split * p.chunk;
  typedef const __attribute__((address_space(4))) int32_t* const_i32_ptr;
  const int n = ((const_i32_ptr)p.seq_lens)[seq];
  if (t0 >= n) return;
  const int t1 = min(n, t0 + p.chunk);
  const int ntiles = (t1 - t0 + kTile - 1) / kTile;
  const int nvalid_last = t1 - t0 - (ntiles - 1) * kTile;
  const unsigned lds_base = (unsigned)(size_t)(__attribute__((address_space(3))) unsigned char*)smem;
  const float sc = p.scale_log2;
  const size_t unit = ((size_t)seq * p.n_blocks + blk) * p.n_splits + split;
  const int head_base = hgrp * kHeadsWG;
  float* ml_lds = (float*)(smem + kMlOff);                // [pair][m | l][64 heads]
  float* zbuf = (float*)smem;                             // epilogue: [128 heads][kZPitch], over the stages

  if (role == 0) {
    // =============================== score waves ===============================
    // queries (B operand of every score MFMA), loaded invisibly to the compiler's wait-count bookkeeping;
    // nothing reads them before the explicit wait below.  Both roles share one register allocation, so
    // everything stays in architectural VGPRs: 256 per wave at two waves per SIMD.
    bf16x8 qreg[2][12];
#pragma unroll
    for (int nt = 0; nt < 2; ++nt) {
      const int head = min(head_base + hw * 64 + nt * 32 + c32, p.h - 1);
      const bf16_t* qa = p.q_abs + (((size_t)seq * p.n_blocks + blk) * p.h + head) * kDcb + g * 8;
      const bf16_t* qr = p.q_rope + ((size_t)seq * p.h + head) * kDr + g * 8;
#pragma unroll
      for (int ks = 0; ks < 8; ++ks)
        asm volatile("global_load_dwordx4 %0, %1, off offset:%2" : "=v"(qreg[nt][ks]) : "v"(qa), "n"(ks * 32) : "memory");
#pragma unroll
      for (int ks = 0; ks < 4; ++ks)
        asm volatile("global_load_dwordx4 %0, %1, off offset:%2" : "=v"(qreg[nt][8 + ks]) : "v"(qr), "n"(ks * 32) : "memory");
    }
    // per-lane LDS read offsets of the K operands (XOR swizzle: see mfma_tile.h and decode_mfma.hip)
    const int s_tok = tw * 32 + c32;
    const unsigned k_lat_off = s_tok * (kDcb * 2) + ((g ^ lat_swz(s_tok)) << 4);
    const unsigned k_rope_off = kLatBytes + s_tok * (kDr * 2) + ((g ^ rope_swz(s_tok)) << 4);
    auto load_k = [&](int st, bf16x8 (&ka)[12]) {
      const unsigned lat = lds_base + st * kStageBytes + k_lat_off;
      const unsigned rope = lds_base + st * kStageBytes + k_rope_off;
#pragma unroll
      for (int ks = 0; ks < 8; ++ks) ka[ks] = *(lds_bf16x8_ptr)(size_t)(lat ^ (ks << 5));
#pragma unroll
      for (int ks = 0; ks < 4; ++ks) ka[8 + ks] = *(lds_bf16x8_ptr)(size_t)(rope ^ (ks << 5));
    };
    auto max16 = [&](const f32x16& sv) {
      float mx = fmaxf(fmaxf(sv[0], sv[1]), sv[2]);
#pragma unroll
      for (int r = 3; r < 15; r += 2) mx = fmaxf(fmaxf(mx, sv[r]), sv[r + 1]);
      return fmaxf(mx, sv[15]);
    };

    float m_run[2] = {kNegBig, kNegBig}, l_run[2] = {0.f, 0.f};
    wait_vmcnt<0>();                 // the queries (this wave issues no other vector-memory loads)
    __builtin_amdgcn_s_barrier();    // tiles 0 and 1 have landed
    bf16x8 ka[12];
    load_k(0, ka);
    int st_next = 1;                 // stage of tile j + 1
    for (int j = 0; j < ntiles; ++j) {
      f32x16 s0, s1;
#pragma unroll
      for (int i = 0; i < 16; ++i) { s0[i] = 0.f; s1[i] = 0.f; }
#pragma unroll
      for (int ks = 0; ks < 12; ++ks) {
        s0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka[ks], qreg[0][ks], s0, 0, 0, 0);
        s1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka[ks], qreg[1][ks], s1, 0, 0, 0);
        // keeps ka[0] alive past the two MFMAs whose accumulator input is the constant 0, so that the
        // allocator cannot place their destination on top of it (the build also scans for that)
        if (ks == 1) asm volatile("" : : "v"(ka[0]));
      }
      // K operands of the next tile (it landed before the previous barrier); a stale stage after the
      // last tile, never used
      load_k(st_next, ka);
      st_next = (st_next + 1 == kSStages) ? 0 : st_next + 1;
      // column maxima of both head tiles: in-register over this lane's 16 token rows, then two
      // half-wave swaps fold in the 16 rows of the lane 32 away
      float mx0 = max16(s0), mx1 = max16(s1);
      swap_halves(mx0, mx1);
      mx0 = fmaxf(mx0, mx1);
      mx1 = mx0;
      swap_halves(mx0, mx1);
      const float cand0 = mx0 * sc, cand1 = mx1 * sc;
      const int par = j & 1;
      float* alpha_lds = (float*)(smem + kAlphaOff) + (par * 4 + pw) * 64;
      int* flag_lds = (int*)(smem + kFlagOff) + par * 4 + pw;
      int flag = 0;
      if (j == 0) {
        m_run[0] = cand0;
        m_run[1] = cand1;
      } else {
        const bool need0 = cand0 > m_run[0] + kLazy, need1 = cand1 > m_run[1] + kLazy;
        if (__any(need0 || need1)) {
          const float mn0 = need0 ? cand0 : m_run[0], mn1 = need1 ? cand1 : m_run[1];
          const float a0 = __builtin_amdgcn_exp2f(m_run[0] - mn0), a1 = __builtin_amdgcn_exp2f(m_run[1] - mn1);
          l_run[0] *= a0;
          l_run[1] *= a1;
          m_run[0] = mn0;
          m_run[1] = mn1;
          if (g == 0) { alpha_lds[c32] = a0; alpha_lds[32 + c32] = a1; }
          flag = 1;
        }
      }
      if (lane == 0) *flag_lds = flag;
      if (j == ntiles - 1 && nvalid_last < kTile) {
        // Rows past the end of a ragged last tile hold copies of its last valid row (see the loader):
        // their scores equal a valid score, so the maxima above are right (and finite even for a wave
        // whose 32 rows are all past the end); their probabilities are what has to vanish.
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int tok = tw * 32 + (r >> 2) * 8 + g * 4 + (r & 3);
          if (tok >= nvalid_last) { s0[r] = -INFINITY; s1[r] = -INFINITY; }
        }
      }
      // probabilities, fp32 row sums, bf16 P^T into the partner's buffer
      unsigned char* pdst = smem + kPOff + par * kPBufBytes + pw * kPPairBytes + lane * 16;
#pragma unroll
      for (int nt = 0; nt < 2; ++nt) {
        const f32x16& sv = nt == 0 ? s0 : s1;
        const float neg_m = -m_run[nt];
        float lsum = 0.f;
#pragma unroll
        for (int ss = 0; ss < 2; ++ss) {
          bf16x8 pb;
#pragma unroll
          for (int e = 0; e < 8; ++e) {
            const float pe = __builtin_amdgcn_exp2f(__builtin_fmaf(sv[ss * 8 + e], sc, neg_m));
            lsum += pe;
            pb[e] = (__bf16)pe;
          }
          *(bf16x8*)(pdst + (nt * 2 + ss) * 1024) = pb;
        }
        l_run[nt] += lsum;
      }
      wait_vm_lgkm<63>();              // the P^T / factor / flag stores have completed (lgkmcnt = 0)
      __builtin_amdgcn_s_barrier();    // barrier of tile j
    }
    __builtin_amdgcn_s_barrier();      // the value waves' last tile
    // final (m, l) of this wave's heads to the value waves
    float l0 = l_run[0], l1 = l_run[1];
    float l0b = l0, l1b = l1;
    swap_halves(l0, l0b);              // l0 = {lower, lower}, l0b = {upper, upper}
    swap_halves(l1, l1b);
    l0 += l0b;
    l1 += l1b;
    if (g == 0) {
      ml_lds[pw * 128 + c32] = m_run[0];
      ml_lds[pw * 128 + 32 + c32] = m_run[1];
      ml_lds[pw * 128 + 64 + c32] = l0;
      ml_lds[pw * 128 + 96 + c32] = l1;
    }
    __syncthreads();   // E1
    __syncthreads();   // E2
    __syncthreads();   // E3
  } else {
    // =============================== value waves ===============================
    const const_i32_ptr pt_row = (const_i32_ptr)(p.page_table + (size_t)seq * p.max_pages);
    int issue_page_idx = t0 / p.page_size;
    int issue_page = pt_row[min(issue_page_idx, p.max_pages - 1)];
    // Tile loads: value wave w fills LDS chunks [256 w, 256 w + 256) of the latent tile with four loads
    // and chunks [128 w, 128 w + 128) of the RoPE tile with two (layout as in decode_mfma.hip).
    unsigned lat_voff[4], rope_voff[2];
#pragma unroll
    for (int q = 0; q < 4; ++q)
      lat_voff[q] = (lane >> 4) * (kDcb * 2) + (((lane & 15) ^ lat_swz(4 * q + (lane >> 4))) << 4);
#pragma unroll
    for (int q = 0; q < 2; ++q)
      rope_voff[q] = (lane >> 3) * (kDr * 2) + (((lane & 7) ^ rope_swz(8 * q + (lane >> 3))) << 4);
    const size_t lat_page_bytes = (size_t)p.n_blocks * p.page_size * (kDcb * 2);
    const size_t rope_page_bytes = (size_t)p.page_size * (kDr * 2);
    const char* lat_blk = (const char*)p.latent + (size_t)blk * p.page_size * (kDcb * 2);
    int issue_slot = t0 % p.page_size;   // slot of the next tile to issue inside its page (tiles go in order)
    int issue_stage = 0;
    auto issue_tile = [&](int jj) {
      const unsigned page = (unsigned)issue_page;
      const int last = min(kTile, t1 - t0 - jj * kTile) - 1;
      const char* lat_tile = lat_blk + page * lat_page_bytes + (unsigned)issue_slot * (unsigned)(kDcb * 2);
      const char* rope_tile = (const char*)p.rope + page * rope_page_bytes + (unsigned)issue_slot * (unsigned)(kDr * 2);
      const unsigned stage = lds_base + issue_stage * kStageBytes;
      if (last == kTile - 1) {
        set_m0(stage + pw_u * 4096);
        lds_dma16<0>(lat_tile + pw_u * 4096, lat_voff[0]);
        lds_dma16<1024>(lat_tile + pw_u * 4096, lat_voff[1]);
        lds_dma16<2048>(lat_tile + pw_u * 4096, lat_voff[2]);
        lds_dma16<3072>(lat_tile + pw_u * 4096, lat_voff[3]);
        set_m0(stage + kLatBytes + pw_u * 2048);
        lds_dma16<0>(rope_tile + pw_u * 2048, rope_voff[0]);
        lds_dma16<1024>(rope_tile + pw_u * 2048, rope_voff[1]);
      } else {
        // ragged end of the chunk: rows past it re-read its last row (finite values, weight 0 later).
        // Offsets are taken from the tile start so that they never go negative.
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const int t = (pw * 4 + q) * 4 + (lane >> 4);        // 0..63
          const unsigned row = (unsigned)min(t, last);           // 0..last
          set_m0(stage + pw_u * 4096 + q * 1024);
          lds_dma16<0>(lat_tile, row * (kDcb * 2) + (((lane & 15) ^ lat_swz(t)) << 4));
        }
#pragma unroll
        for (int q = 0; q < 2; ++q) {
          const int t = (pw * 2 + q) * 8 + (lane >> 3);        // 0..63
          const unsigned row = (unsigned)min(t, last);
          set_m0(stage + kLatBytes + pw_u * 2048 + q * 1024);
          lds_dma16<0>(rope_tile, row * (kDr * 2) + (((lane & 7) ^ rope_swz(t)) << 4));
        }
      }
      issue_slot += kTile;
      if (issue_slot >= p.page_size) {
        issue_slot = 0;
        ++issue_page_idx;
        issue_page = pt_row[min(issue_page_idx, p.max_pages - 1)];
      }
      issue_stage = (issue_stage + 1 == kSStages) ? 0 : issue_stage + 1;
    };
    // transpose-read offsets of the V operands
    unsigned v_off[2];
    {
      const int k = (lane & 15) >> 2, seg = lane & 3, hb = (lane >> 4) & 1;
#pragma unroll
      for (int half = 0; half < 2; ++half) {
        const int ta = tw * 32 + 8 * half + 4 * g + k;
        v_off[half] = ta * (kDcb * 2) + (((2 * hb + (seg >> 1)) ^ lat_swz(ta)) << 4) + ((seg & 1) << 3);
      }
    }
    f32x16 zacc[4][2];
#pragma unroll
    for (int mt = 0; mt < 4; ++mt)
#pragma unroll
      for (int nt = 0; nt < 2; ++nt)
#pragma unroll
        for (int i = 0; i < 16; ++i) zacc[mt][nt][i] = 0.f;

    for (int jj = 0; jj < kSStages && jj < ntiles; ++jj) issue_tile(jj);
    if (ntiles >= kSStages) wait_vmcnt<kSLoadsPerTile * (kSStages - 2)>(); else wait_vmcnt<0>();
    __builtin_amdgcn_s_barrier();    // tiles 0 and 1 have landed
    // barrier of tile 0: tile 2 has landed (tiles 3 and 4 may still be in flight)
    if (ntiles >= kSStages) wait_vmcnt<kSLoadsPerTile * (kSStages - 3)>(); else wait_vmcnt<0>();
    __builtin_amdgcn_s_barrier();
    int st_cur = 0;                  // stage of tile j - 1
    for (int j = 1; j <= ntiles; ++j) {
      const int par = (j - 1) & 1;
      // the stage of tile j-2 is free: every wave passed the previous barrier (tiles 0..4 went out in
      // the prologue, so the first tile issued here is tile 5 at j = 2)
      if (j >= 2 && j + 3 < ntiles) issue_tile(j + 3);
      const int flag = __builtin_amdgcn_readfirstlane(*((const int*)(smem + kFlagOff) + par * 4 + pw));
      if (flag) {
        const float* alpha_lds = (const float*)(smem + kAlphaOff) + (par * 4 + pw) * 64;
        const float a0 = alpha_lds[c32], a1 = alpha_lds[32 + c32];
#pragma unroll
        for (int mt = 0; mt < 4; ++mt)
#pragma unroll
          for (int i = 0; i < 16; ++i) { zacc[mt][0][i] *= a0; zacc[mt][1][i] *= a1; }
      }
      bf16x8 pb[2][2], va[2][4];
      const unsigned char* psrc = smem + kPOff + par * kPBufBytes + pw * kPPairBytes + lane * 16;
#pragma unroll
      for (int nt = 0; nt < 2; ++nt)
#pragma unroll
        for (int ss = 0; ss < 2; ++ss) pb[nt][ss] = *(const bf16x8*)(psrc + (nt * 2 + ss) * 1024);
      {
        const unsigned lo_base = lds_base + st_cur * kStageBytes + v_off[0];
        const unsigned hi_base = lds_base + st_cur * kStageBytes + v_off[1];
#pragma unroll
        for (int mt = 0; mt < 4; ++mt) {
          const lds_byte_ptr lo_p = (lds_byte_ptr)(size_t)(lo_base ^ (mt << 6));
          const lds_byte_ptr hi_p = (lds_byte_ptr)(size_t)(hi_base ^ (mt << 6));
#pragma unroll
          for (int ss = 0; ss < 2; ++ss) {
            const short4v lo = lds_tr16(lo_p + ss * 16 * (kDcb * 2));
            const short4v hi = lds_tr16(hi_p + ss * 16 * (kDcb * 2));
            va[ss][mt] = __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
          }
        }
      }
#pragma unroll
      for (int ss = 0; ss < 2; ++ss)
#pragma unroll
        for (int mt = 0; mt < 4; ++mt) {
          zacc[mt][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(va[ss][mt], pb[0][ss], zacc[mt][0], 0, 0, 0);
          zacc[mt][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(va[ss][mt], pb[1][ss], zacc[mt][1], 0, 0, 0);
        }
      st_cur = (st_cur + 1 == kSStages) ? 0 : st_cur + 1;
      // barrier of tile j: tile j+2 has landed (tile j+3 may still be in flight) and this wave's LDS
      // reads have returned
      if (j + 3 < ntiles) wait_vm_lgkm<kSLoadsPerTile>(); else wait_vm_lgkm<0>();
      __builtin_amdgcn_s_barrier();
    }
    // ---- merge the two token halves of each head half through LDS, write the chunk's partial ----
    __syncthreads();   // E1: the score waves' (m, l) are in LDS; nobody reads a stage any more
    float m_out[2], l_out[2];
#pragma unroll
    for (int nt = 0; nt < 2; ++nt) {
      const float m_own = ml_lds[pw * 128 + nt * 32 + c32], l_own = ml_lds[pw * 128 + 64 + nt * 32 + c32];
      const float mp = ml_lds[(pw ^ 2) * 128 + nt * 32 + c32], lp = ml_lds[(pw ^ 2) * 128 + 64 + nt * 32 + c32];
      const float ms = fmaxf(m_own, mp);
      const float w_own = __builtin_amdgcn_exp2f(m_own - ms);
      const float w_par = __builtin_amdgcn_exp2f(mp - ms);
      m_out[nt] = ms;
      l_out[nt] = l_own * w_own + lp * w_par;
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
    __syncthreads();   // E2
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
      if (g == 0) {
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
    __syncthreads();   // E3
  }
  // all 512 threads copy the merged Z of the workgroup's 128 heads to the partial
  for (int idx = tid; idx < kHeadsWG * (kDcb / 4); idx += 512) {
    const int hl = idx / (kDcb / 4), f4 = idx % (kDcb / 4);
    if (head_base + hl < p.h)
      *(f32x4*)(p.part_z + (unit * p.h + head_base + hl) * kDcb + f4 * 4) = *(const f32x4*)(zbuf + hl * kZPitch + f4 * 4);
  }
}

}  // namespace

bool decode_split_supported(const DecodeArgs& a) {
  return a.dtype == MLRA_BF16 && a.d_cb == kDcb && a.d_r == kDr && a.page_size % kTile == 0 &&
         a.plan.chunk_tokens % kTile == 0;
}

int launch_decode_split(const DecodeArgs& a) {
  static bool configured = false;
  if (!configured) {
    if (hipFuncSetAttribute((const void*)decode_split_kernel, hipFuncAttributeMaxDynamicSharedMemorySize,
                            kSplitLdsBytes) != hipSuccess)
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
  p.batch = a.batch;
  p.scale_log2 = a.softmax_scale * 1.4426950408889634f;
  const int n_hg = (a.h + kHeadsWG - 1) / kHeadsWG;
  const long long n_wg = (long long)a.plan.n_splits * a.n_blocks * n_hg * a.batch;
  if (n_wg <= 0 || n_wg > 0x7fffffffLL) return MLRA_ERR_SHAPE;
  decode_split_kernel<<<dim3((unsigned)n_wg), 512, kSplitLdsBytes, a.stream>>>(p);
  return check_launch();
}

}  // namespace mlra
