// MFMA decode kernel for the MLA comparison: one 512-dim latent plus a 64-dim RoPE key per token
// (Section 2.1, Steps 1-3 with d_c = 512; bf16 caches).
//
// One workgroup (4 wavefronts) owns one (sequence, context chunk, 64 query heads) and walks the chunk in
// tiles of 32 tokens [C | K^RoPE] that stream HBM -> LDS with direct-to-LDS loads, four stages deep
// (three tiles in flight while one is worked on).  The two products split the work differently:
//   * scores and softmax by heads: wave w owns heads [16 w, 16 w + 16) and computes their complete scores
//     S^T = [C | K^R] [q~ | q^R]^T over all 576 channels with 16x16x32 MFMAs (tokens x heads), so the
//     softmax of a head is computed once, by one wave, with its running maximum and sum in that wave;
//   * values by channels: wave w accumulates Z_w^T += C_w^T P^T for channels [128 w, 128 w + 128) and all
//     64 heads (32x32x16 MFMAs; C_w^T from LDS transpose reads of the same tile), so the 64 x 512
//     accumulator is spread over the four waves (128 registers each).
// Between the two, the probabilities P^T (bf16, 4 KiB per tile) go through LDS in the layout of the second
// product's B operand, together with the factors by which a wave lowered the weight of its heads'
// history when their running maximum grew (refreshed lazily, so almost always none).  Two workgroup
// barriers per tile: one hands the landed tile and the freed stage around, one publishes P^T.
// The two head halves of a sequence are placed on the same XCD (ids 8 apart), so the cache is fetched
// from HBM once.  Partials go to the workspace in the layout of the MLRA path with n_blocks = 1,
// d_cb = 512.
#include "mfma_tile.h"

namespace mlra {
namespace {

using namespace mfma_tile;

constexpr int kMDc = 512;                          // latent channels
constexpr int kMTok = 32;                          // tokens per tile
constexpr int kMHeads = 64;                        // query heads per workgroup
constexpr int kMLatBytes = kMTok * kMDc * 2;       // 32 KiB
constexpr int kMRopeBytes = kMTok * kDr * 2;       //  4 KiB
constexpr int kMStage = kMLatBytes + kMRopeBytes;  // 36 KiB
constexpr int kMStages = 4;
constexpr int kMPOff = kMStages * kMStage;         // P^T: [2 tiles][2 head tiles][2 token halves][64 lanes][16 B]
constexpr int kMPBytes = 4 * 1024;
constexpr int kMAOff = kMPOff + 2 * kMPBytes;      // rescale factors: [2 tiles][64 heads] floats, then [2][4] flags
constexpr int kMFOff = kMAOff + 2 * kMHeads * 4;
constexpr int kMLds = kMFOff + 2 * 4 * 4;          // 156,192 bytes
constexpr int kMLoads = 9;                         // direct-to-LDS loads per wave and tile

typedef const __attribute__((address_space(3))) bf16x8* lds_bf16x8_ptr;
typedef const __attribute__((address_space(3))) unsigned char* lds_byte_ptr;

// The four lanes c16, c16 + 16, c16 + 32, c16 + 48 hold parts of one head: these combine them in every
// lane without a trip through LDS.  v_permlane16_swap exchanges the odd 16-lane rows of its first operand
// with the even rows of its second, v_permlane32_swap the upper half of the first with the lower half of
// the second; applied to two copies of a value, every lane ends up with its own and its partner's.
__device__ __forceinline__ void row_pairs(float& a, float& b) {
  asm volatile("s_nop 1\n\tv_permlane16_swap_b32 %0, %1\n\ts_nop 1" : "+v"(a), "+v"(b));
}
__device__ __forceinline__ void half_pairs(float& a, float& b) {
  asm volatile("s_nop 1\n\tv_permlane32_swap_b32 %0, %1\n\ts_nop 1" : "+v"(a), "+v"(b));
}
__device__ __forceinline__ float head_max(float v) {
  float a = v, b = v;
  row_pairs(a, b);
  a = fmaxf(a, b);
  b = a;
  half_pairs(a, b);
  return fmaxf(a, b);
}
__device__ __forceinline__ float head_sum(float v) {
  float a = v, b = v;
  row_pairs(a, b);
  a += b;
  b = a;
  half_pairs(a, b);
  return a + b;
}

__global__ __launch_bounds__(256) void mla_mfma_kernel(MfmaParams p) {
  extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
  // workgroup -> (sequence, chunk, head half); the halves of one (sequence, chunk) get ids 8 apart
  const int n_hg = (p.h + kMHeads - 1) / kMHeads;
  const int n_units = p.n_splits * p.batch;
  const int full_units = n_units & ~7;
  int wg = blockIdx.x, su, hgrp;
  if (wg < full_units * n_hg) {
    const int r = wg >> 3;
    hgrp = r % n_hg;
    su = (r / n_hg) * 8 + (wg & 7);
  } else {
    wg -= full_units * n_hg;
    su = full_units + wg / n_hg;
    hgrp = wg % n_hg;
  }
  int split, seq, chunk_len;
  if (p.unit_tab) {            // chunk lengths follow the sequence lengths: active units listed first
    const int code = p.unit_tab[su];
    if (code < 0) return;
    seq = code >> 10;
    split = code & 1023;
    chunk_len = p.chunk_tab[seq];
  } else {
    split = su % p.n_splits;
    seq = p.seq_order ? p.seq_order[su / p.n_splits] : su / p.n_splits;
    chunk_len = p.chunk;
  }
  typedef const __attribute__((address_space(4))) int32_t* const_i32_ptr;
  const int n = ((const_i32_ptr)p.seq_lens)[seq];
  const int t0 = split * chunk_len;
  if (t0 >= n) return;
  const int t1 = min(n, t0 + chunk_len);
  const int ntiles = (t1 - t0 + kMTok - 1) / kMTok;
  const int nvalid_last = t1 - t0 - (ntiles - 1) * kMTok;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int g = lane >> 5, c32 = lane & 31;         // 32x32 MFMA roles (values)
  const int q4 = lane >> 4, c16 = lane & 15;        // 16x16 MFMA roles (scores)
  const int wave_u = __builtin_amdgcn_readfirstlane(wave);
  const unsigned lds_base = (unsigned)(size_t)(__attribute__((address_space(3))) unsigned char*)smem;
  const float sc = p.scale_log2;
  const int head_base = hgrp * kMHeads;

  // ---- this wave's 16 heads, complete: absorbed (512) and RoPE (64) query channels as B operands of the
  // 16x16x32 MFMA (lane: head c16, eight channels from 32 ks + 8 q4)
  bf16x8 qreg[18];
  {
    const int head = min(head_base + 16 * wave + c16, p.h - 1);
    const bf16_t* qa = p.q_abs + ((size_t)seq * p.h + head) * kMDc + q4 * 8;
    const bf16_t* qr = p.q_rope + ((size_t)seq * p.h + head) * kDr + q4 * 8;
#pragma unroll
    for (int ks = 0; ks < 16; ++ks) qreg[ks] = *(const bf16x8*)(qa + ks * 32);
    qreg[16] = *(const bf16x8*)qr;
    qreg[17] = *(const bf16x8*)(qr + 32);
  }
  // consumed here, before any direct-to-LDS load is in flight (a compiler-placed wait would drain them)
#pragma unroll
  for (int ks = 0; ks < 18; ++ks) asm volatile("" : "+v"(qreg[ks]));

  // ---- tile loads.  Latent rows are 1 KiB: one load moves one token row (lane i: 16-byte chunk i, i.e.
  // 256-byte sub-row i / 16, stored at chunk position (i % 16) ^ lat_swz(token) inside the sub-row);
  // wave w loads tokens 8w .. 8w+7 and RoPE rows 8w .. 8w+7 (one load).
  const const_i32_ptr pt_row = (const_i32_ptr)(p.page_table + (size_t)seq * p.max_pages);
  const size_t lat_page_bytes = (size_t)p.page_size * (kMDc * 2);
  const size_t rope_page_bytes = (size_t)p.page_size * (kDr * 2);
  unsigned lat_voff[8];
#pragma unroll
  for (int i = 0; i < 8; ++i)
    lat_voff[i] = (lane >> 4) * 256 + (((lane & 15) ^ lat_swz(8 * wave + i)) << 4);
  const int rope_t = 8 * wave + (lane >> 3);
  // A tile is issued in parts so that the parts can sit behind different MFMAs: issue_begin (scalar
  // address work), nine loads (0..7: latent rows, 8: the RoPE rows).
  const char* iss_lat = nullptr;
  const char* iss_rope = nullptr;
  unsigned iss_dst = 0;
  int iss_last = 0;
  auto issue_begin = [&](int jj) {
    const int tok = t0 + jj * kMTok;
    const unsigned page = (unsigned)pt_row[min(tok / p.page_size, p.max_pages - 1)];
    const int slot = tok % p.page_size;
    iss_lat = (const char*)p.latent + page * lat_page_bytes + (size_t)slot * (kMDc * 2);
    iss_rope = (const char*)p.rope + page * rope_page_bytes + (size_t)slot * (kDr * 2);
    iss_last = min(kMTok, t1 - tok) - 1;     // rows past it re-read it (finite values, weight 0 later)
    iss_dst = lds_base + (jj % kMStages) * kMStage;
  };
  auto issue_part = [&](int i) {
    if (i < 8) {
      const int t = 8 * wave_u + i;
      set_m0(iss_dst + t * 1024);
      lds_dma16<0>(iss_lat + (size_t)min(t, iss_last) * 1024, lat_voff[i]);
    } else {
      set_m0(iss_dst + kMLatBytes + wave_u * 1024);
      lds_dma16<0>(iss_rope, (unsigned)min(rope_t, iss_last) * (kDr * 2) + (((lane & 7) ^ rope_swz(rope_t)) << 4));
    }
  };
  auto issue_tile = [&](int jj) {
    issue_begin(jj);
#pragma unroll
    for (int i = 0; i < kMLoads; ++i) issue_part(i);
  };

  // ---- per-lane LDS read offsets inside a stage (XOR swizzle, see mfma_tile.h and decode_mfma.hip).
  // Scores, A operand of the 16x16x32 MFMA: lane = operand row c16 (+ 16 th) and eight channels from
  // 32 ks + 8 q4, i.e. 16-byte chunk 4 ks + q4 of the token row: sub-row ks / 4, chunk 4 (ks % 4) + q4.
  // A 128-bit LDS read is served sixteen lanes a cycle, and the sixteen are lanes 0-3, 12-15, 20-27 (then
  // 4-11, 16-19, 28-31; the same in the upper half): rows 4..11 of one chunk column meet rows 0-3 and 12-15
  // of the neighbouring column.  With operand row r holding token r ^ 8 (r in 4..7 or 12..15), i.e. rows
  // 4..11 = tokens 8..15, the chunk positions c ^ lat_swz(t) of such a group are all different (measured:
  // 4.6 instead of 8 cycles per read).  Output rows 4 q4 .. + 3 are then tokens 4 q4t .. + 3.
  const int k_tok = c16 ^ ((c16 & 4) << 1);
  const int q4t = q4 ^ ((q4 & 1) << 1);
  unsigned k_lat_off[2], k_rope_off[2];
#pragma unroll
  for (int th = 0; th < 2; ++th) {
    const int t = 16 * th + k_tok;
    k_lat_off[th] = t * 1024 + ((q4 ^ lat_swz(t)) << 4);                         // ^ ((ks % 4) << 6), + 256 (ks / 4)
    k_rope_off[th] = kMLatBytes + t * (kDr * 2) + ((q4 ^ rope_swz(t)) << 4);     // ^ (kr << 6)
  }
  unsigned v_off[2];                                                          // ^ (mt << 6), + 16 KiB ss
  {
    const int k = (lane & 15) >> 2, seg = lane & 3, hb = (lane >> 4) & 1;
#pragma unroll
    for (int half = 0; half < 2; ++half) {
      const int ta = 8 * half + 4 * g + k;
      v_off[half] = ta * 1024 + wave * 256 + (((2 * hb + (seg >> 1)) ^ lat_swz(ta)) << 4) + ((seg & 1) << 3);
    }
  }
  // P^T: the B operand (head tile w / 2, token half th) pairs with the transposed value operand, whose
  // lane group g holds tokens 4 g .. 4 g + 3 and 8 + 4 g .. 8 + 4 g + 3 of the 16.  This lane's four
  // probabilities (tokens 4 q4t .. + 3 of the half, head 16 w + c16) are therefore the first (q4t < 2) or
  // second four of lane n + 32 (q4t % 2), n = 16 (w % 2) + c16.
  const unsigned p_wr_off = (wave >> 1) * 2048 + (16 * (wave & 1) + c16 + 32 * (q4t & 1)) * 16 + (q4t >> 1) * 8;  // + 1024 th

  float m_run = kNegBig, l_run = 0.f;      // of head 16 w + c16 (the four lanes of a head hold equal m)
  f32x16 zacc[4][2];
#pragma unroll
  for (int mt = 0; mt < 4; ++mt)
#pragma unroll
    for (int nt = 0; nt < 2; ++nt)
#pragma unroll
      for (int i = 0; i < 16; ++i) zacc[mt][nt][i] = 0.f;

  for (int jj = 0; jj < kMStages - 1 && jj < ntiles; ++jj) issue_tile(jj);
  for (int j = 0; j < ntiles; ++j) {
    // tile j landed in this wave's share (the tiles issued after it may still be in flight) ...
    if (j + 2 < ntiles) wait_vm_lgkm<2 * kMLoads>();
    else if (j + 1 < ntiles) wait_vm_lgkm<kMLoads>();
    else wait_vm_lgkm<0>();
    // ... and in everybody's; every wave is also done with tile j-1, whose stage is refilled now
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
    const bool refill = j + kMStages - 1 < ntiles;     // its loads go out behind the value MFMAs below
    if (refill) issue_begin(j + kMStages - 1);
    const unsigned base = lds_base + (j % kMStages) * kMStage;
    const int par = j & 1;

    // ---- scores of this wave's 16 heads: 36 MFMAs, operand reads twelve ahead
    f32x4 s[2] = {{0.f, 0.f, 0.f, 0.f}, {0.f, 0.f, 0.f, 0.f}};
    {
      auto k_read = [&](int i) {     // i = 2 ks + th
        const int ks = i >> 1, th = i & 1;
        const unsigned addr = ks < 16 ? ((base + k_lat_off[th] + (ks >> 2) * 256) ^ ((ks & 3) << 6))
                                      : ((base + k_rope_off[th]) ^ ((ks - 16) << 6));
        return *(lds_bf16x8_ptr)(size_t)addr;
      };
      constexpr int kAhead = 12;
      bf16x8 ka[kAhead];
#pragma unroll
      for (int i = 0; i < kAhead; ++i) ka[i] = k_read(i);
#pragma unroll
      for (int i = 0; i < 36; ++i) {
        const bf16x8 cur = ka[i % kAhead];
        if (i + kAhead < 36) ka[i % kAhead] = k_read(i + kAhead);
        s[i & 1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(cur, qreg[i >> 1], s[i & 1], 0, 0, 0);
      }
    }

    // ---- softmax of the 16 heads (running maximum refreshed lazily, see decode_mfma.hip)
    float mx = fmaxf(fmaxf(fmaxf(s[0][0], s[0][1]), fmaxf(s[0][2], s[0][3])),
                     fmaxf(fmaxf(s[1][0], s[1][1]), fmaxf(s[1][2], s[1][3])));
    mx = head_max(mx);
    const float cand = mx * sc;
    const bool grow = cand > m_run + kLazy;
    const bool any_grow = __any(grow);
    float alpha = 1.f;
    if (any_grow) {
      const float m_new = grow ? cand : m_run;
      alpha = __builtin_amdgcn_exp2f(m_run - m_new);
      l_run *= alpha;
      m_run = m_new;
    }
    const int valid = (j == ntiles - 1) ? nvalid_last : kMTok;
    const float neg_m = -m_run;
#pragma unroll
    for (int th = 0; th < 2; ++th) {
      float pe[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        pe[i] = __builtin_amdgcn_exp2f(__builtin_fmaf(s[th][i], sc, neg_m));
        if (16 * th + 4 * q4t + i >= valid) pe[i] = 0.f;     // rows past a ragged end are copies of the last valid row
        l_run += pe[i];
      }
      typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
      const bf16x4 pk = {(__bf16)pe[0], (__bf16)pe[1], (__bf16)pe[2], (__bf16)pe[3]};
      *(bf16x4*)(smem + kMPOff + par * kMPBytes + th * 1024 + p_wr_off) = pk;
    }
    if (q4 == 0) ((float*)(smem + kMAOff))[par * kMHeads + 16 * wave + c16] = alpha;
    if (lane == 0) ((int*)(smem + kMFOff))[par * 4 + wave] = any_grow ? 1 : 0;

    // ---- the transposed value operands of this wave's channels do not depend on P^T: fetch them first
    bf16x8 va[2][4];
#pragma unroll
    for (int mt = 0; mt < 4; ++mt) {
      const lds_byte_ptr lo_p = (lds_byte_ptr)(size_t)((base + v_off[0]) ^ (mt << 6));
      const lds_byte_ptr hi_p = (lds_byte_ptr)(size_t)((base + v_off[1]) ^ (mt << 6));
#pragma unroll
      for (int ss = 0; ss < 2; ++ss) {
        const short4v lo = lds_tr16(lo_p + ss * 16 * 1024);
        const short4v hi = lds_tr16(hi_p + ss * 16 * 1024);
        va[ss][mt] = __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
      }
    }
    __syncthreads();     // P^T, the factors and the flags of every wave are visible

    // ---- a head's history loses weight when its maximum grew: the owner of the head said by how much
    {
      const int4 fl = *(const int4*)(smem + kMFOff + par * 16);
      if (__builtin_amdgcn_readfirstlane(fl.x | fl.y | fl.z | fl.w)) {
#pragma unroll
        for (int nt = 0; nt < 2; ++nt) {
          const float a_h = ((const float*)(smem + kMAOff))[par * kMHeads + nt * 32 + c32];
#pragma unroll
          for (int mt = 0; mt < 4; ++mt)
#pragma unroll
            for (int i = 0; i < 16; ++i) zacc[mt][nt][i] *= a_h;
        }
      }
    }
    // ---- values: Z_w^T += C_w^T P^T
    bf16x8 pb[2][2];
#pragma unroll
    for (int nt = 0; nt < 2; ++nt)
#pragma unroll
      for (int ss = 0; ss < 2; ++ss)
        pb[nt][ss] = *(const bf16x8*)(smem + kMPOff + par * kMPBytes + (nt * 2 + ss) * 1024 + lane * 16);
#pragma unroll
    for (int ss = 0; ss < 2; ++ss)
#pragma unroll
      for (int mt = 0; mt < 4; ++mt) {
        zacc[mt][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(va[ss][mt], pb[0][ss], zacc[mt][0], 0, 0, 0);
        zacc[mt][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(va[ss][mt], pb[1][ss], zacc[mt][1], 0, 0, 0);
        // the loads of tile j+3 into the stage tile j-1 left (free since the barrier at the top), one or
        // two behind each pair of MFMAs: the CU's address unit takes about 16 cycles per load
        if (refill) {
          const int k = ss * 4 + mt;       // 0..7
          issue_part(k);
          if (k == 7) issue_part(8);
        }
        __builtin_amdgcn_sched_barrier(0);
      }
  }

  // ---- write the chunk's partial: every wave its 128 channels of all 64 heads, and (m, l) of its 16 heads
  l_run = head_sum(l_run);
  const size_t unit = (size_t)seq * p.n_splits + split;
#pragma unroll
  for (int nt = 0; nt < 2; ++nt) {
    const int head = head_base + nt * 32 + c32;
    if (head < p.h) {
      float* dst = p.part_z + (unit * p.h + head) * kMDc + wave * 128 + g * 4;
#pragma unroll
      for (int mt = 0; mt < 4; ++mt)
#pragma unroll
        for (int r4 = 0; r4 < 4; ++r4) {
          const f32x4 v = {zacc[mt][nt][r4 * 4], zacc[mt][nt][r4 * 4 + 1], zacc[mt][nt][r4 * 4 + 2],
                           zacc[mt][nt][r4 * 4 + 3]};
          *(f32x4*)(dst + mt * 32 + r4 * 8) = v;
        }
    }
  }
  {
    const int head = head_base + 16 * wave + c16;
    if (q4 == 0 && head < p.h) {
      p.part_ml[(unit * p.h + head) * 2 + 0] = m_run;
      p.part_ml[(unit * p.h + head) * 2 + 1] = l_run;
    }
  }
}

}  // namespace

bool mla_mfma_supported(const DecodeArgs& a) {
  return a.dtype == MLRA_BF16 && a.n_blocks == 1 && a.d_cb == kMDc && a.d_r == kDr && a.page_size % kMTok == 0 &&
         a.plan.chunk_tokens % kMTok == 0;
}

int launch_mla_mfma(const DecodeArgs& a) {
  static PerDeviceSetup setup;
  int setup_dev = -1;
  if (setup.needed(&setup_dev)) {
    if (hipFuncSetAttribute((const void*)mla_mfma_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, kMLds) !=
        hipSuccess)
      return MLRA_ERR_LAUNCH;
    setup.done(setup_dev);
  }
  MfmaParams p;
  p.latent = (const bf16_t*)a.latent;
  p.rope = (const bf16_t*)a.rope;
  p.page_table = a.page_table;
  p.seq_lens = a.seq_lens;
  p.seq_order = nullptr;   // set below when the launch needs more than one round of workgroups
  p.chunk_tab = a.balanced ? a.chunk_tab : nullptr;
  p.unit_tab = a.balanced ? a.unit_tab : nullptr;
  p.q_abs = (const bf16_t*)a.q_abs;
  p.q_rope = (const bf16_t*)a.q_rope;
  p.part_z = a.part_z;
  p.part_ml = a.part_ml;
  p.page_size = a.page_size;
  p.max_pages = a.max_pages;
  p.n_blocks = 1;
  p.h = a.h;
  p.groups = a.groups;
  p.n_splits = a.plan.n_splits;
  p.chunk = a.plan.chunk_tokens;
  p.batch = a.batch;
  p.scale_log2 = softmax_scale_log2(a.softmax_scale);
  p.rows_bf16 = 0;
  const int n_hg = (a.h + kMHeads - 1) / kMHeads;
  const long long n_wg = (long long)a.plan.n_splits * n_hg * a.batch;
  if (n_wg <= 0 || n_wg > 0x7fffffffLL) return MLRA_ERR_SHAPE;
  if (!a.balanced && (n_wg > device_cu_count() || a.q_group > 1) && launch_seq_order(a) == MLRA_OK) p.seq_order = a.seq_order;
  MLRA_LAUNCH_TIMED(a.t_main, mla_mfma_kernel, dim3((unsigned)n_wg), dim3(256), kMLds, a.stream, p);
  return check_launch();
}

}  // namespace mlra
