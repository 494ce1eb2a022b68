// MFMA decode kernel for the MLA comparison: one 512-dim latent plus a 64-dim RoPE key per token
// (Section 2.1, Steps 1-3 with d_c = 512; bf16 caches).
//
// One workgroup (4 wavefronts) owns one (sequence, context chunk, 64 query heads) and walks the chunk in
// tiles of 32 tokens [C | K^RoPE] that stream HBM -> LDS with direct-to-LDS loads, three stages deep.
// The 512 latent channels are split over the waves: wave w owns channels [128 w, 128 w + 128).
//   * scores: wave w computes the partial S_w^T = C_w Q_w^T (+ one 16-dim slice of the RoPE product) for
//     all 32 tokens x 64 heads; the four partials are exchanged through LDS and every wave forms the same
//     full S^T (summed in one fixed order), the same running maxima and the same P^T (the softmax is recomputed four times rather
//     than exchanged once more: it is cheap next to the MFMAs);
//   * values: wave w accumulates Z_w^T += C_w^T P^T for its 128 channels, with C_w^T from LDS transpose
//     reads of the same tile, so the Z accumulators (128 registers) and the queries (72) fit one wave.
// Two workgroup barriers per tile order the loads, the stage reuse and the exchange buffer.  The two head
// halves of a sequence are placed on the same XCD (ids 8 apart), so the cache is fetched from HBM once.
// Partials go to the workspace in the layout of the MLRA path with n_blocks = 1, d_cb = 512.
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
constexpr int kMStages = 3;
constexpr int kMXOff = kMStages * kMStage;         // exchange buffer: [4 waves][8 operands][64 lanes][16 B]
constexpr int kMXWave = 8 * 1024;
constexpr int kMLds = kMXOff + 4 * kMXWave;        // 143,360 bytes
constexpr int kMLoads = 9;                         // direct-to-LDS loads per wave and tile

typedef const __attribute__((address_space(3))) bf16x8* lds_bf16x8_ptr;
typedef const __attribute__((address_space(3))) unsigned char* lds_byte_ptr;

__device__ __forceinline__ void swap_halves(float& a, float& b) {
  // exchanges the upper half of a with the lower half of b
  asm volatile("s_nop 1\n\tv_permlane32_swap_b32 %0, %1\n\ts_nop 1" : "+v"(a), "+v"(b));
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
  const int g = lane >> 5, c32 = lane & 31;
  const int wave_u = __builtin_amdgcn_readfirstlane(wave);
  const unsigned lds_base = (unsigned)(size_t)(__attribute__((address_space(3))) unsigned char*)smem;
  const float sc = p.scale_log2;
  const int head_base = hgrp * kMHeads;

  // ---- this wave's slice of the absorbed queries (128 of 512 channels) and of the RoPE queries (16 of 64
  // dims) as MFMA B operands
  bf16x8 qreg[2][9];
#pragma unroll
  for (int nt = 0; nt < 2; ++nt) {
    const int head = min(head_base + nt * 32 + c32, p.h - 1);
    const bf16_t* qa = p.q_abs + ((size_t)seq * p.h + head) * kMDc + wave * 128 + g * 8;
    const bf16_t* qr = p.q_rope + ((size_t)seq * p.h + head) * kDr + wave * 16 + g * 8;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) qreg[nt][ks] = *(const bf16x8*)(qa + ks * 16);
    qreg[nt][8] = *(const bf16x8*)qr;
  }
  // consumed here, before any direct-to-LDS load is in flight (a compiler-placed wait would drain them)
#pragma unroll
  for (int nt = 0; nt < 2; ++nt)
#pragma unroll
    for (int ks = 0; ks < 9; ++ks) asm volatile("" : "+v"(qreg[nt][ks]));

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
  auto issue_tile = [&](int jj, int stage) {
    const int tok = t0 + jj * kMTok;
    const unsigned page = (unsigned)pt_row[min(tok / p.page_size, p.max_pages - 1)];
    const int slot = tok % p.page_size;
    const char* lat_tile = (const char*)p.latent + page * lat_page_bytes + (size_t)slot * (kMDc * 2);
    const char* rope_tile = (const char*)p.rope + page * rope_page_bytes + (size_t)slot * (kDr * 2);
    const int last = min(kMTok, t1 - tok) - 1;     // rows past it re-read it (finite values, weight 0 later)
    const unsigned dst = lds_base + stage * kMStage;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int t = 8 * wave_u + i;
      set_m0(dst + t * 1024);
      lds_dma16<0>(lat_tile + (size_t)min(t, last) * 1024, lat_voff[i]);
    }
    set_m0(dst + kMLatBytes + wave_u * 1024);
    lds_dma16<0>(rope_tile, (unsigned)min(rope_t, last) * (kDr * 2) + (((lane & 7) ^ rope_swz(rope_t)) << 4));
  };

  // ---- per-lane LDS read offsets inside a stage (XOR swizzle, see mfma_tile.h and decode_mfma.hip)
  const unsigned k_lat_off = c32 * 1024 + wave * 256 + ((g ^ lat_swz(c32)) << 4);                       // ^ (ks << 5)
  const unsigned k_rope_off = kMLatBytes + c32 * (kDr * 2) + (((2 * wave + g) ^ rope_swz(c32)) << 4);
  unsigned v_off[2];                                                          // ^ (mt << 6), + 16 KiB ss
  {
    const int k = (lane & 15) >> 2, seg = lane & 3, hb = (lane >> 4) & 1;
#pragma unroll
    for (int half = 0; half < 2; ++half) {
      const int ta = 8 * half + 4 * g + k;
      v_off[half] = ta * 1024 + wave * 256 + (((2 * hb + (seg >> 1)) ^ lat_swz(ta)) << 4) + ((seg & 1) << 3);
    }
  }
  unsigned char* xbuf = smem + kMXOff;

  float m_run[2] = {kNegBig, kNegBig}, l_run[2] = {0.f, 0.f};
  f32x16 zacc[4][2];
#pragma unroll
  for (int mt = 0; mt < 4; ++mt)
#pragma unroll
    for (int nt = 0; nt < 2; ++nt)
#pragma unroll
      for (int i = 0; i < 16; ++i) zacc[mt][nt][i] = 0.f;

  for (int jj = 0; jj < kMStages - 1 && jj < ntiles; ++jj) issue_tile(jj, jj);
  int st_cur = 0;
  for (int j = 0; j < ntiles; ++j) {
    // tile j landed for every wave; everyone is done with tile j-1 (its stage, the exchange buffer)
    if (j + 1 < ntiles) wait_vm_lgkm<kMLoads>(); else wait_vm_lgkm<0>();
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
    const unsigned base = lds_base + st_cur * kMStage;

    // ---- partial scores over this wave's 128 channels and its RoPE slice
    f32x16 s[2];
#pragma unroll
    for (int nt = 0; nt < 2; ++nt)
#pragma unroll
      for (int i = 0; i < 16; ++i) s[nt][i] = 0.f;
    {
      bf16x8 ka[9];
#pragma unroll
      for (int ks = 0; ks < 8; ++ks) ka[ks] = *(lds_bf16x8_ptr)(size_t)((base + k_lat_off) ^ (ks << 5));
      ka[8] = *(lds_bf16x8_ptr)(size_t)(base + k_rope_off);
#pragma unroll
      for (int ks = 0; ks < 9; ++ks) {
        s[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka[ks], qreg[0][ks], s[0], 0, 0, 0);
        s[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka[ks], qreg[1][ks], s[1], 0, 0, 0);
        // keeps ka[0] alive past the two MFMAs whose accumulator input is the constant 0, so that the
        // allocator cannot place their destination on top of it (the build also scans for that)
        if (ks == 1) asm volatile("" : : "v"(ka[0]));
      }
    }
    // ---- while the matrix pipe works: loads of tile j+2 into the stage tile j-1 left (the CU's address
    // unit takes about 16 cycles per load), and the transposed value operands of this wave's channels
    __builtin_amdgcn_sched_barrier(0);
    if (j + kMStages - 1 < ntiles) issue_tile(j + kMStages - 1, (st_cur + kMStages - 1) % kMStages);
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
    __builtin_amdgcn_sched_barrier(0);
    // ---- exchange: own partial out, the other three in
#pragma unroll
    for (int nt = 0; nt < 2; ++nt)
#pragma unroll
      for (int r4 = 0; r4 < 4; ++r4) {
        const f32x4 v = {s[nt][r4 * 4], s[nt][r4 * 4 + 1], s[nt][r4 * 4 + 2], s[nt][r4 * 4 + 3]};
        *(f32x4*)(xbuf + wave * kMXWave + (nt * 4 + r4) * 1024 + lane * 16) = v;
      }
    __syncthreads();
    // every wave sums the four partials in the same order, so all four hold bit-identical S^T and take
    // identical softmax decisions
#pragma unroll
    for (int nt = 0; nt < 2; ++nt)
#pragma unroll
      for (int r4 = 0; r4 < 4; ++r4) {
        f32x4 acc = *(const f32x4*)(xbuf + (nt * 4 + r4) * 1024 + lane * 16);
#pragma unroll
        for (int w = 1; w < 4; ++w) {
          const f32x4 v = *(const f32x4*)(xbuf + w * kMXWave + (nt * 4 + r4) * 1024 + lane * 16);
          acc[0] += v[0]; acc[1] += v[1]; acc[2] += v[2]; acc[3] += v[3];
        }
        s[nt][r4 * 4] = acc[0];
        s[nt][r4 * 4 + 1] = acc[1];
        s[nt][r4 * 4 + 2] = acc[2];
        s[nt][r4 * 4 + 3] = acc[3];
      }

    // ---- online softmax (running maximum refreshed lazily, see decode_mfma.hip) and Z accumulation
    const int valid = (j == ntiles - 1) ? nvalid_last : kMTok;
    bf16x8 pb[2][2];
#pragma unroll
    for (int nt = 0; nt < 2; ++nt) {
      float mx = fmaxf(fmaxf(s[nt][0], s[nt][1]), s[nt][2]);
#pragma unroll
      for (int i = 3; i < 15; i += 2) mx = fmaxf(fmaxf(mx, s[nt][i]), s[nt][i + 1]);
      mx = fmaxf(mx, s[nt][15]);
      float mx2 = mx;
      swap_halves(mx, mx2);
      mx = fmaxf(mx, mx2);
      const float cand = mx * sc;
      if (__any(cand > m_run[nt] + kLazy)) {
        const float m_new = cand > m_run[nt] + kLazy ? cand : m_run[nt];
        const float alpha = __builtin_amdgcn_exp2f(m_run[nt] - m_new);
#pragma unroll
        for (int mt = 0; mt < 4; ++mt)
#pragma unroll
          for (int i = 0; i < 16; ++i) zacc[mt][nt][i] *= alpha;
        l_run[nt] *= alpha;
        m_run[nt] = m_new;
      }
      const float neg_m = -m_run[nt];
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const int tok = (i >> 2) * 8 + g * 4 + (i & 3);
        float pe = __builtin_amdgcn_exp2f(__builtin_fmaf(s[nt][i], sc, neg_m));
        if (tok >= valid) pe = 0.f;       // rows past a ragged end are copies of the last valid row
        l_run[nt] += pe;
        pb[nt][i >> 3][i & 7] = (__bf16)pe;
      }
    }
#pragma unroll
    for (int ss = 0; ss < 2; ++ss)
#pragma unroll
      for (int mt = 0; mt < 4; ++mt) {
        zacc[mt][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(va[ss][mt], pb[0][ss], zacc[mt][0], 0, 0, 0);
        zacc[mt][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(va[ss][mt], pb[1][ss], zacc[mt][1], 0, 0, 0);
      }
    st_cur = (st_cur + 1 == kMStages) ? 0 : st_cur + 1;
  }

  // ---- write the chunk's partial: every wave its 128 channels (the four waves hold identical m and l)
#pragma unroll
  for (int nt = 0; nt < 2; ++nt) {
    float l2 = l_run[nt];
    swap_halves(l_run[nt], l2);
    l_run[nt] += l2;
  }
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
      if (wave == 0 && g == 0) {
        p.part_ml[(unit * p.h + head) * 2 + 0] = m_run[nt];
        p.part_ml[(unit * p.h + head) * 2 + 1] = l_run[nt];
      }
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
  p.scale_log2 = a.softmax_scale * 1.4426950408889634f;
  const int n_hg = (a.h + kMHeads - 1) / kMHeads;
  const long long n_wg = (long long)a.plan.n_splits * n_hg * a.batch;
  if (n_wg <= 0 || n_wg > 0x7fffffffLL) return MLRA_ERR_SHAPE;
  if (!a.balanced && n_wg > device_cu_count() && launch_seq_order(a) == MLRA_OK) p.seq_order = a.seq_order;
  mla_mfma_kernel<<<dim3((unsigned)n_wg), 256, kMLds, a.stream>>>(p);
  return check_launch();
}

}  // namespace mlra
