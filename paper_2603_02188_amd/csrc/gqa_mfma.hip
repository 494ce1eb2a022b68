// MFMA decode kernel for the GQA comparison (Appendix C: MQA/GQA), bf16 K/V caches with d_h = 128 and at
// most 32 query heads per KV head.  GQA decode is bound by HBM alone (16 flop per cache byte), so the
// design aim is streaming, not matrix-pipe occupancy:
//   * one workgroup (4 wavefronts) per (sequence, KV head, context chunk);
//   * each wave runs a private pipeline over its own 32-token sub-tiles (sub-tile i goes to wave i % 4):
//     direct-to-LDS loads of K and V rows into a two-stage ring in the wave's quarter of LDS, waited for
//     with the wave's own vmcnt, so the loop has no workgroup barrier at all;
//   * scores transposed, S^T = K Q^T (tokens x heads, query heads padded to 32), so a lane owns one head
//     column; P^T rounded to bf16 is the B operand of O^T += V^T P^T, V^T through LDS transpose reads;
//   * the four waves' (m, l, O) are merged through LDS at the end and written as one partial per chunk
//     in the layout the generic GQA merge kernel reads.
#include "mfma_tile.h"

namespace mlra {
namespace {

using namespace mfma_tile;

constexpr int kGDh = 128;                       // head dimension
constexpr int kGTok = 32;                       // tokens per wave sub-tile
constexpr int kGHalf = kGTok * kGDh * 2;        // K (or V) rows of a sub-tile: 8 KiB
constexpr int kGStage = 2 * kGHalf;             // K + V
constexpr int kGWaveLds = 2 * kGStage;          // two stages per wave
constexpr int kGLds = 4 * kGWaveLds;            // 128 KiB
constexpr int kGLoads = 16;                     // direct-to-LDS loads per sub-tile
constexpr int kGPitch = kGDh + 4;               // floats per head row of the merge buffer

typedef const __attribute__((address_space(3))) bf16x8* lds_bf16x8_ptr;
typedef const __attribute__((address_space(3))) unsigned char* lds_byte_ptr;

struct GqaMfmaParams {
  const bf16_t* k_pool;
  const bf16_t* v_pool;
  const int32_t* page_table;
  const int32_t* seq_lens;
  const bf16_t* q;
  float* part_o;
  float* part_ml;
  int page_size, max_pages, h, g, n_splits, chunk;
  float scale_log2;
};

__device__ __forceinline__ void swap_halves(float& a, float& b) {
  // exchanges the upper half of a with the lower half of b
  asm volatile("s_nop 1\n\tv_permlane32_swap_b32 %0, %1\n\ts_nop 1" : "+v"(a), "+v"(b));
}

__global__ __launch_bounds__(256) void gqa_mfma_kernel(GqaMfmaParams p) {
  extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
  const int split = blockIdx.x, kvh = blockIdx.y, seq = blockIdx.z;
  const int r = p.h / p.g;                       // query heads per KV head (<= 32)
  typedef const __attribute__((address_space(4))) int32_t* const_i32_ptr;
  const int n = ((const_i32_ptr)p.seq_lens)[seq];
  const int t0 = split * p.chunk;
  if (t0 >= n) return;
  const int t1 = min(n, t0 + p.chunk);
  const int n_sub = (t1 - t0 + kGTok - 1) / kGTok;          // sub-tiles of this chunk
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int g = lane >> 5, c32 = lane & 31;
  const int wave_u = __builtin_amdgcn_readfirstlane(wave);   // wave-uniform copy: keeps tile addresses in SGPRs
  const unsigned lds_base = (unsigned)(size_t)(__attribute__((address_space(3))) unsigned char*)smem;
  const unsigned ring = lds_base + wave_u * kGWaveLds;
  const float sc = p.scale_log2;

  // queries of this KV head's group as MFMA B operands (zero for the padding heads)
  bf16x8 qreg[8];
  {
    const bf16_t* qrow = p.q + ((size_t)seq * p.h + kvh * r + min(c32, r - 1)) * kGDh + g * 8;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) {
      qreg[ks] = *(const bf16x8*)(qrow + ks * 16);
      if (c32 >= r) {
#pragma unroll
        for (int e = 0; e < 8; ++e) qreg[ks][e] = (__bf16)0.0f;
      }
    }
  }

  // ---- loads: a sub-tile is 32 K rows + 32 V rows of 256 bytes; load q covers rows 4q .. 4q+3 (lane i:
  // row 4q + i / 16, 16-byte chunk i % 16, stored swizzled as in mfma_tile.h)
  const const_i32_ptr pt_row = (const_i32_ptr)(p.page_table + (size_t)seq * p.max_pages);
  const size_t page_bytes = (size_t)p.g * p.page_size * (kGDh * 2);
  const size_t head_off = (size_t)kvh * p.page_size * (kGDh * 2);
  unsigned voff[4];
#pragma unroll
  for (int q = 0; q < 4; ++q) voff[q] = (lane >> 4) * (kGDh * 2) + (((lane & 15) ^ lat_swz(4 * q + (lane >> 4))) << 4);
  auto issue = [&](int sub, int stage) {
    const int tok = t0 + sub * kGTok;
    const unsigned page = (unsigned)pt_row[min(tok / p.page_size, p.max_pages - 1)];
    const size_t off = page * page_bytes + head_off + (size_t)(tok % p.page_size) * (kGDh * 2);
    const char* ksrc = (const char*)p.k_pool + off;
    const char* vsrc = (const char*)p.v_pool + off;
    const int last = min(kGTok, t1 - tok) - 1;
    const unsigned dst = ring + stage * kGStage;
    if (last == kGTok - 1) {
#pragma unroll
      for (int part = 0; part < 4; ++part) {      // K rows 0..15, K rows 16..31, V rows 0..15, V rows 16..31
        const char* src = (part < 2 ? ksrc : vsrc) + (part & 1) * 4096;
        set_m0(dst + part * 4096);
        lds_dma16<0>(src, voff[0]);
        lds_dma16<1024>(src, voff[1]);
        lds_dma16<2048>(src, voff[2]);
        lds_dma16<3072>(src, voff[3]);
      }
    } else {
      // ragged end of the chunk: rows past it re-read its last row (finite values, weight 0 later)
#pragma unroll
      for (int part = 0; part < 4; ++part) {
        const char* src = part < 2 ? ksrc : vsrc;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const int t = (part & 1) * 16 + 4 * q + (lane >> 4);      // 0..31
          const unsigned row = (unsigned)min(t, last);
          set_m0(dst + part * 4096 + q * 1024);
          lds_dma16<0>(src, row * (kGDh * 2) + (((lane & 15) ^ lat_swz(t)) << 4));
        }
      }
    }
  };

  // per-lane LDS read offsets inside a stage (see decode_mfma.hip)
  const unsigned k_off = c32 * (kGDh * 2) + ((g ^ lat_swz(c32)) << 4);           // ^ (ks << 5)
  unsigned v_off[2];                                                            // ^ (mt << 6), + 4096 ss
  {
    const int k = (lane & 15) >> 2, seg = lane & 3, hb = (lane >> 4) & 1;
#pragma unroll
    for (int half = 0; half < 2; ++half) {
      const int ta = 8 * half + 4 * g + k;
      v_off[half] = kGHalf + ta * (kGDh * 2) + (((2 * hb + (seg >> 1)) ^ lat_swz(ta)) << 4) + ((seg & 1) << 3);
    }
  }

  float m_run = kNegBig, l_run = 0.f;
  f32x16 zacc[4];
#pragma unroll
  for (int mt = 0; mt < 4; ++mt)
#pragma unroll
    for (int i = 0; i < 16; ++i) zacc[mt][i] = 0.f;

  int stage = 0;
  if (wave_u < n_sub) issue(wave_u, 0);
  for (int sub = wave_u; sub < n_sub; sub += 4) {
    // the other stage was last read one iteration ago; those reads returned before its MFMAs issued
    if (sub + 4 < n_sub) {
      issue(sub + 4, stage ^ 1);
      wait_vmcnt<kGLoads>();
    } else {
      wait_vmcnt<0>();
    }
    // the LDS reads below must stay behind the wait (the compiler does not know what the loads wrote)
    asm volatile("" ::: "memory");
    __builtin_amdgcn_sched_barrier(0);
    const unsigned base = ring + stage * kGStage;
    // scores S^T (32 tokens x 32 heads)
    f32x16 s;
#pragma unroll
    for (int i = 0; i < 16; ++i) s[i] = 0.f;
    bf16x8 ka[8];
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) ka[ks] = *(lds_bf16x8_ptr)(size_t)((base + k_off) ^ (ks << 5));
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) {
      s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka[ks], qreg[ks], s, 0, 0, 0);
      // keeps ka[0] alive past the MFMA whose accumulator input is the constant 0, so that the allocator
      // cannot place its destination on top of it (the build also scans for that)
      if (ks == 1) asm volatile("" : : "v"(ka[0]));
    }
    // transposed V operands
    bf16x8 va[2][4];
#pragma unroll
    for (int mt = 0; mt < 4; ++mt) {
      const lds_byte_ptr lo_p = (lds_byte_ptr)(size_t)((base + v_off[0]) ^ (mt << 6));
      const lds_byte_ptr hi_p = (lds_byte_ptr)(size_t)((base + v_off[1]) ^ (mt << 6));
#pragma unroll
      for (int ss = 0; ss < 2; ++ss) {
        const short4v lo = lds_tr16(lo_p + ss * 16 * (kGDh * 2));
        const short4v hi = lds_tr16(hi_p + ss * 16 * (kGDh * 2));
        va[ss][mt] = __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
      }
    }
    // column maxima (rows past a ragged end are copies of the last valid row, so they do not disturb it)
    float mx = fmaxf(fmaxf(s[0], s[1]), s[2]);
#pragma unroll
    for (int i = 3; i < 15; i += 2) mx = fmaxf(fmaxf(mx, s[i]), s[i + 1]);
    mx = fmaxf(mx, s[15]);
    float mx2 = mx;
    swap_halves(mx, mx2);               // mx = {lower, lower}, mx2 = {upper, upper}
    mx = fmaxf(mx, mx2);
    const float m_new = fmaxf(m_run, mx * sc);
    const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);
    m_run = m_new;
    l_run *= alpha;
#pragma unroll
    for (int mt = 0; mt < 4; ++mt)
#pragma unroll
      for (int i = 0; i < 16; ++i) zacc[mt][i] *= alpha;
    const int valid = min(kGTok, t1 - (t0 + sub * kGTok));
    bf16x8 pb[2];
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const int tok = (i >> 2) * 8 + g * 4 + (i & 3);
      float pe = __builtin_amdgcn_exp2f(__builtin_fmaf(s[i], sc, -m_new));
      if (tok >= valid) pe = 0.f;
      l_run += pe;
      pb[i >> 3][i & 7] = (__bf16)pe;
    }
#pragma unroll
    for (int ss = 0; ss < 2; ++ss)
#pragma unroll
      for (int mt = 0; mt < 4; ++mt)
        zacc[mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(va[ss][mt], pb[ss], zacc[mt], 0, 0, 0);
    stage ^= 1;
  }

  // ---- merge the four waves' (m, l, O) through LDS and write the chunk's partial ----
  {
    float l2 = l_run;
    swap_halves(l_run, l2);             // l_run = {lower, lower}, l2 = {upper, upper}
    l_run += l2;
  }
  __syncthreads();                      // every wave is done with its ring
  float* mbuf = (float*)smem;           // [4][32]
  float* lbuf = mbuf + 128;             // [4][32]
  float* zbuf = (float*)(smem + 1024);  // [4 waves][32 heads][kGPitch]
  if (g == 0) {
    mbuf[wave * 32 + c32] = m_run;
    lbuf[wave * 32 + c32] = l_run;
  }
  __syncthreads();
  float m_star = mbuf[c32];
#pragma unroll
  for (int w = 1; w < 4; ++w) m_star = fmaxf(m_star, mbuf[w * 32 + c32]);
  const float w_own = __builtin_amdgcn_exp2f(m_run - m_star);
#pragma unroll
  for (int mt = 0; mt < 4; ++mt)
#pragma unroll
    for (int r4 = 0; r4 < 4; ++r4) {
      f32x4 v = {zacc[mt][r4 * 4] * w_own, zacc[mt][r4 * 4 + 1] * w_own, zacc[mt][r4 * 4 + 2] * w_own,
                 zacc[mt][r4 * 4 + 3] * w_own};
      *(f32x4*)(zbuf + (wave * 32 + c32) * kGPitch + mt * 32 + r4 * 8 + g * 4) = v;
    }
  __syncthreads();
  const size_t unit = (size_t)seq * p.n_splits + split;
  for (int idx = tid; idx < r * (kGDh / 4); idx += 256) {
    const int hh = idx / (kGDh / 4), f4 = idx % (kGDh / 4);
    f32x4 acc = *(const f32x4*)(zbuf + hh * kGPitch + f4 * 4);
#pragma unroll
    for (int w = 1; w < 4; ++w) {
      const f32x4 v = *(const f32x4*)(zbuf + (w * 32 + hh) * kGPitch + f4 * 4);
      acc[0] += v[0]; acc[1] += v[1]; acc[2] += v[2]; acc[3] += v[3];
    }
    *(f32x4*)(p.part_o + (unit * p.h + kvh * r + hh) * kGDh + f4 * 4) = acc;
  }
  if (tid < r) {
    float ms = mbuf[tid];
#pragma unroll
    for (int w = 1; w < 4; ++w) ms = fmaxf(ms, mbuf[w * 32 + tid]);
    float L = 0.f;
#pragma unroll
    for (int w = 0; w < 4; ++w) L += lbuf[w * 32 + tid] * __builtin_amdgcn_exp2f(mbuf[w * 32 + tid] - ms);
    p.part_ml[(unit * p.h + kvh * r + tid) * 2 + 0] = ms;
    p.part_ml[(unit * p.h + kvh * r + tid) * 2 + 1] = L;
  }
}

}  // namespace

bool gqa_mfma_supported(const GqaArgs& a) {
  return a.dtype == MLRA_BF16 && a.d_h == kGDh && a.h % a.g == 0 && a.h / a.g <= 32 && a.page_size % kGTok == 0 &&
         a.plan.chunk_tokens % kGTok == 0 && a.g <= 65535;
}

int launch_gqa_mfma(const GqaArgs& a) {
  static PerDeviceSetup setup;
  int setup_dev = -1;
  if (setup.needed(&setup_dev)) {
    if (hipFuncSetAttribute((const void*)gqa_mfma_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, kGLds) !=
        hipSuccess)
      return MLRA_ERR_LAUNCH;
    setup.done(setup_dev);
  }
  GqaMfmaParams p;
  p.k_pool = (const bf16_t*)a.k_pool;
  p.v_pool = (const bf16_t*)a.v_pool;
  p.page_table = a.page_table;
  p.seq_lens = a.seq_lens;
  p.q = (const bf16_t*)a.q;
  p.part_o = a.part_o;
  p.part_ml = a.part_ml;
  p.page_size = a.page_size;
  p.max_pages = a.max_pages;
  p.h = a.h;
  p.g = a.g;
  p.n_splits = a.plan.n_splits;
  p.chunk = a.plan.chunk_tokens;
  p.scale_log2 = a.softmax_scale * 1.4426950408889634f;
  dim3 grid(a.plan.n_splits, a.g, a.batch);
  gqa_mfma_kernel<<<grid, 256, kGLds, a.stream>>>(p);
  return check_launch();
}

}  // namespace mlra
