// Pre-attention of the new token of every sequence (Section 2.1; Appendix C, subsection "Multi-Head Latent Attention (MLA)", the form MLRA
// keeps; scaling factors of Eq. (9)):
//   C^Q  = alpha_q  RMSNorm(H W^DQ),   Q^NoPE = C^Q W^UQ,   Q^RoPE = RoPE(C^Q W^QR)
//   C^KV = alpha_kv RMSNorm(H W^DKV),  K^RoPE = RoPE(H W^KR);   C^KV and K^RoPE go into the cache.
// With one token per sequence these are matrix products with a handful of rows (the batch) against
// weights that have to be streamed from HBM once, so the work is organised around the weights:
//   1. skinny GEMM  H [B][d] x [W^DQ | W^DKV | W^KR]           -> fp32 partial sums per K slice
//   2. finish:      sum the slices, RMSNorm + scaling, RoPE, store C^Q (cache dtype) and the cache row
//   3. skinny GEMM  C^Q [B][d_cq] x [W^UQ | W^QR]              -> fp32 partial sums per K slice
//   4. finish:      sum the slices, RoPE on the RoPE part, store q_nope and q_rope
// The bf16 GEMM runs on MFMA with the batch as the M dimension; the weights pass through LDS 128 rows at
// a time and reach the B operand through transpose reads.  Other dtypes and odd shapes use a plain kernel.
#include "mlra_internal.h"
#include "mfma_tile.h"

namespace mlra {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) short short4v;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;

constexpr int kColsWG = 128;     // output columns per workgroup (32 per wave)
constexpr int kRowsChunk = 128;  // weight rows per LDS stage (32 KiB)
constexpr int kMaxMTiles = 4;    // 32-row tiles of the batch held in accumulators at once
constexpr int kWBytes = kRowsChunk * 256;                 // weight tile of a stage
__host__ __device__ constexpr int gemm_stage_bytes(int mt) { return kWBytes + 32 * mt * (kRowsChunk * 2); }
__host__ __device__ constexpr int gemm_stages(int mt) { return mt <= 2 ? 3 : 2; }   // what fits 160 KiB

__device__ __forceinline__ int swz(int t) { return ((t & 3) << 1) | ((t >> 2) & 1); }

__device__ __forceinline__ short4v lds_tr16(const void* p) {
  return __builtin_amdgcn_ds_read_tr16_b64_v4i16((short4v __attribute__((address_space(3)))*)p);
}

// out_part[slice][m][col0 + j] = sum_{k in slice} A[m][k] W[k][j] for the workgroup's column tile.
// Column tiles are numbered over the segments side by side; a segment narrower than its last tile
// repeats valid columns in the padding (never stored).  K and the slice length are multiples of
// kRowsChunk.  Chunks of 128 weight rows (32 KiB) and the matching 128 columns of the A rows stream
// HBM -> LDS with direct-to-LDS loads through a ring of stages: while one chunk is multiplied the
// following one or two are in flight, and nothing passes through registers on the way.  16-byte chunk c
// of weight row r sits at chunk position c ^ swz(r & 7) of its 256-byte LDS row (what the transpose
// reads want), chunk c of A row r at c ^ (r & 15) (so that the 16 lanes a 128-bit read serves together
// hit 16 different bank groups).
// Rotation of the 2-D block (x0, x1) by the angle of (position, frequency index l) held as (cos, sin).
__device__ __forceinline__ void rotate(float x0, float x1, float c, float s, float& y0, float& y1) {
  y0 = x0 * c - x1 * s;
  y1 = x0 * s + x1 * c;
}

// Epilogue of the query up-projection when K is not cut into slices (nothing is left to sum): segment 0
// (W^UQ) leaves as q_nope, segment 1 (W^QR) is rotated (RoPE, angles from the table that the
// down-projection's finishing kernel wrote) and leaves as q_rope, both in the storage dtype.
struct GemmFinishUp {
  const float* cs_tab;   // [M][d_r / 2] (cos, sin)
  bf16_t* q_nope;        // [M][cols of segment 0]
  bf16_t* q_rope;        // [M][cols of segment 1]
  int d_r;
};

template <int MT, bool FINISH_UP>   // MT: 32-row tiles of A per workgroup (1..kMaxMTiles)
__global__ __launch_bounds__(256) void skinny_gemm_mfma_kernel(const bf16_t* __restrict__ A, int lda, int M,
                                                               GemmSegments segs, int K, int rows_per_slice,
                                                               float* __restrict__ out_part, int ld_out,
                                                               GemmFinishUp fin) {
  extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
  constexpr int kStages = gemm_stages(MT);
  constexpr int kStageB = gemm_stage_bytes(MT);
  constexpr int kALoads = 2 * MT;                 // direct-to-LDS loads per wave and chunk: A rows ...
  constexpr int kLoads = 8 + kALoads;             // ... and 8 for the weights
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, g = lane >> 5, c32 = lane & 31;
  // column tile -> segment
  int tile = blockIdx.x, seg = 0;
  while (seg < segs.count - 1 && tile >= (segs.cols[seg] + kColsWG - 1) / kColsWG) {
    tile -= (segs.cols[seg] + kColsWG - 1) / kColsWG;
    ++seg;
  }
  const unsigned char* Wb = (const unsigned char*)segs.w[seg];
  const unsigned char* Ab = (const unsigned char*)A;
  const int ldw = segs.cols[seg], n0 = tile * kColsWG;
  const int out_col0 = segs.out_col[seg] + n0;
  const int n_valid = min(kColsWG, ldw - n0);          // multiple of 8
  const int slice = blockIdx.y;
  const int k_begin = slice * rows_per_slice, k_end = min(K, k_begin + rows_per_slice);
  const int n_chunks = (k_end - k_begin) / kRowsChunk;
  const int m_base = blockIdx.z * (32 * MT);   // (rows past M repeat row M - 1 and are never stored)
  if (n_chunks <= 0) return;

  // Per-lane source offsets inside a chunk (byte offsets fit 32 bits: checked by the launcher).  A load
  // fills 1 KiB of LDS = 4 rows x 16 chunks; lane l lands at row l / 16, chunk position l % 16, so it
  // fetches the chunk that the swizzle puts there.  Wave w moves weight rows [32 w, 32 w + 32) and A rows
  // [8 MT w, 8 MT w + 8 MT).
  const unsigned lds_base = (unsigned)(size_t)(__attribute__((address_space(3))) unsigned char*)smem;
  const unsigned wave_u = __builtin_amdgcn_readfirstlane(wave);
  unsigned w_voff[8], a_voff[kALoads];
#pragma unroll
  for (int q = 0; q < 8; ++q) {
    const int row = 32 * wave + 4 * q + (lane >> 4);
    const int col = min(n0 + (((lane & 15) ^ swz(row & 7)) << 3), ldw - 8);
    w_voff[q] = (unsigned)(row * ldw + col) * 2u;
  }
#pragma unroll
  for (int q = 0; q < kALoads; ++q) {
    const int row = 8 * MT * wave + 4 * q + (lane >> 4);
    a_voff[q] = (unsigned)(min(m_base + row, M - 1) * lda + (((lane & 15) ^ (row & 15)) << 3)) * 2u;
  }
  // chunk ci of the slice -> stage ci % kStages (chunks past the slice re-read its last chunk: the
  // number of loads per step stays fixed, which the wait counts below rely on; nobody reads them)
  int issue_stage = 0;
  auto issue = [&](int ci) {
    const int k0 = k_begin + min(ci, n_chunks - 1) * kRowsChunk;
    const unsigned char* wsrc = Wb + (size_t)k0 * ldw * 2;
    const unsigned char* asrc = Ab + (size_t)k0 * 2;
    const unsigned st = lds_base + issue_stage * kStageB;
#pragma unroll
    for (int q = 0; q < 8; ++q) {
      mfma_tile::set_m0(st + (wave_u * 8 + q) * 1024);
      mfma_tile::lds_dma16<0>(wsrc, w_voff[q]);
    }
#pragma unroll
    for (int q = 0; q < kALoads; ++q) {
      mfma_tile::set_m0(st + kWBytes + (wave_u * kALoads + q) * 1024);
      mfma_tile::lds_dma16<0>(asrc, a_voff[q]);
    }
    issue_stage = (issue_stage + 1 == kStages) ? 0 : issue_stage + 1;
  };

  // transpose-read offsets: the 16 lanes of a block fetch 4 consecutive rows x 16 output columns
  unsigned tr_off[2];
  {
    const int k = (lane & 15) >> 2, sg = lane & 3, hb = (lane >> 4) & 1;
#pragma unroll
    for (int half = 0; half < 2; ++half) {
      const int row = 8 * g + 4 * half + k;                 // + 16 per MFMA k-step (same swizzle: row & 7)
      const int c16 = 4 * wave + 2 * hb + (sg >> 1);
      tr_off[half] = row * 256 + ((c16 ^ swz(row & 7)) << 4) + ((sg & 1) << 3);
    }
  }
  f32x16 acc[MT];
  {
    float z = 0.f;
    asm volatile("" : "+v"(z));   // a register zero: every MFMA below is emitted in the tied form
#pragma unroll
    for (int t = 0; t < MT; ++t)
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[t][i] = z;
  }

  // all 8 k-steps of a chunk, straight-line so that the LDS reads of later steps are issued ahead of
  // the MFMAs of earlier ones
  auto multiply = [&](const unsigned char* wt) {
    const unsigned char* at = wt + kWBytes;
#pragma unroll
    for (int ks = 0; ks < kRowsChunk / 16; ++ks) {
      const short4v lo = lds_tr16(wt + ks * 16 * 256 + tr_off[0]);
      const short4v hi = lds_tr16(wt + ks * 16 * 256 + tr_off[1]);
      const bf16x8 bm = __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
#pragma unroll
      for (int t = 0; t < MT; ++t) {
        const int row = t * 32 + c32;
        const bf16x8 a = *(const bf16x8*)(at + row * 256 + (((2 * ks + g) ^ (row & 15)) << 4));
        acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, bm, acc[t], 0, 0, 0);
      }
    }
  };
#pragma unroll
  for (int ci = 0; ci < kStages - 1; ++ci) issue(ci);
  int st = 0;
  for (int ci = 0; ci < n_chunks; ++ci) {
    // chunk ci has landed in this wave's share (the chunks issued after it may still be in flight) ...
    mfma_tile::wait_vmcnt<kLoads * (kStages - 2)>();
    // ... and in everybody's; every wave is also done with chunk ci - 1, whose stage is refilled now
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
    issue(ci + kStages - 1);
    multiply(smem + st * kStageB);
    asm volatile("" ::: "memory");
    st = (st + 1 == kStages) ? 0 : st + 1;
  }
  mfma_tile::wait_vmcnt<0>();   // the loads past the slice target this workgroup's LDS: let them land
  const int j = wave * 32 + c32;
  if (FINISH_UP) {
    // The tile's sums go through LDS (the stages are free now) so that a thread finishes eight neighbouring
    // columns of a row: four RoPE 2-D blocks [2l, 2l+1] with their angles side by side in the table, one
    // 16-byte store.
    constexpr int kPitch = kColsWG + 4;          // floats per staged row (+4: rows start on different banks)
    float* tile = (float*)smem;
    __syncthreads();                             // every wave is past its last read of the stages
#pragma unroll
    for (int t = 0; t < MT; ++t)
#pragma unroll
      for (int r = 0; r < 16; ++r)
        tile[(t * 32 + (r >> 2) * 8 + g * 4 + (r & 3)) * kPitch + j] = acc[t][r];
    __syncthreads();
    bf16_t* dst = seg == 0 ? fin.q_nope : fin.q_rope;
    for (int id = tid; id < 32 * MT * (kColsWG / 8); id += 256) {
      const int row = id / (kColsWG / 8), pc = id % (kColsWG / 8), m = m_base + row, col = n0 + pc * 8;
      if (m >= M || pc * 8 >= n_valid) continue;
      const f32x4 lo = *(const f32x4*)(tile + row * kPitch + pc * 8), hi = *(const f32x4*)(tile + row * kPitch + pc * 8 + 4);
      float v[8] = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
      if (seg != 0) {
        const int l0 = (col % fin.d_r) >> 1;     // d_r is a multiple of 8: the four blocks share the head
        const float* cs = fin.cs_tab + ((size_t)m * (fin.d_r / 2) + l0) * 2;
        const f32x4 c01 = *(const f32x4*)cs, c23 = *(const f32x4*)(cs + 4);
        const float cv[4] = {c01[0], c01[2], c23[0], c23[2]}, sv[4] = {c01[1], c01[3], c23[1], c23[3]};
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          float y0, y1;
          rotate(v[2 * q], v[2 * q + 1], cv[q], sv[q], y0, y1);
          v[2 * q] = y0;
          v[2 * q + 1] = y1;
        }
      }
      bf16x8 packed;
#pragma unroll
      for (int e = 0; e < 8; ++e) packed[e] = (__bf16)v[e];
      *(bf16x8*)(dst + (size_t)m * ldw + col) = packed;
    }
  } else if (j < n_valid) {
#pragma unroll
    for (int t = 0; t < MT; ++t) {
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int m = m_base + t * 32 + (r >> 2) * 8 + g * 4 + (r & 3);
        if (m < M) out_part[((size_t)slice * M + m) * ld_out + out_col0 + j] = acc[t][r];
      }
    }
  }
}

// Any dtype / shape: one thread per output element, fp32 accumulation, a single K slice.
template <typename T>
__global__ void skinny_gemm_generic_kernel(const T* __restrict__ A, int lda, int M, GemmSegments segs, int K,
                                           float* __restrict__ out_part, int ld_out, int n_total) {
  const int col = blockIdx.x * blockDim.x + threadIdx.x, m = blockIdx.y;
  if (col >= n_total) return;
  int seg = 0, j = col;
  while (seg < segs.count - 1 && j >= segs.cols[seg]) { j -= segs.cols[seg]; ++seg; }
  const T* W = (const T*)segs.w[seg];
  const int ldw = segs.cols[seg];
  float acc = 0.f;
  for (int k = 0; k < K; ++k) acc += load_f32(A, (size_t)m * lda + k) * load_f32(W, (size_t)k * ldw + j);
  out_part[(size_t)m * ld_out + segs.out_col[seg] + j] = acc;
}

__device__ __forceinline__ float block_sum(float v, float* red) {
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  __syncthreads();
  if (lane == 0) red[wave] = v;
  __syncthreads();
  float s = 0.f;
  for (int w = 0; w < (int)(blockDim.x >> 6); ++w) s += red[w];
  return s;
}


// Step 2.  One workgroup per sequence.  Columns of the summed down-projection: [0, d_cq) C^Q,
// [d_cq, d_cq + d_c) C^KV, then d_r RoPE-key channels.
template <typename T, typename TC>
__global__ __launch_bounds__(256) void pre_finish_down_kernel(
    const float* __restrict__ part, int n_slices, int batch, int d_cq, int d_c, int d_r, int n_blocks,
    const T* __restrict__ gain_q, const T* __restrict__ gain_kv, float alpha_q, float alpha_kv, float eps,
    float rope_base, const int32_t* __restrict__ positions, const int32_t* __restrict__ page_table, int max_pages,
    int page_size, T* __restrict__ c_q, TC* __restrict__ latent, TC* __restrict__ rope_pool,
    float* __restrict__ cs_tab) {
  extern __shared__ float row[];             // [d_cq + d_c + d_r] summed projections
  __shared__ float red[4];
  __shared__ float cs_sh[256];               // (cos, sin) per RoPE frequency of this sequence's position
  const int s = blockIdx.x, tid = threadIdx.x;
  const int n1 = d_cq + d_c + d_r;
  const int pos = positions[s];
  float ss_q = 0.f, ss_kv = 0.f;
  // kU columns per thread and kKK slices at a time, all loads of such a round in flight together: the
  // kernel is a chain of memory round trips (one workgroup per sequence), so it wants as few rounds as
  // possible (the benchmark shape, 2112 columns in 14 slices, takes one)
  constexpr int kU = 9, kKK = 16;
  for (int j0 = 0; j0 < n1; j0 += kU * 256) {
    float v[kU];
#pragma unroll
    for (int u = 0; u < kU; ++u) v[u] = 0.f;
    for (int k = 0; k < n_slices; k += kKK) {
      float t[kKK][kU];
#pragma unroll
      for (int kk = 0; kk < kKK; ++kk) {
        const float* src = part + ((size_t)min(k + kk, n_slices - 1) * batch + s) * n1;
#pragma unroll
        for (int u = 0; u < kU; ++u) t[kk][u] = src[min(j0 + u * 256 + tid, n1 - 1)];   // unconditional: all in flight
      }
#pragma unroll
      for (int kk = 0; kk < kKK; ++kk)
#pragma unroll
        for (int u = 0; u < kU; ++u) v[u] += (k + kk < n_slices) ? t[kk][u] : 0.f;   // slices summed in order
    }
#pragma unroll
    for (int u = 0; u < kU; ++u) {
      const int j = j0 + u * 256 + tid;
      if (j < n1) {
        row[j] = v[u];
        if (j < d_cq) ss_q += v[u] * v[u];
        else if (j < d_cq + d_c) ss_kv += v[u] * v[u];
      }
    }
  }
  ss_q = block_sum(ss_q, red);
  ss_kv = block_sum(ss_kv, red);
  const float rq = alpha_q * rsqrtf(ss_q / d_cq + eps), rkv = alpha_kv * rsqrtf(ss_kv / d_c + eps);
  // cos / sin of position * theta_l.  Positions reach 10^5 and beyond, so the product and its reduction
  // to [-pi, pi] are done in double (a float angle would be off by ~1e-2 rad there); the reduced angle is
  // then accurate to ~1e-11 and float sine / cosine of it are good to a few ulp.
  if (tid < d_r / 2) {
    const double theta = exp2(-2.0 * tid / d_r * log2((double)rope_base));
    const double ang = (double)max(pos, 0) * theta;
    const double two_pi = 6.283185307179586476925287;
    const float red_ang = (float)(ang - two_pi * rint(ang / two_pi));
    float sn, cs;
    sincosf(red_ang, &sn, &cs);
    cs_sh[2 * tid] = (float)cs;
    cs_sh[2 * tid + 1] = (float)sn;
    cs_tab[((size_t)s * (d_r / 2) + tid) * 2 + 0] = (float)cs;   // for the query side (step 4)
    cs_tab[((size_t)s * (d_r / 2) + tid) * 2 + 1] = (float)sn;
  }
  for (int j = tid; j < d_cq; j += 256)
    store_f32(c_q, (size_t)s * d_cq + j, row[j] * rq * (gain_q ? load_f32(gain_q, j) : 1.f));
  if (pos < 0) return;                        // no cache row for this sequence (as in mlra_append_kv)
  const int page = page_table[(size_t)s * max_pages + pos / page_size], slot = pos % page_size;
  const int d_cb = d_c / n_blocks;
  for (int j = tid; j < d_c; j += 256) {
    const int b = j / d_cb, c = j % d_cb;
    const float v = row[d_cq + j] * rkv * (gain_kv ? load_f32(gain_kv, j) : 1.f);
    store_f32(latent, (((size_t)page * n_blocks + b) * page_size + slot) * d_cb + c, v);
  }
  __syncthreads();   // cs_sh is complete
  for (int l = tid; l < d_r / 2; l += 256) {
    const float c = cs_sh[2 * l], sn = cs_sh[2 * l + 1];
    float y0, y1;
    rotate(row[d_cq + d_c + 2 * l], row[d_cq + d_c + 2 * l + 1], c, sn, y0, y1);
    store_f32(rope_pool, ((size_t)page * page_size + slot) * d_r + 2 * l, y0);
    store_f32(rope_pool, ((size_t)page * page_size + slot) * d_r + 2 * l + 1, y1);
  }
}

// Step 4.  Columns of the summed up-projection: [0, h d_h) Q^NoPE, then h d_r RoPE-query channels.
template <typename T>
__global__ __launch_bounds__(256) void pre_finish_up_kernel(const float* __restrict__ part, int n_slices, int batch,
                                                            int h, int d_h, int d_r,
                                                            const float* __restrict__ cs_tab, T* __restrict__ q_nope,
                                                            T* __restrict__ q_rope) {
  const int s = blockIdx.y;
  const int n2 = h * (d_h + d_r), n_nope = h * d_h;
  // one thread per pair of neighbouring columns (a RoPE 2-D block never straddles two threads)
  const int pair = blockIdx.x * 256 + threadIdx.x;
  if (2 * pair >= n2) return;
  float v0 = 0.f, v1 = 0.f;
  for (int k = 0; k < n_slices; ++k) {
    const float2 p = *(const float2*)(part + ((size_t)k * batch + s) * n2 + 2 * pair);
    v0 += p.x;
    v1 += p.y;
  }
  if (2 * pair < n_nope) {
    store_f32(q_nope, (size_t)s * n_nope + 2 * pair, v0);
    store_f32(q_nope, (size_t)s * n_nope + 2 * pair + 1, v1);
  } else {
    const int j = 2 * pair - n_nope, l = (j % d_r) / 2;
    const float c = cs_tab[((size_t)s * (d_r / 2) + l) * 2], sn = cs_tab[((size_t)s * (d_r / 2) + l) * 2 + 1];
    float y0, y1;
    rotate(v0, v1, c, sn, y0, y1);
    store_f32(q_rope, (size_t)s * h * d_r + j, y0);
    store_f32(q_rope, (size_t)s * h * d_r + j + 1, y1);
  }
}

bool gemm_mfma_ok(int dtype, int M, int K, int lda, const GemmSegments& segs) {
  if (dtype != MLRA_BF16 || K % kRowsChunk != 0 || lda % 8 != 0) return false;
  const long long lim = 1ll << 30;   // elements: byte offsets stay below 2^31
  if ((long long)M * lda >= lim) return false;
  for (int i = 0; i < segs.count; ++i)
    if (segs.cols[i] % 8 != 0 || (long long)K * segs.cols[i] >= lim) return false;
  return true;
}

// fin != nullptr (one K slice, MFMA path): the up-projection epilogue instead of partial sums
int launch_gemm(int dtype, const void* A, int lda, int M, const GemmSegments& segs, int K, int n_slices,
                int rows_per_slice, float* part, int ld_out, hipStream_t stream, const GemmFinishUp* fin = nullptr) {
  if (gemm_mfma_ok(dtype, M, K, lda, segs)) {
    static PerDeviceSetup setup;
    int setup_dev = -1;
    if (setup.needed(&setup_dev)) {
      bool ok = true;
#define MLRA_GEMM_LDS(MT)                                                                                            \
  ok = ok &&                                                                                                         \
       hipFuncSetAttribute((const void*)skinny_gemm_mfma_kernel<MT, false>, hipFuncAttributeMaxDynamicSharedMemorySize, \
                           gemm_stages(MT) * gemm_stage_bytes(MT)) == hipSuccess &&                                   \
       hipFuncSetAttribute((const void*)skinny_gemm_mfma_kernel<MT, true>, hipFuncAttributeMaxDynamicSharedMemorySize,  \
                           gemm_stages(MT) * gemm_stage_bytes(MT)) == hipSuccess
      MLRA_GEMM_LDS(1);
      MLRA_GEMM_LDS(2);
      MLRA_GEMM_LDS(3);
      MLRA_GEMM_LDS(4);
#undef MLRA_GEMM_LDS
      if (!ok)
        return MLRA_ERR_LAUNCH;
      setup.done(setup_dev);
    }
    int tiles = 0;
    for (int i = 0; i < segs.count; ++i) tiles += (segs.cols[i] + kColsWG - 1) / kColsWG;
    const int mt = M >= 32 * kMaxMTiles ? kMaxMTiles : (M + 31) / 32;
    dim3 grid(tiles, n_slices, (M + 32 * mt - 1) / (32 * mt));
    const size_t lds = (size_t)gemm_stages(mt) * gemm_stage_bytes(mt);
    const bf16_t* a = (const bf16_t*)A;
    GemmFinishUp f = {};
    if (fin) f = *fin;
#define MLRA_GEMM_LAUNCH(MT)                                                                                          \
  if (fin)                                                                                                            \
    skinny_gemm_mfma_kernel<MT, true><<<grid, 256, lds, stream>>>(a, lda, M, segs, K, rows_per_slice, part, ld_out, f); \
  else                                                                                                                \
    skinny_gemm_mfma_kernel<MT, false><<<grid, 256, lds, stream>>>(a, lda, M, segs, K, rows_per_slice, part, ld_out, f)
    if (mt == 1) { MLRA_GEMM_LAUNCH(1); }
    else if (mt == 2) { MLRA_GEMM_LAUNCH(2); }
    else if (mt == 3) { MLRA_GEMM_LAUNCH(3); }
    else { MLRA_GEMM_LAUNCH(4); }
#undef MLRA_GEMM_LAUNCH
  } else {
    dim3 grid((ld_out + 255) / 256, M);
    if (dtype == MLRA_BF16)
      skinny_gemm_generic_kernel<bf16_t><<<grid, 256, 0, stream>>>((const bf16_t*)A, lda, M, segs, K, part, ld_out,
                                                                   ld_out);
    else
      skinny_gemm_generic_kernel<float><<<grid, 256, 0, stream>>>((const float*)A, lda, M, segs, K, part, ld_out,
                                                                  ld_out);
  }
  return check_launch();
}

}  // namespace

// K slices of a skinny GEMM: enough workgroups to cover the chip, whole chunks of kRowsChunk rows per slice.
PrePlan pre_plan(int dtype, int batch, int d, int d_cq, int d_c, int d_r, int h, int d_h) {
  PrePlan p;
  p.n1 = d_cq + d_c + d_r;
  p.n2 = h * (d_h + d_r);
  auto slices = [&](int K, int tiles, int& n_slices, int& rows) {
    const int chunks = (K + kRowsChunk - 1) / kRowsChunk;
    int want = (device_cu_count() + tiles / 2) / tiles;   // nearest: a second partial round costs more than idle CUs
    if (want > chunks) want = chunks;
    if (want < 1) want = 1;
    const int per = (chunks + want - 1) / want;
    rows = per * kRowsChunk;
    n_slices = (chunks + per - 1) / per;
  };
  GemmSegments s1, s2;
  s1.count = 3; s1.cols[0] = d_cq; s1.cols[1] = d_c; s1.cols[2] = d_r;
  s2.count = 2; s2.cols[0] = h * d_h; s2.cols[1] = h * d_r; s2.cols[2] = 0;
  p.mfma1 = gemm_mfma_ok(dtype, batch, d, d, s1);
  p.mfma2 = gemm_mfma_ok(dtype, batch, d_cq, d_cq, s2);
  p.slices1 = p.slices2 = 1;
  p.rows1 = d;
  p.rows2 = d_cq;
  if (p.mfma1) slices(d, (d_cq + 127) / 128 + (d_c + 127) / 128 + (d_r + 127) / 128, p.slices1, p.rows1);
  if (p.mfma2) slices(d_cq, (h * d_h + 127) / 128 + (h * d_r + 127) / 128, p.slices2, p.rows2);
  const size_t elt = dtype == MLRA_BF16 ? 2 : 4;
  p.off_part1 = 0;
  p.off_cq = align_up((size_t)p.slices1 * batch * p.n1 * sizeof(float), 256);
  p.off_cs = p.off_cq + align_up((size_t)batch * d_cq * elt, 256);
  p.off_part2 = p.off_cs + align_up((size_t)batch * d_r * sizeof(float), 256);
  p.bytes = p.off_part2 + align_up((size_t)p.slices2 * batch * p.n2 * sizeof(float), 256);
  return p;
}

int launch_pre_attention(const mlra_cache* c, const mlra_pre_weights* w, int batch, const void* hidden,
                         const int32_t* positions, void* q_nope, void* q_rope, void* workspace,
                         hipStream_t stream) {
  const int d_c = c->n_blocks * c->d_cb;
  const PrePlan p = pre_plan(w->dtype, batch, w->d, w->d_cq, d_c, c->d_r, w->h, w->d_h);
  float* part1 = (float*)((char*)workspace + p.off_part1);
  void* c_q = (char*)workspace + p.off_cq;
  float* cs_tab = (float*)((char*)workspace + p.off_cs);
  float* part2 = (float*)((char*)workspace + p.off_part2);

  GemmSegments s1;
  s1.count = 3;
  s1.w[0] = w->w_dq;  s1.cols[0] = w->d_cq; s1.out_col[0] = 0;
  s1.w[1] = w->w_dkv; s1.cols[1] = d_c;     s1.out_col[1] = w->d_cq;
  s1.w[2] = w->w_kr;  s1.cols[2] = c->d_r;  s1.out_col[2] = w->d_cq + d_c;
  int st = launch_gemm(w->dtype, hidden, w->d, batch, s1, w->d, p.slices1, p.rows1, part1, p.n1, stream);
  if (st != MLRA_OK) return st;

  const size_t lds = (size_t)p.n1 * sizeof(float);
#define MLRA_PRE_DOWN(T, TC)                                                                                       \
  pre_finish_down_kernel<T, TC><<<batch, 256, lds, stream>>>(                                                      \
      part1, p.slices1, batch, w->d_cq, d_c, c->d_r, c->n_blocks, (const T*)w->gain_q, (const T*)w->gain_kv,        \
      w->alpha_q, w->alpha_kv, w->eps, w->rope_base, positions, c->page_table, c->max_pages_per_seq, c->page_size, \
      (T*)c_q, (TC*)c->latent, (TC*)c->rope, cs_tab)
  if (w->dtype == MLRA_BF16 && c->dtype == MLRA_BF16) MLRA_PRE_DOWN(bf16_t, bf16_t);
  else if (w->dtype == MLRA_BF16) MLRA_PRE_DOWN(bf16_t, float);
  else if (c->dtype == MLRA_BF16) MLRA_PRE_DOWN(float, bf16_t);
  else MLRA_PRE_DOWN(float, float);
#undef MLRA_PRE_DOWN
  if ((st = check_launch()) != MLRA_OK) return st;

  GemmSegments s2;
  s2.count = 2;
  s2.w[0] = w->w_uq; s2.cols[0] = w->h * w->d_h;  s2.out_col[0] = 0;
  s2.w[1] = w->w_qr; s2.cols[1] = w->h * c->d_r;  s2.out_col[1] = w->h * w->d_h;
  s2.w[2] = nullptr; s2.cols[2] = 0;              s2.out_col[2] = 0;
  if (p.mfma2 && p.slices2 == 1 && c->d_r % 8 == 0) {
    // one K slice: the GEMM's own epilogue writes q_nope and the rotated q_rope
    const GemmFinishUp fin = {cs_tab, (bf16_t*)q_nope, (bf16_t*)q_rope, c->d_r};
    return launch_gemm(w->dtype, c_q, w->d_cq, batch, s2, w->d_cq, 1, p.rows2, part2, p.n2, stream, &fin);
  }
  st = launch_gemm(w->dtype, c_q, w->d_cq, batch, s2, w->d_cq, p.slices2, p.rows2, part2, p.n2, stream);
  if (st != MLRA_OK) return st;

  dim3 grid((p.n2 / 2 + 255) / 256, batch);
  if (w->dtype == MLRA_BF16)
    pre_finish_up_kernel<bf16_t><<<grid, 256, 0, stream>>>(part2, p.slices2, batch, w->h, w->d_h, c->d_r, cs_tab,
                                                            (bf16_t*)q_nope, (bf16_t*)q_rope);
  else
    pre_finish_up_kernel<float><<<grid, 256, 0, stream>>>(part2, p.slices2, batch, w->h, w->d_h, c->d_r, cs_tab,
                                                           (float*)q_nope, (float*)q_rope);
  return check_launch();
}

}  // namespace mlra
