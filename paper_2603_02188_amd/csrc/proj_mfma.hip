// MFMA kernels for the two per-head projections around the decode kernel (bf16, d_h = 128):
//   * absorb_q:  q~_b[i] = W^UK_(b),(i) q_i                (Step 1, Section 2.1, per block)
//   * merge + up-projection + block sum:  out[i] = out_scale * sum_b z_b[i] W^UV_(b),(i)
//     (log-sum-exp merge of the context chunks, then Step 3 and the block sum of Eq. (5) as one
//      contraction over all n_blocks * d_cb latent channels)
// Both are batched over sequences as the MFMA M dimension so that each weight element is read once
// per workgroup, and both put the head index on the grid.
#include <type_traits>

#include "mlra_internal.h"

namespace mlra {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(4))) short short4v;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;

constexpr int kDh = 128;
constexpr float kNegBig = -1.0e30f;
constexpr float kLn2 = 0.6931471805599453f;

__device__ __forceinline__ int swz(int t) { return ((t & 3) << 1) | ((t >> 2) & 1); }

// Zero that the compiler cannot fold: an accumulator initialised from it is a real register operand, so
// every MFMA is emitted in the tied form (destination = accumulator input) and its destination can
// never be placed on top of its A / B operands.
__device__ __forceinline__ f32x16 opaque_zero() {
  float z = 0.f;
  asm volatile("" : "+v"(z));
  f32x16 acc;
#pragma unroll
  for (int i = 0; i < 16; ++i) acc[i] = z;
  return acc;
}

__device__ __forceinline__ short4v lds_tr16(const void* p) {
  return __builtin_amdgcn_ds_read_tr16_b64_v4i16((short4v __attribute__((address_space(3)))*)p);
}

// ------------------------------------------------------------------------------------------------
// absorb_q.  One workgroup per (head, block, 64 sequences); wave w produces the 32-channel tile ct0 + w of
// each pass over four tiles: out[seq][c] = sum_p q[seq][p] W[c][p].  An MFMA operand wants sixteen bytes of
// each of 32 rows per lane group, and rows of q (one per sequence) and of W (one per channel) lie 32 KiB
// apart: read in that shape, every load instruction touches 64 cache lines for 1 KiB.  So both are fetched
// as whole 256-byte rows (sixteen lanes a row), laid into LDS with a chunk swizzle, and the operands are
// read from there; the 64 query rows are fetched once per workgroup instead of once per wave.  The results
// pass through LDS as well, so that they leave as whole 16-byte pieces of the q_abs rows.  Larger batches
// put their 64-sequence tiles on the grid (the weights of a head are then read once from HBM and again
// from L2).
// ------------------------------------------------------------------------------------------------
constexpr int kAbsPitch = 128 * 2 + 16;   // bytes per staged sequence row (128 channels; +16: rows on different banks)
constexpr int kAbsQ = 64 * 256;           // LDS: the 64 query rows of the head ...
constexpr int kAbsW = 4 * 32 * 256;       // ... and 32 weight rows per wave (the result staging reuses this part)
static_assert(64 * kAbsPitch <= kAbsW, "the staged results must fit the weight rows' space");

__global__ __launch_bounds__(256) void absorb_q_mfma_kernel(const bf16_t* __restrict__ q_nope,
                                                            const bf16_t* __restrict__ w_uk,
                                                            bf16_t* __restrict__ q_abs, int batch, int h,
                                                            int n_blocks, int groups, int d_cb, float fold,
                                                            const bf16_t* __restrict__ q_rope,
                                                            bf16_t* __restrict__ q_rope_out, int d_r) {
  // h: heads per block; q_nope holds groups * h heads and block b reads those of its group (Eq. (6))
  // fold: factor applied to the absorbed queries before they are rounded (1, or tau log2(e) when the
  // softmax scale is folded into the queries); the workgroups with blockIdx.y == n_blocks (launched only
  // then) apply it to the RoPE queries of head blockIdx.x of every group.
  __shared__ __attribute__((aligned(16))) unsigned char smem[kAbsQ + kAbsW];
  if (blockIdx.y == (unsigned)n_blocks) {
    const int m0r = blockIdx.z * 64, q_heads_r = h * groups, per_row = d_r >> 3;   // d_r % 8 == 0 (launcher)
    for (int id = threadIdx.x; id < 64 * groups * per_row; id += 256) {
      const int pc = id % per_row, grp = (id / per_row) % groups, s_ = m0r + id / (per_row * groups);
      if (s_ >= batch) continue;
      const size_t off = ((size_t)s_ * q_heads_r + grp * h + blockIdx.x) * d_r + pc * 8;
      bf16x8 v = *(const bf16x8*)(q_rope + off);
#pragma unroll
      for (int e = 0; e < 8; ++e) v[e] = (__bf16)((float)v[e] * fold);
      *(bf16x8*)(q_rope_out + off) = v;
    }
    return;
  }
  unsigned char* const qs = smem;
  unsigned char* const ws = smem + kAbsQ;
  unsigned char* const stage = ws;
  const int head = blockIdx.x, b = blockIdx.y;
  const int q_head = (b / (n_blocks / groups)) * h + head, q_heads = h * groups;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, g = lane >> 5, c32 = lane & 31;
  const size_t ldw = (size_t)h * kDh;
  const int m0 = blockIdx.z * 64;      // 64 sequences per workgroup
  // rows are stored with 16-byte chunk c at position c ^ (row % 16): the sixteen lanes that a 128-bit LDS
  // read serves together (rows 0-3, 12-15, 20-27 of one chunk column, and so on) then hit sixteen positions
  const int ld_chunk = tid & 15, ld_row = tid >> 4;          // loads: thread = (row % 16 of its pass, chunk)
  bf16x8 qld[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int seq = min(m0 + 16 * i + ld_row, batch - 1);
    qld[i] = *(const bf16x8*)(q_nope + ((size_t)seq * q_heads + q_head) * kDh + ld_chunk * 8);
  }
  bf16x8 areg[2][8];
  for (int ct0 = 0; ct0 * 32 < d_cb; ct0 += 4) {
    const int ct = ct0 + wave;
    const bool live = ct * 32 < d_cb;                       // (uniform per wave)
    // this wave's 32 weight rows (a wave past the last channel tile repeats the last row and stores nothing)
    bf16x8 wld[8];
    {
      const int wl_chunk = lane & 15, wl_row = lane >> 4;
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const int c = min(ct * 32 + 4 * i + wl_row, d_cb - 1);
        wld[i] = *(const bf16x8*)(w_uk + ((size_t)b * d_cb + c) * ldw + (size_t)head * kDh + wl_chunk * 8);
      }
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const int r = 4 * i + wl_row;
        *(bf16x8*)(ws + wave * (32 * 256) + r * 256 + ((wl_chunk ^ (r & 15)) << 4)) = wld[i];
      }
    }
    if (ct0 == 0) {
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int r = 16 * i + ld_row;
        *(bf16x8*)(qs + r * 256 + ((ld_chunk ^ (r & 15)) << 4)) = qld[i];
      }
    }
    __syncthreads();
    bf16x8 breg[8];
#pragma unroll
    for (int ks = 0; ks < 8; ++ks)
      breg[ks] = *(const bf16x8*)(ws + wave * (32 * 256) + c32 * 256 + (((2 * ks + g) ^ (c32 & 15)) << 4));
    if (ct0 == 0) {
#pragma unroll
      for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int ks = 0; ks < 8; ++ks)
          areg[t][ks] = *(const bf16x8*)(qs + (32 * t + c32) * 256 + (((2 * ks + g) ^ (c32 & 15)) << 4));
    }
    __syncthreads();      // every wave holds its operands: the weight rows' space becomes the result staging
    const int pass_ch = min(128, d_cb - ct0 * 32);          // channels this pass produces
    f32x16 acc[2] = {opaque_zero(), opaque_zero()};
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) {
      acc[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(areg[0][ks], breg[ks], acc[0], 0, 0, 0);
      acc[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(areg[1][ks], breg[ks], acc[1], 0, 0, 0);
    }
    if (live) {
#pragma unroll
      for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int row = 32 * t + (r >> 2) * 8 + g * 4 + (r & 3);
          *(bf16_t*)(stage + row * kAbsPitch + (wave * 32 + c32) * 2) = f32_to_bf16(acc[t][r] * fold);
        }
    }
    __syncthreads();
    // 64 rows x (pass_ch / 8) 16-byte pieces, one piece per thread and step
    const int pieces = pass_ch >> 3;
    for (int id = tid; id < 64 * pieces; id += 256) {
      const int row = id / pieces, pc = id - row * pieces, s_ = m0 + row;
      if (s_ < batch)
        *(bf16x8*)(q_abs + (((size_t)s_ * n_blocks + b) * h + head) * d_cb + ct0 * 32 + pc * 8) =
            *(const bf16x8*)(stage + row * kAbsPitch + pc * 16);
    }
    __syncthreads();
  }
}

// ------------------------------------------------------------------------------------------------
// merge + up-projection.  One workgroup per (head, tile of up to 32 sequences).
//   phase 0: the loads of the first 512 rows of this head's W^UV slice are issued into registers, so
//            that they are in flight while phase 1 runs (and, when every sequence has a single chunk, the
//            loads of the rows that the decode kernel already normalised and rounded: see `direct`);
//   phase 1a: one thread per (sequence, block) turns the chunk partials' (m, l) into normalised merge
//            weights w_k = 2^(m_k - m*) / L in LDS and writes the log-sum-exp;
//   phase 1b: merged z = sum_k w_k z_k of the 32 sequences for all R = n_blocks*d_cb latent channels,
//            rounded to bf16, is built in LDS (row = sequence), four independent items per thread at a
//            time so that their loads overlap (`direct`: the rows arrive merged, they are only copied);
//   phase 2: out[seq][j] = sum_r z[seq][r] W^UV[r][head*128 + j]; W^UV goes through LDS 256 rows at a
//            time and reaches the MFMA B operand through transpose reads; wave w owns output columns
//            [32 w, 32 w + 32).
// ------------------------------------------------------------------------------------------------
constexpr int kWRowsLds = 256;    // W^UV rows resident in LDS at a time (64 KiB)
constexpr int kWRowsRegs = 512;   // W^UV rows prefetched into registers at a time (32 loads per thread)

template <typename TO>
__global__ __launch_bounds__(256) void merge_upproj_mfma_kernel(
    const float* __restrict__ part_z, const float* __restrict__ part_ml, const int32_t* __restrict__ seq_lens,
    const bf16_t* __restrict__ w_uv, TO* __restrict__ out, float* __restrict__ lse, int batch, int h, int nb_total,
    int d_cb, int n_splits, int chunk, const int32_t* __restrict__ chunk_tab, float out_scale,
    const bf16_t* __restrict__ gate, int rows_bf16, int spw) {
  extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
  // blockIdx.z = head group (Eq. (6)); one group of all blocks is Eq. (5).  h: heads per block; this
  // workgroup's head is h * group + head in out, and its branches are blocks [b0, b0 + n_blocks).
  const int n_blocks = nb_total / gridDim.z, b0 = blockIdx.z * n_blocks;
  const int R = n_blocks * d_cb;
  const int zpitch = R + 8;                               // bf16 elements per z row (+16 B against conflicts)
  const int units_per_seq = n_blocks * n_splits;
  unsigned char* wt = smem;                               // [256 rows][256 B], 16-byte chunks swizzled
  bf16_t* zt = (bf16_t*)(smem + kWRowsLds * 256);         // [32][zpitch]
  float* wtab = (float*)(smem + kWRowsLds * 256 + (size_t)32 * zpitch * 2);   // [32][units_per_seq]
  float* ltab = wtab + 32 * units_per_seq;                 // [32][units_per_seq] row sums of the partials
  int* act = (int*)(ltab + 32 * units_per_seq);           // [32] active chunks per sequence
  // spw: sequences per workgroup (32, or fewer for small batches so that more workgroups share the merge;
  // the rest of the 32 MFMA rows is zero padding)
  const int head = blockIdx.x, m0 = blockIdx.y * spw;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, g = lane >> 5, c32 = lane & 31;
  const size_t ldw = (size_t)h * kDh;

  // ---- phase 0: thread t owns 16-byte chunk t % 16 of rows t / 16 + 16 i
  bf16x8 wreg[kWRowsRegs / 16];
  const bf16_t* wsrc = w_uv + ((size_t)b0 * d_cb + (tid >> 4)) * ldw + (size_t)head * kDh + (tid & 15) * 8;
  auto fetch_w = [&](int row0) {
#pragma unroll
    for (int i = 0; i < kWRowsRegs / 16; ++i)
      if (row0 + 16 * i < R) wreg[i] = *(const bf16x8*)(wsrc + (size_t)(row0 + 16 * i) * ldw);
  };
  fetch_w(0);
  // (single-chunk rows, see phase 1b: their loads do not depend on phase 1a, so they go out here as well;
  // what a sequence without tokens leaves in the workspace is discarded below)
  constexpr int kZPre = 8;
  bf16x8 zpre[kZPre];
  const int items_per_row = R / 8;
  const int n_valid = min(spw, batch - m0);
  const int n_items = n_valid * items_per_row;
  // normalised bf16 rows, one chunk per sequence: the rows are final (see phase 1b)
  const bool direct = rows_bf16 && n_splits == 1;
  const bool z_early = direct && n_items <= kZPre * 256;
  if (z_early) {
#pragma unroll
    for (int u = 0; u < kZPre; ++u) {
      const int item = min(tid + u * 256, n_items - 1);
      const int sl = item / items_per_row, r0 = (item % items_per_row) * 8;
      zpre[u] = *(const bf16x8*)((const bf16_t*)part_z +
                                 (((size_t)(m0 + sl) * nb_total + b0 + r0 / d_cb) * h + head) * d_cb + r0 % d_cb);
    }
  }

  // ---- phase 1a: every (sequence, block, chunk) partial's (m, l) goes to LDS with one load per thread,
  // then one thread per (sequence, block) reduces them
  for (int t = tid; t < 32 * units_per_seq; t += 256) {
    const int sl = t / units_per_seq, seq = m0 + sl, k = t % n_splits;
    float2 ml = make_float2(kNegBig, 0.f);
    if (sl < n_valid) {
      // the slot exists in the workspace whether or not its chunk ran: loaded without waiting for the
      // sequence length (one round trip instead of two), kept only if the chunk is active
      const float2 got =
          *(const float2*)(part_ml + ((((size_t)seq * nb_total + b0) * n_splits + t % units_per_seq) * h + head) * 2);
      const int ch = chunk_tab ? chunk_tab[seq] : chunk;
      const int active = min(n_splits, (seq_lens[seq] + ch - 1) / ch);
      if (k < active) ml = got;
    }
    wtab[t] = ml.x;
    ltab[t] = ml.y;
  }
  __syncthreads();
  for (int t = tid; t < 32 * n_blocks; t += 256) {
    const int sl = t / n_blocks, b = t % n_blocks, seq = m0 + sl;
    float* wrow = wtab + sl * units_per_seq + b * n_splits;
    const float* lrow = ltab + sl * units_per_seq + b * n_splits;
    int active = 0;
    if (sl < n_valid) {
      const int ch = chunk_tab ? chunk_tab[seq] : chunk;
      active = min(n_splits, (seq_lens[seq] + ch - 1) / ch);
      float m_star = kNegBig;
      for (int k = 0; k < active; ++k) m_star = fmaxf(m_star, wrow[k]);
      float L = 0.f;
      for (int k = 0; k < active; ++k) {
        const float w = exp2f(wrow[k] - m_star);
        L += w * lrow[k];
        // (a partial that arrives normalised, z_k / l_k, carries its row sum in its weight)
        wrow[k] = rows_bf16 ? w * lrow[k] : w;
      }
      const float inv = L > 0.f ? 1.f / L : 0.f;
      for (int k = 0; k < active; ++k) wrow[k] *= inv;
      if (lse) lse[((size_t)seq * nb_total + b0 + b) * h + head] = L > 0.f ? (m_star + log2f(L)) * kLn2 : -INFINITY;
    }
    if (b == 0) act[sl] = active;
  }
  __syncthreads();

  // ---- phase 1b: item = (valid sequence slot, 8 consecutive latent channels).  A thread takes U items
  // at a time and KK chunks of each per round trip, U * KK = 16 (32 loads in flight): many chunks (small
  // batches) go one item per thread with sixteen chunks in flight, one or two chunks eight items per
  // thread.
  // rows of sequences past the batch feed MFMA rows that are never stored; they only have to be finite
  for (int t = n_items + tid; t < 32 * items_per_row; t += 256) {
    bf16x8 zero;
#pragma unroll
    for (int e = 0; e < 8; ++e) zero[e] = (__bf16)0.0f;
    *(bf16x8*)(zt + (t / items_per_row) * zpitch + (t % items_per_row) * 8) = zero;
  }
  const size_t z_stride = (size_t)h * d_cb;
  auto merge_items = [&](auto u_tag) {
    constexpr int U = decltype(u_tag)::value, KK = 16 / U;
    for (int base = tid; base < n_items; base += U * 256) {
      float z[U][8];
      const float* pz[U];
      const float* wk[U];
      int na[U], sl[U], r0[U], kmax = 0;
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int item = base + u * 256;
        sl[u] = min(item, n_items - 1) / items_per_row;
        r0[u] = (min(item, n_items - 1) % items_per_row) * 8;
        const int b = r0[u] / d_cb, c0 = r0[u] % d_cb;
        na[u] = item < n_items ? act[sl[u]] : 0;
        kmax = max(kmax, na[u]);
        pz[u] = part_z + ((((size_t)(m0 + sl[u]) * nb_total + b0 + b) * n_splits) * h + head) * d_cb + c0;
        wk[u] = wtab + sl[u] * units_per_seq + b * n_splits;
#pragma unroll
        for (int e = 0; e < 8; ++e) z[u][e] = 0.f;
      }
      for (int k0 = 0; k0 < kmax; k0 += KK) {
        f32x4 lo[KK][U], hi[KK][U];
        float w[KK][U];
#pragma unroll
        for (int kk = 0; kk < KK; ++kk)
#pragma unroll
          for (int u = 0; u < U; ++u) {
            const int k = k0 + kk;
            const bool on = k < na[u];
            const f32x4* src = (const f32x4*)(pz[u] + (on ? k : 0) * z_stride);
            w[kk][u] = on ? wk[u][k] : 0.f;
            if (on) { lo[kk][u] = src[0]; hi[kk][u] = src[1]; }
            else { lo[kk][u] = f32x4{0.f, 0.f, 0.f, 0.f}; hi[kk][u] = lo[kk][u]; }
          }
#pragma unroll
        for (int kk = 0; kk < KK; ++kk)
#pragma unroll
          for (int u = 0; u < U; ++u)
#pragma unroll
            for (int e = 0; e < 4; ++e) {
              z[u][e] += w[kk][u] * lo[kk][u][e];
              z[u][4 + e] += w[kk][u] * hi[kk][u][e];
            }
      }
#pragma unroll
      for (int u = 0; u < U; ++u) {
        if (base + u * 256 < n_items) {
          bf16x8 packed;
#pragma unroll
          for (int e = 0; e < 8; ++e) packed[e] = (__bf16)z[u][e];
          *(bf16x8*)(zt + sl[u] * zpitch + r0[u]) = packed;
        }
      }
    }
  };
  // the same for partials that are normalised bf16 rows (16 bytes per item and chunk)
  auto merge_rows = [&](auto u_tag) {
    constexpr int U = decltype(u_tag)::value, KK = 16 / U;
    const bf16_t* zn = (const bf16_t*)part_z;
    for (int base = tid; base < n_items; base += U * 256) {
      float z[U][8];
      const bf16_t* pz[U];
      const float* wk[U];
      int na[U], sl[U], r0[U], kmax = 0;
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int item = base + u * 256;
        sl[u] = min(item, n_items - 1) / items_per_row;
        r0[u] = (min(item, n_items - 1) % items_per_row) * 8;
        const int b = r0[u] / d_cb, c0 = r0[u] % d_cb;
        na[u] = item < n_items ? act[sl[u]] : 0;
        kmax = max(kmax, na[u]);
        pz[u] = zn + ((((size_t)(m0 + sl[u]) * nb_total + b0 + b) * n_splits) * h + head) * d_cb + c0;
        wk[u] = wtab + sl[u] * units_per_seq + b * n_splits;
#pragma unroll
        for (int e = 0; e < 8; ++e) z[u][e] = 0.f;
      }
      for (int k0 = 0; k0 < kmax; k0 += KK) {
        bf16x8 row[KK][U];
        float w[KK][U];
#pragma unroll
        for (int kk = 0; kk < KK; ++kk)
#pragma unroll
          for (int u = 0; u < U; ++u) {
            const int k = k0 + kk;
            const bool on = k < na[u];
            w[kk][u] = on ? wk[u][k] : 0.f;
            row[kk][u] = *(const bf16x8*)(pz[u] + (on ? k : 0) * z_stride);   // (chunk 0's slot always exists)
          }
#pragma unroll
        for (int kk = 0; kk < KK; ++kk)
#pragma unroll
          for (int u = 0; u < U; ++u)
#pragma unroll
            for (int e = 0; e < 8; ++e)
              // (an inactive chunk has weight 0; what its slot holds may be anything, NaN included)
              z[u][e] += w[kk][u] != 0.f ? w[kk][u] * (float)row[kk][u][e] : 0.f;
      }
#pragma unroll
      for (int u = 0; u < U; ++u) {
        if (base + u * 256 < n_items) {
          bf16x8 packed;
#pragma unroll
          for (int e = 0; e < 8; ++e) packed[e] = (__bf16)z[u][e];
          *(bf16x8*)(zt + sl[u] * zpitch + r0[u]) = packed;
        }
      }
    }
  };
  if (z_early) {
    // one chunk per sequence and the decode kernel wrote z / l as bf16 rows [.][block][head][d_cb]: the
    // rows fetched at the top go to LDS
    bf16x8 zero;
#pragma unroll
    for (int e = 0; e < 8; ++e) zero[e] = (__bf16)0.0f;
#pragma unroll
    for (int u = 0; u < kZPre; ++u) {
      const int item = tid + u * 256;
      if (item < n_items) {
        const int sl = item / items_per_row, r0 = (item % items_per_row) * 8;
        *(bf16x8*)(zt + sl * zpitch + r0) = act[sl] > 0 ? zpre[u] : zero;
      }
    }
  } else if (direct) {
    // (the same for more rows than a thread prefetches)
    const bf16_t* zn = (const bf16_t*)part_z;
    for (int item = tid; item < n_items; item += 256) {
      const int sl = item / items_per_row, r0 = (item % items_per_row) * 8;
      const int b = r0 / d_cb, c0 = r0 % d_cb;
      bf16x8 v;
#pragma unroll
      for (int e = 0; e < 8; ++e) v[e] = (__bf16)0.0f;
      if (act[sl] > 0) v = *(const bf16x8*)(zn + (((size_t)(m0 + sl) * nb_total + b0 + b) * h + head) * d_cb + c0);
      *(bf16x8*)(zt + sl * zpitch + r0) = v;
    }
  } else if (rows_bf16) {
    if (n_splits > 8) merge_rows(std::integral_constant<int, 1>{});
    else if (n_splits > 4) merge_rows(std::integral_constant<int, 2>{});
    else if (n_splits > 2) merge_rows(std::integral_constant<int, 4>{});
    else merge_rows(std::integral_constant<int, 8>{});
  } else if (n_splits > 8) merge_items(std::integral_constant<int, 1>{});
  else if (n_splits > 4) merge_items(std::integral_constant<int, 2>{});
  else if (n_splits > 2) merge_items(std::integral_constant<int, 4>{});
  else merge_items(std::integral_constant<int, 8>{});

  // ---- phase 2 ----
  f32x16 acc = opaque_zero();
  // transpose-read offsets: the 16 lanes of a block fetch 4 consecutive rows x 16 output columns
  unsigned tr_off[2];
  {
    const int k = (lane & 15) >> 2, seg = lane & 3, hb = (lane >> 4) & 1;
#pragma unroll
    for (int half = 0; half < 2; ++half) {
      const int row = 8 * g + 4 * half + k;                 // + 16 per MFMA k-step (same swizzle: row & 7)
      const int cc = 4 * wave + 2 * hb + (seg >> 1);
      tr_off[half] = row * 256 + ((cc ^ swz(row & 7)) << 4) + ((seg & 1) << 3);
    }
  }
  for (int pass0 = 0; pass0 < R; pass0 += kWRowsRegs) {
    if (pass0 > 0) fetch_w(pass0);
#pragma unroll
    for (int part = 0; part < kWRowsRegs / kWRowsLds; ++part) {
      const int row_base = pass0 + part * kWRowsLds;
      if (row_base >= R) break;
      __syncthreads();   // phase 1 done / previous rows consumed
#pragma unroll
      for (int i = 0; i < kWRowsLds / 16; ++i) {
        const int row = (tid >> 4) + 16 * i, cc = tid & 15;
        if (row_base + row < R)
          *(bf16x8*)(wt + row * 256 + ((cc ^ swz(row & 7)) << 4)) = wreg[part * (kWRowsLds / 16) + i];
      }
      __syncthreads();
      const int rows = min(kWRowsLds, R - row_base);
      auto k_step = [&](int ks) {
        const bf16x8 a = *(const bf16x8*)(zt + c32 * zpitch + row_base + ks * 16 + g * 8);
        const short4v lo = lds_tr16(wt + ks * 16 * 256 + tr_off[0]);
        const short4v hi = lds_tr16(wt + ks * 16 * 256 + tr_off[1]);
        const bf16x8 bm = __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
        acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, bm, acc, 0, 0, 0);
      };
      if (rows == kWRowsLds) {
        // straight-line, so that the LDS reads of later steps are issued ahead of the MFMAs of earlier ones
#pragma unroll
        for (int ks = 0; ks < kWRowsLds / 16; ++ks) k_step(ks);
      } else {
        for (int ks = 0; ks < rows / 16; ++ks) k_step(ks);
      }
    }
  }
  const int j = wave * 32 + c32;
#pragma unroll
  for (int r = 0; r < 16; ++r) {
    const int sl = (r >> 2) * 8 + g * 4 + (r & 3), s = m0 + sl;
    if (sl < n_valid) {
      const size_t o = ((size_t)s * h * gridDim.z + blockIdx.z * h + head) * kDh + j;
      store_f32(out, o, acc[r] * out_scale * (gate ? bf16_to_f32(gate[o]) : 1.f));   // gate: Appendix E
    }
  }
}

}  // namespace

bool absorb_q_mfma_supported(int d_h, int d_cb, int dtype) {
  return dtype == MLRA_BF16 && d_h == kDh && d_cb % 32 == 0;
}

int launch_absorb_q_mfma(int batch, int h, int d_h, int n_blocks, int groups, int d_cb, const void* q_nope,
                         const void* w_uk, void* q_abs, hipStream_t stream, float fold, const void* q_rope,
                         void* q_rope_out, int d_r) {
  (void)d_h;
  dim3 grid(h, n_blocks + (q_rope_out ? 1 : 0), (batch + 63) / 64);
  absorb_q_mfma_kernel<<<grid, 256, 0, stream>>>((const bf16_t*)q_nope, (const bf16_t*)w_uk, (bf16_t*)q_abs, batch, h,
                                                 n_blocks, groups, d_cb, fold, (const bf16_t*)q_rope,
                                                 (bf16_t*)q_rope_out, d_r);
  return check_launch();
}

// Dynamic LDS of the merge + up-projection kernel: the weight rows, the normalised z rows of 32 sequences,
// the merge weights of every (sequence, block, chunk), the active-chunk counts.
static size_t merge_upproj_lds_bytes(const DecodeArgs& a) {
  const int bpg = a.n_blocks / a.groups, R = bpg * a.d_cb;
  return (size_t)kWRowsLds * 256 + (size_t)32 * (R + 8) * 2 + (size_t)64 * bpg * a.plan.n_splits * sizeof(float) +
         32 * sizeof(int);
}
constexpr size_t kMergeLdsLimit = 160 * 1024;

// (shapes whose tables would not fit the 160 KiB of LDS take the generic epilogue instead of failing at launch)
bool merge_upproj_mfma_supported(const DecodeArgs& a) {
  return a.dtype == MLRA_BF16 && a.d_h == kDh && a.d_cb % 32 == 0 && a.n_blocks / a.groups * a.d_cb <= 1024 &&
         a.n_blocks / a.groups * a.plan.n_splits <= 128 && merge_upproj_lds_bytes(a) <= kMergeLdsLimit;
}

int launch_merge_upproj_mfma(const DecodeArgs& a) {
  const size_t lds = merge_upproj_lds_bytes(a);
  static PerDeviceSetup setup;
  int setup_dev = -1;
  if (setup.needed(&setup_dev)) {
    if (hipFuncSetAttribute((const void*)merge_upproj_mfma_kernel<bf16_t>, hipFuncAttributeMaxDynamicSharedMemorySize,
                            (int)kMergeLdsLimit) != hipSuccess ||
        hipFuncSetAttribute((const void*)merge_upproj_mfma_kernel<float>, hipFuncAttributeMaxDynamicSharedMemorySize,
                            (int)kMergeLdsLimit) != hipSuccess)
      return MLRA_ERR_LAUNCH;
    setup.done(setup_dev);
  }
  // small batches: fewer sequences per workgroup while that brings more workgroups onto idle CUs
  int spw = 32;
  while (spw > 8 && (long)a.h * a.groups * ((a.batch + spw - 1) / spw) < device_cu_count()) spw /= 2;
  dim3 grid(a.h, (a.batch + spw - 1) / spw, a.groups);
  const int32_t* const chunk_tab = a.balanced ? a.chunk_tab : nullptr;
  const int direct = a.rows_bf16 ? 1 : 0;
  if (a.out_dtype == MLRA_BF16)
    MLRA_LAUNCH_TIMED(a.t_epi, merge_upproj_mfma_kernel<bf16_t>, grid, dim3(256), lds, a.stream, (const float*)a.part_z,
                      (const float*)a.part_ml, a.seq_lens, (const bf16_t*)a.w_uv, (bf16_t*)a.out, a.lse, a.batch, a.h,
                      a.n_blocks, a.d_cb, a.plan.n_splits, a.plan.chunk_tokens, chunk_tab, a.out_scale,
                      (const bf16_t*)a.gate, direct, spw);
  else
    MLRA_LAUNCH_TIMED(a.t_epi, merge_upproj_mfma_kernel<float>, grid, dim3(256), lds, a.stream, (const float*)a.part_z,
                      (const float*)a.part_ml, a.seq_lens, (const bf16_t*)a.w_uv, (float*)a.out, a.lse, a.batch, a.h,
                      a.n_blocks, a.d_cb, a.plan.n_splits, a.plan.chunk_tokens, chunk_tab, a.out_scale,
                      (const bf16_t*)a.gate, direct, spw);
  return check_launch();
}

}  // namespace mlra
