// MFMA decode kernel for bf16 latent caches with d_cb = 128, d_r = 64 (Step 2 of the absorbed decode,
// Eq. (1), applied to one latent block; the blocks of Eq. (5) are spread over the grid).
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
//   * The queries carry tau log2(e), and the first MFMA of a tile's score chain starts from minus the
//     running maximum, so a probability is exp2 of what the matrix pipe delivers.
//   * Z^T and the row sums live in accumulation registers a0..a135 that only inline asm names (the MFMAs of
//     the main loop are asm statements); the compiler never sees them as values.
//   * The chunk's partial leaves as the normalised row z / l in bf16 with (m, l) in fp32 beside it (fp32,
//     un-normalised, for shapes whose epilogue is the generic merge kernel).
//
// PAIRED form, for blocks that serve 64 heads (MLRA-2, Eq. (6), at h = 128): one workgroup owns two
// neighbouring latent blocks and 64 heads.  The head half hw of a wave becomes its block: wave (hw, tw)
// runs block 2 pair + hw for all 64 heads on tokens [32 tw, +32).  Each wave does exactly the work it
// does in the plain form; the tile in LDS holds both blocks' latent rows and the shared RoPE rows
// (40 KiB per stage, four stages), so the RoPE rows are fetched once for the two branches.
//
// GLA form, for the GLA-2 baseline (Section 2.3, Eq. (3)-(4)): one latent head of 256 channels serves 64
// heads.  The workgroup is laid out as in the PAIRED form, but the two "blocks" are the two 128-channel
// halves of the one latent head: wave (hw, tw) computes the partial scores of its half (and of half of
// the RoPE channels), the two waves of a token half exchange their partial scores through LDS and add
// them (a + b and b + a are the same float, so both hold identical scores and take identical softmax
// decisions), and each then accumulates Z for its own 128 channels.  Three stages of 40 KiB plus a
// 32 KiB exchange buffer; two workgroup barriers per tile.
#include "mfma_tile.h"

#include <type_traits>

namespace mlra {
namespace {

using namespace mfma_tile;

// Sequence ids sorted by length, longest first (rank sort; ties keep index order).  Used when a launch has
// more workgroups than the chip runs at once: workgroups are dispatched in id order, so handing out
// the long sequences first is the longest-processing-time rule and keeps the last round short.
// group > 1 (several query tokens per sequence): entries [i group, i group + group) of seq_lens are the
// queries of one sequence, which read the same cache rows.  Whole sequences are ranked (by their longest
// query) and the queries of the sequence of rank r get the dispatch slots (r / 8) 8 group + 8 q + r % 8:
// the decode kernels put slot k on XCD k % 8 and slots of one run of 8 group side by side in time, so the
// queries of a sequence meet in one L2 and its rows come from HBM once.
__global__ __launch_bounds__(256) void seq_order_kernel(const int32_t* __restrict__ seq_lens,
                                                        int32_t* __restrict__ order, int n_seqs, int group) {
  extern __shared__ int32_t lens[];            // every length once, then the comparisons run out of LDS
  for (int j = threadIdx.x; j < n_seqs; j += 256) lens[j] = seq_lens[(size_t)j * group + group - 1];
  __syncthreads();
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i >= n_seqs) return;
  const int n = lens[i];
  int rank = 0;
  for (int j = 0; j < n_seqs; ++j) {
    const int nj = lens[j];
    rank += (nj > n || (nj == n && j < i)) ? 1 : 0;
  }
  const int full = n_seqs & ~7;                // ranks below this fill whole runs of 8 sequences
  for (int q = 0; q < group; ++q) {
    const int slot = rank < full ? (rank >> 3) * 8 * group + 8 * q + (rank & 7) : full * group + (rank - full) * group + q;
    order[slot] = i * group + q;
  }
}

// Chunk lengths that follow the sequence lengths.  With uniform chunks a ragged batch leaves workgroups
// idle (a sequence half as long as the longest uses half of its chunk slots); here sequence i gets
// S_i ~ target * n_i / sum(n) chunks of ceil(n_i / S_i) tokens (rounded up to the tile, at least
// min_chunk), so that about `target` chunks per block are active in total and they are about equally long.
// unit_tab lists the active (sequence, chunk) pairs, packed as sequence * 1024 + chunk, and -1 after
// them: workgroup ids go round-robin over the XCDs, so the active ones must be contiguous to spread
// evenly (scattered, they leave some XCDs with more work than CUs and others idle).  The pairs are listed
// longest chunk first (for batches of up to 512 sequences): when they need more than one round of
// workgroups, that is the longest-processing-time rule.  With single_if_uniform, a batch whose longest
// sequence is within 25 % of the mean keeps one chunk per sequence (cutting it would only add partials).
__global__ __launch_bounds__(256) void plan_chunks_kernel(const int32_t* __restrict__ seq_lens,
                                                          int32_t* __restrict__ chunk_tab,
                                                          int32_t* __restrict__ unit_tab, int batch, int target,
                                                          int max_slots, int min_chunk, int single_if_uniform) {
  __shared__ float part[4];
  __shared__ int part_max[4];
  __shared__ int wave_tot[4];
  extern __shared__ int32_t tab[];             // [batch] lengths, [batch] chunk lengths, [batch] dispatch order
  int32_t* lens = tab;
  int32_t* chunks = tab + batch;
  int32_t* order = tab + 2 * batch;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  float sum = 0.f;
  int longest = 0;
  for (int i = threadIdx.x; i < batch; i += 256) {
    lens[i] = seq_lens[i];
    sum += (float)lens[i];
    longest = max(longest, lens[i]);
  }
  // (lengths are integers below 2^31 and their partial sums are added in one fixed order)
  for (int o = 32; o > 0; o >>= 1) {
    sum += __shfl_xor(sum, o);
    longest = max(longest, __shfl_xor(longest, o));
  }
  if (lane == 0) { part[wave] = sum; part_max[wave] = longest; }
  __syncthreads();
  const float total = (part[0] + part[1]) + (part[2] + part[3]);
  longest = max(max(part_max[0], part_max[1]), max(part_max[2], part_max[3]));
  const bool single = single_if_uniform && (float)longest * (float)batch <= 1.25f * total;
  for (int i = threadIdx.x; i < batch; i += 256) {
    const int n = lens[i];
    int s_i = (total > 0.f && !single) ? (int)((float)target * (float)n / total + 0.5f) : 1;
    s_i = min(max(s_i, 1), max_slots);
    int chunk = (n + s_i - 1) / s_i;
    chunk = max(min_chunk, (chunk + kTile - 1) / kTile * kTile);
    chunks[i] = chunk;         // ceil(n / chunk) <= s_i <= max_slots
    chunk_tab[i] = chunk;
  }
  __syncthreads();
  // dispatch order: rank sort by chunk length, longest first (ties keep index order)
  for (int i = threadIdx.x; i < batch; i += 256) {
    int rank = i;
    if (batch <= 512) {
      const int c = chunks[i];
      rank = 0;
      for (int j = 0; j < batch; ++j) {
        const int cj = chunks[j];
        rank += (cj > c || (cj == c && j < i)) ? 1 : 0;
      }
    }
    order[rank] = i;
  }
  __syncthreads();
  // exclusive scan of the active chunk counts in dispatch order: 256 contiguous segments, one per thread
  const int per = (batch + 255) / 256, lo = min(batch, (int)threadIdx.x * per), hi = min(batch, lo + per);
  int mine = 0;
  for (int r = lo; r < hi; ++r) {
    const int i = order[r];
    mine += (lens[i] + chunks[i] - 1) / chunks[i];
  }
  // (scan over the 256 threads: inside a wave with shuffles, across the four waves through LDS)
  int incl = mine;
  for (int o = 1; o < 64; o <<= 1) {
    const int v = __shfl_up(incl, o);
    if (lane >= o) incl += v;
  }
  if (lane == 63) wave_tot[wave] = incl;
  __syncthreads();
  int u = incl - mine;
  for (int w = 0; w < wave; ++w) u += wave_tot[w];
  const int n_active = wave_tot[0] + wave_tot[1] + wave_tot[2] + wave_tot[3];
  for (int r = lo; r < hi; ++r) {
    const int i = order[r];
    const int active = (lens[i] + chunks[i] - 1) / chunks[i];
    for (int k = 0; k < active; ++k) unit_tab[u++] = i * 1024 + k;
  }
  for (int u = n_active + threadIdx.x; u < batch * max_slots; u += 256) unit_tab[u] = -1;
}


// ---- value accumulators in fixed accumulation registers ---------------------------------------------
// Z^T (four 32-channel x two 32-head tiles of fp32, 128 registers per lane) and the row sums l (two
// 16x16 tiles, 8 registers) live in a[0:135] for the whole chunk and are touched only by the inline asm
// below, by register NAME: tile (mt, nt) is a[16 (2 mt + nt) : +15], the row sums of head tile nt are
// a[128 + 4 nt : +3].  The compiler never sees them as values (left to it, it moved the 16-register
// tuples between loops with copies placed right behind MFMAs it cannot see, and ran out of accumulation
// registers for the queries); the clobber list keeps its own values out of these registers, and the
// build checks that no instruction outside the asm blocks names them.  An MFMA writes its result several
// passes after it issues: acc_settle() lets the last one retire before acc_read / acc_scale.
#define MLRA_ACC_CLOBBERS "a0","a1","a2","a3","a4","a5","a6","a7","a8","a9","a10","a11","a12","a13","a14","a15","a16","a17","a18","a19","a20","a21","a22","a23","a24","a25","a26","a27","a28","a29","a30","a31","a32","a33","a34","a35","a36","a37","a38","a39","a40","a41","a42","a43","a44","a45","a46","a47","a48","a49","a50","a51","a52","a53","a54","a55","a56","a57","a58","a59","a60","a61","a62","a63","a64","a65","a66","a67","a68","a69","a70","a71","a72","a73","a74","a75","a76","a77","a78","a79","a80","a81","a82","a83","a84","a85","a86","a87","a88","a89","a90","a91","a92","a93","a94","a95","a96","a97","a98","a99","a100","a101","a102","a103","a104","a105","a106","a107","a108","a109","a110","a111","a112","a113","a114","a115","a116","a117","a118","a119","a120","a121","a122","a123","a124","a125","a126","a127","a128","a129","a130","a131","a132","a133","a134","a135"
constexpr int kAccRegs = 136;
template <int TILE>
__device__ __forceinline__ void acc_pv_mfma(const bf16x8& vt, const bf16x8& pt) {   // Z^T tile += V^T P^T
  asm volatile("v_mfma_f32_32x32x16_bf16 a[%c2:%c3], %0, %1, a[%c2:%c3]"
               : : "v"(vt), "v"(pt), "n"(16 * TILE), "n"(16 * TILE + 15) : MLRA_ACC_CLOBBERS);
}
template <int NT>
__device__ __forceinline__ void acc_row_sum_mfma(const bf16x8& sel, const bf16x8& pt) {
  asm volatile("v_mfma_f32_16x16x32_bf16 a[%c2:%c3], %0, %1, a[%c2:%c3]"
               : : "v"(sel), "v"(pt), "n"(128 + 4 * NT), "n"(128 + 4 * NT + 3) : MLRA_ACC_CLOBBERS);
}
// all 136 registers to zero: products of a zero operand, no accumulator input
__device__ __forceinline__ void acc_zero(const bf16x8& zero) {
  // (the leading wait: the zero operand may have been written by the instruction just before this asm, and
  // nothing orders a vector write before an MFMA read that the compiler cannot see; measured: without it
  // the first tile came out as garbage)
  asm volatile(
      "s_nop 7\n\t"
      "v_mfma_f32_32x32x16_bf16 a[0:15], %0, %0, 0\n\tv_mfma_f32_32x32x16_bf16 a[16:31], %0, %0, 0\n\t"
      "v_mfma_f32_32x32x16_bf16 a[32:47], %0, %0, 0\n\tv_mfma_f32_32x32x16_bf16 a[48:63], %0, %0, 0\n\t"
      "v_mfma_f32_32x32x16_bf16 a[64:79], %0, %0, 0\n\tv_mfma_f32_32x32x16_bf16 a[80:95], %0, %0, 0\n\t"
      "v_mfma_f32_32x32x16_bf16 a[96:111], %0, %0, 0\n\tv_mfma_f32_32x32x16_bf16 a[112:127], %0, %0, 0\n\t"
      "v_mfma_f32_16x16x32_bf16 a[128:131], %0, %0, 0\n\tv_mfma_f32_16x16x32_bf16 a[132:135], %0, %0, 0\n\t"
      "s_nop 15\n\ts_nop 15"
      : : "v"(zero) : MLRA_ACC_CLOBBERS);
}
template <int REG>
__device__ __forceinline__ float acc_read() {
  float x;
  asm volatile("v_accvgpr_read_b32 %0, a%c1" : "=v"(x) : "n"(REG));
  return x;
}
// a[REG .. REG + COUNT) *= factor (per lane), one register at a time through one ordinary register
template <int REG, int COUNT>
__device__ __forceinline__ void acc_scale(float factor) {
  if constexpr (COUNT > 0) {
    float t;
    asm volatile("v_accvgpr_read_b32 %0, a%c2\n\tv_mul_f32 %0, %1, %0\n\tv_accvgpr_write_b32 a%c2, %0"
                 : "=&v"(t) : "v"(factor), "n"(REG) : MLRA_ACC_CLOBBERS);
    acc_scale<REG + 1, COUNT - 1>(factor);
  }
}
// four consecutive registers of tile (MT, NT) starting at element 4 R4
template <int MT, int NT, int R4>
__device__ __forceinline__ f32x4 acc_read4() {
  constexpr int base = 16 * (2 * MT + NT) + 4 * R4;
  return f32x4{acc_read<base>(), acc_read<base + 1>(), acc_read<base + 2>(), acc_read<base + 3>()};
}

template <int STAGES, int MODE>   // MODE 0: plain, 1: PAIRED, 2: GLA (see the head of the file)
__global__ __launch_bounds__(256) void decode_mfma_kernel(MfmaParams p) {
  extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
  constexpr bool PAIRED = MODE != 0;                        // two 128-channel latent tiles per stage, 64 heads
  constexpr bool GLA = MODE == 2;                           // ... that are the halves of one 256-channel block
  constexpr int kLatRow = GLA ? 2 * kDcb * 2 : kDcb * 2;    // bytes of one cached latent row of a block
  constexpr int kBlocksWG = PAIRED ? 2 : 1;                 // latent tiles that share a stage
  constexpr int kRopeOff = kBlocksWG * kLatBytes;           // RoPE tile behind the latent tile(s)
  constexpr int kStageB = kRopeOff + kRopeBytes;            // 24 KiB, or 40 KiB
  constexpr int kLoadsTile = 4 * kBlocksWG + 2;             // direct-to-LDS loads per wave and tile
  constexpr int kHeadsPerWG = PAIRED ? 64 : kHeadsWG;
  // Workgroup -> (sequence, chunk, block, head group).  The workgroups of one (sequence, chunk) read the
  // same RoPE rows (and, across head groups, the same latent rows).  Workgroup ids go round-robin over
  // the 8 XCDs, each with its own L2, so the members of such a family are given ids 8 apart: they land
  // on one XCD at about the same time and all but the first read of a shared row hit in that L2.
  const int n_hg = (p.h + kHeadsPerWG - 1) / kHeadsPerWG;
  const int fam = (GLA ? p.n_blocks : p.n_blocks / kBlocksWG) * n_hg;
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
  const int hgrp = member % n_hg;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int hw = wave & 1, tw = wave >> 1, g = lane >> 5, c32 = lane & 31;
  const int blk0 = member / n_hg * (GLA ? 1 : kBlocksWG);   // first (or only) block of this workgroup
  const int blk = (PAIRED && !GLA) ? blk0 + hw : blk0;      // this wave's block
  const int wave_head0 = PAIRED ? hgrp * 64 : hgrp * kHeadsWG + hw * 64;   // this wave's first head

  // ---- absorbed + RoPE queries: MFMA B operands, resident in accumulation registers for the whole chunk
  // (MFMA reads its B operand from there directly, which leaves the architectural VGPRs to the per-tile
  // working set).  They travel global -> LDS -> registers: the workgroup's 128 q_abs rows (256 B each) and
  // its RoPE query rows (128 B each) are fetched once with direct-to-LDS loads into the end of the tile
  // buffer, which the first tiles do not need yet, and every wave then reads its own B operands from
  // there (the two waves of a head half would otherwise both fetch the same 24 KiB from L2).  16-byte
  // chunk c of q_abs row r sits at chunk position c ^ (r & 15), chunk c of RoPE row r at c ^ ((r >> 1) & 7):
  // the 16 lanes that a 128-bit LDS read serves together then hit 16 different bank groups.
  constexpr int kQRopeRows = PAIRED ? 64 : kHeadsWG;
  constexpr int kQBytes = kHeadsWG * (kDcb * 2) + kQRopeRows * (kDr * 2);     // 48 KiB, or 40 KiB
  constexpr int kQStages = (kQBytes + kStageB - 1) / kStageB;                 // stages the queries occupy
  const unsigned lds_base = (unsigned)(size_t)(__attribute__((address_space(3))) unsigned char*)smem;
  const unsigned wave_u = __builtin_amdgcn_readfirstlane(wave);
  const unsigned q_lds = lds_base + STAGES * kStageB - kQBytes;
  const int grp_head0 = (blk0 / (p.n_blocks / p.groups)) * p.h;   // first head of this block's group in q_rope
  {
#pragma unroll
    for (int q = 0; q < 8; ++q) {                                  // q_abs rows 32 w + 4 q + lane / 16
      const int row = 32 * wave + 4 * q + (lane >> 4);
      const int row_blk = (PAIRED && !GLA) ? blk0 + (row >> 6) : blk0;
      const int head = min(PAIRED ? hgrp * 64 + (row & 63) : hgrp * kHeadsWG + row, p.h - 1);
      // (GLA: LDS rows 64..127 hold channels 128..255 of the same 64 heads)
      const unsigned voff = ((unsigned)(seq * p.n_blocks + row_blk) * p.h + head) * kLatRow +
                            (GLA ? (row >> 6) * (kDcb * 2) : 0) + (((lane & 15) ^ (row & 15)) << 4);
      set_m0(q_lds + (32 * wave_u + 4 * q) * (kDcb * 2));
      lds_dma16<0>(p.q_abs, voff);
    }
#pragma unroll
    for (int q = 0; q < kQRopeRows / 32; ++q) {                    // RoPE rows (rows per wave) w + 8 q + lane / 8
      const int row = (kQRopeRows / 4) * wave + 8 * q + (lane >> 3);
      const int head = min(hgrp * kHeadsPerWG + row, p.h - 1);
      const unsigned voff = ((unsigned)seq * p.h * p.groups + grp_head0 + head) * (kDr * 2) +
                            (((lane & 7) ^ ((row >> 1) & 7)) << 4);
      set_m0(q_lds + kHeadsWG * (kDcb * 2) + ((kQRopeRows / 4) * wave_u + 8 * q) * (kDr * 2));
      lds_dma16<0>(p.q_rope, voff);
    }
  }

  const int t0 = split * chunk_len;
  // page id of the first tile, fetched before the sequence length is known (the index is in range for
  // any length)
  typedef const __attribute__((address_space(4))) int32_t* const_i32_ptr;
  const const_i32_ptr pt_row = (const_i32_ptr)(p.page_table + (size_t)seq * p.max_pages);
  // (pages hold a multiple of 16 tokens and chunks start on multiples of 64, so the 16 rows that a wave
  // loads of each tile lie in one page: the page ids below are this wave's; with pages of 16 or 32 tokens
  // the four waves of a tile read different pages)
  int issue_page_idx = (t0 + 16 * (int)wave_u) / p.page_size;
  int issue_page = pt_row[min(issue_page_idx, p.max_pages - 1)];
  const int n = ((const_i32_ptr)p.seq_lens)[seq];
  if (t0 >= n) {
    wait_vmcnt<0>();   // the query loads target this workgroup's LDS: let them land before it is released
    return;
  }
  const int t1 = min(n, t0 + chunk_len);
  const int ntiles = (t1 - t0 + kTile - 1) / kTile;
  const int nvalid_last = t1 - t0 - (ntiles - 1) * kTile;

  // ---- tile order.  Only the chunk's last tile can be ragged, and softmax does not care about the order
  // of the tokens, so that tile is processed FIRST: it is issued and masked in the prologue, and every
  // tile that the main loop issues is a full one (straight-line code, no masks in the loop).  Processing
  // index 0 is the chunk's last tile, processing index jj >= 1 its tile jj - 1.

  // ---- page ids: scalar loads through the constant address space (the table is read-only here), so
  // that the compiler's vector-memory wait counts never see a load inside the main loop: a wait for one
  // would also drain every direct-to-LDS load in flight.  The id of the next tile's page is fetched one
  // tile ahead of its use.

  // ---- tile loads.  Wave w fills LDS chunks [256 w, 256 w + 256) of the latent tile with four loads
  // and chunks [128 w, 128 w + 128) of the RoPE tile with two; load q of a wave sits 1024 bytes after
  // load q-1 both in LDS and (four latent rows / eight RoPE rows further) in global memory, so the
  // instruction offset covers it and only the swizzle of the row changes the lane offset.
  unsigned lat_voff[4], rope_voff[2];
#pragma unroll
  for (int q = 0; q < 4; ++q)
    // (the instruction offset 1024 q moves both sides; rows twice as long need the rest of the step here)
    lat_voff[q] = (lane >> 4) * kLatRow + (((lane & 15) ^ lat_swz(4 * q + (lane >> 4))) << 4) +
                  q * (4 * kLatRow - 1024);
#pragma unroll
  for (int q = 0; q < 2; ++q)
    rope_voff[q] = (lane >> 3) * (kDr * 2) + (((lane & 7) ^ rope_swz(8 * q + (lane >> 3))) << 4);
  // (bytes of one page: below 2^32, checked by the launcher, so page id x bytes is one 32 x 32 -> 64 bit product)
  const unsigned lat_page_bytes = (unsigned)p.n_blocks * (unsigned)p.page_size * (unsigned)kLatRow;
  const unsigned rope_page_bytes = (unsigned)p.page_size * (unsigned)(kDr * 2);
  const size_t lat_plane_bytes = (size_t)p.page_size * kLatRow;        // one block's rows inside a page
  const size_t lat_half_step = GLA ? kDcb * 2 : lat_plane_bytes;       // from the first latent tile's source to the second's
  const char* lat_blk = (const char*)p.latent + (size_t)blk0 * lat_plane_bytes;
  // slot, inside its page, of this wave's first row of the next full tile to issue (they go in order)
  int issue_slot = (t0 + 16 * (int)wave_u) % p.page_size;
  int issue_stage = 0;

  // A full tile is issued in parts so that the parts can sit behind different MFMAs: issue_begin (scalar
  // address work), six loads, issue_end (bookkeeping, next page id).
  const char* iss_lat = nullptr;
  const char* iss_rope = nullptr;
  unsigned iss_stage = 0;
  auto issue_begin = [&](unsigned stage_off) {   // stage_off: byte offset of the stage that receives the tile
    const unsigned page = (unsigned)issue_page;
    // start of this wave's 16 latent rows (block plane blk0) and RoPE rows of the tile inside the page
    iss_lat = lat_blk + (unsigned long long)page * lat_page_bytes + (unsigned)issue_slot * (unsigned)kLatRow;
    iss_rope = (const char*)p.rope + (unsigned long long)page * rope_page_bytes + (unsigned)issue_slot * (unsigned)(kDr * 2);
    iss_stage = lds_base + stage_off;
  };
  // parts 0..3 = latent loads (PAIRED: 4..7 = the second block's), then two RoPE loads
  auto issue_full_part = [&](int part) {
    if (part < 4 * kBlocksWG) {
      const int jb = part >> 2, q = part & 3;
      const char* src = iss_lat + jb * lat_half_step;
      if (q == 0) set_m0(iss_stage + jb * kLatBytes + wave_u * 4096);
      if (q == 0) lds_dma16<0>(src, lat_voff[0]);
      if (q == 1) lds_dma16<1024>(src, lat_voff[1]);
      if (q == 2) lds_dma16<2048>(src, lat_voff[2]);
      if (q == 3) lds_dma16<3072>(src, lat_voff[3]);
    } else {
      const int q = part - 4 * kBlocksWG;
      if (q == 0) set_m0(iss_stage + kRopeOff + wave_u * 2048);
      if (q == 0) lds_dma16<0>(iss_rope, rope_voff[0]);
      if (q == 1) lds_dma16<1024>(iss_rope, rope_voff[1]);
    }
  };
  auto issue_end = [&]() {
    issue_slot += kTile;
    if (issue_slot >= p.page_size) {
      do {                       // (up to four pages further with 16-token pages)
        issue_slot -= p.page_size;
        ++issue_page_idx;
      } while (issue_slot >= p.page_size);
      issue_page = pt_row[min(issue_page_idx, p.max_pages - 1)];
    }
  };
  auto issue_tile = [&]() {   // a whole full tile at once (prologue)
    issue_begin(issue_stage * kStageB);
#pragma unroll
    for (int part = 0; part < kLoadsTile; ++part) issue_full_part(part);
    issue_end();
    issue_stage = (issue_stage + 1 == STAGES) ? 0 : issue_stage + 1;
  };
  // The chunk's last tile, into the current stage: rows past the chunk's end re-read its last valid row
  // (finite values; their probabilities are masked to zero).  The rows of this wave that exist lie in its
  // own page; if none exists, every lane reads the tile's last valid row, whose page may be another one
  // (pages shorter than a tile).  Leaves the page bookkeeping of the full tiles untouched.
  auto issue_last_tile = [&]() {
    const int last = nvalid_last - 1;                // last valid row of the tile, 0..63
    const int w0 = 16 * (int)wave_u;                 // first tile row of this wave
    const int first = w0 > last ? last : w0;         // the tile row that src_lat / src_rope point at
    const int tok = t0 + (ntiles - 1) * kTile + first;
    const int idx = tok / p.page_size, slot = tok - idx * p.page_size;
    const unsigned page = (unsigned)pt_row[idx];
    const char* src_lat = lat_blk + (unsigned long long)page * lat_page_bytes + (unsigned)slot * (unsigned)kLatRow;
    const char* src_rope = (const char*)p.rope + (unsigned long long)page * rope_page_bytes + (unsigned)slot * (unsigned)(kDr * 2);
    const unsigned stage = lds_base + issue_stage * kStageB;
#pragma unroll
    for (int jb = 0; jb < kBlocksWG; ++jb)
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int t = (wave * 4 + q) * 4 + (lane >> 4);          // 0..63
        const unsigned row = (unsigned)(min(t, last) - first);   // rows from src_lat, never negative
        set_m0(stage + jb * kLatBytes + wave_u * 4096 + q * 1024);
        lds_dma16<0>(src_lat + jb * lat_half_step, row * kLatRow + (((lane & 15) ^ lat_swz(t)) << 4));
      }
#pragma unroll
    for (int q = 0; q < 2; ++q) {
      const int t = (wave * 2 + q) * 8 + (lane >> 3);          // 0..63
      const unsigned row = (unsigned)(min(t, last) - first);
      set_m0(stage + kRopeOff + wave_u * 2048 + q * 1024);
      lds_dma16<0>(src_rope, row * (kDr * 2) + (((lane & 7) ^ rope_swz(t)) << 4));
    }
    issue_stage = (issue_stage + 1 == STAGES) ? 0 : issue_stage + 1;
  };

  // ---- per-lane LDS read offsets inside a stage.  The swizzle is an XOR on the chunk index, so the
  // offsets of the 12 score reads (and of the 16 transpose reads) of a lane differ from one base offset
  // by XORs with constants and by multiples of 2 KiB: four registers hold them all.  (Stage starts are
  // multiples of 8 KiB and the LDS buffer is 1 KiB aligned, so the XORs commute with adding them.) ----
  const int s_tok = tw * 32 + c32;
  const unsigned own_lat = PAIRED ? hw * kLatBytes : 0;   // this wave's block inside a stage
  const unsigned k_lat_off = own_lat + s_tok * (kDcb * 2) + ((g ^ lat_swz(s_tok)) << 4);      // ^ (ks << 5)
  const unsigned k_rope_off = kRopeOff + s_tok * (kDr * 2) + ((g ^ rope_swz(s_tok)) << 4);    // ^ (ks << 5)
  unsigned v_off[2];                                                          // ^ (mt << 6), + 4096 ss
  {
    const int k = (lane & 15) >> 2, seg = lane & 3, hb = (lane >> 4) & 1;
#pragma unroll
    for (int half = 0; half < 2; ++half) {
      const int ta = tw * 32 + 8 * half + 4 * g + k;
      v_off[half] = own_lat + ta * (kDcb * 2) + (((2 * hb + (seg >> 1)) ^ lat_swz(ta)) << 4) + ((seg & 1) << 3);
    }
  }

  // Running reference maximum of each head column (log2 domain) and, as 16-register vectors, its negative:
  // the first score MFMA of a tile takes that vector as its accumulator input, so the scores come out of
  // the matrix pipe already relative to the reference and feed exp2 directly.  (GLA: the two waves whose
  // partial scores are added each start from half of it; halving is exact.)
  float m_run[2] = {0.f, 0.f};
  f32x16 negm[2];
  // Row sums l = sum_t P[t][head] come from the matrix pipe as well: one 16x16x32 MFMA per P^T operand
  // with a 0/1 selector as A.  Read as a 16x16x32 B operand, lane (16 b + c) of a P^T register holds head
  // c + 16 (b & 1), eight tokens; selector row 4 q has ones where (b & 1) == (q & 1), every other row is
  // zero, so accumulator register 0 of lane (16 q + c) ends up with the sum over the operand's 16 tokens
  // of that lane's own head, both token halves included.
  bf16x8 row_sel;
  {
    const int i = lane & 15, b = lane >> 4;
    const __bf16 v = ((i & 3) == 0 && ((i >> 2) & 1) == (b & 1)) ? (__bf16)1.0f : (__bf16)0.0f;
#pragma unroll
    for (int e = 0; e < 8; ++e) row_sel[e] = v;
  }
  const float sc = p.scale_log2;

  typedef const __attribute__((address_space(3))) bf16x8* lds_bf16x8_ptr;
  typedef const __attribute__((address_space(3))) unsigned char* lds_byte_ptr;
  // K operand ks (this wave's 32 token rows x 16 channels) of the tile in the stage at byte offset st_off
  auto load_k_part = [&](unsigned st_off, int ks, bf16x8 (&ka)[12]) {
    const unsigned base = lds_base + st_off + (ks < 8 ? k_lat_off : k_rope_off);
    ka[ks] = *(lds_bf16x8_ptr)(size_t)(base ^ ((ks & 7) << 5));
  };
  auto load_k = [&](unsigned st_off, bf16x8 (&ka)[12]) {
#pragma unroll
    for (int ks = 0; ks < 12; ++ks) load_k_part(st_off, ks, ka);
  };
  // transposed V operand (32 channels of tile mt x 16 of this wave's token rows) of the tile in that stage
  auto load_v_part = [&](unsigned st_off, int ss, int mt, bf16x8 (&va)[2][4]) {
    const unsigned lo_base = lds_base + st_off + v_off[0];
    const unsigned hi_base = lds_base + st_off + v_off[1];
    const lds_byte_ptr lo_p = (lds_byte_ptr)(size_t)(lo_base ^ (mt << 6));
    const lds_byte_ptr hi_p = (lds_byte_ptr)(size_t)(hi_base ^ (mt << 6));
    const short4v lo = lds_tr16(lo_p + ss * 16 * (kDcb * 2));
    const short4v hi = lds_tr16(hi_p + ss * 16 * (kDcb * 2));
    va[ss][mt] = __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
  };
  // Column maxima.  In the accumulator layout a lane holds 16 of the 32 token rows of its head column
  // and the lane 32 away holds the other 16.  max8 folds eight more rows into a running maximum;
  // cross_max finishes both head tiles at once with two half-wave swaps (v_permlane32_swap exchanges
  // the upper half of its first operand with the lower half of its second).
  // (v_max3 through asm: the library fmaxf would first canonicalise every operand, one more
  // instruction each; four of them in one statement, because the compiler separates dependent asm
  // statements by a wait state each.  The operands are score accumulators whose MFMAs retired several
  // MFMAs earlier.)
  auto max8 = [&](float mx, const f32x16& sv, int r) {
    float res;
    asm("v_max3_f32 %0, %1, %2, %3\n\t"
        "v_max3_f32 %0, %0, %4, %5\n\t"
        "v_max3_f32 %0, %0, %6, %7\n\t"
        "v_max3_f32 %0, %0, %8, %9"
        : "=&v"(res)
        : "v"(mx), "v"(sv[r]), "v"(sv[r + 1]), "v"(sv[r + 2]), "v"(sv[r + 3]), "v"(sv[r + 4]), "v"(sv[r + 5]),
          "v"(sv[r + 6]), "v"(sv[r + 7]));
    return res;
  };
  auto swap_halves = [&](float& a, float& b) {
    asm volatile("s_nop 1\n\tv_permlane32_swap_b32 %0, %1\n\ts_nop 1" : "+v"(a), "+v"(b));
  };
  auto cross_max = [&](float& mx0, float& mx1) {
    swap_halves(mx0, mx1);            // mx0 = {tile 0 lower, tile 1 lower}, mx1 = {tile 0 upper, tile 1 upper}
    asm("v_max_f32 %0, %0, %1" : "+v"(mx0) : "v"(mx1));   // lanes 0..31: maxima of head tile 0, 32..63: of head tile 1
    mx1 = mx0;
    swap_halves(mx0, mx1);            // mx0 = tile 0 maxima in both halves, mx1 = tile 1 maxima in both halves
  };
  auto col_max2 = [&](const f32x16& s0, const f32x16& s1, float& mx0, float& mx1) {
    mx0 = max8(max8(s0[0], s0, 0), s0, 8);
    mx1 = max8(max8(s1[0], s1, 0), s1, 8);
    cross_max(mx0, mx1);
  };
  // Operands of the PV MFMAs (transposed value tiles, bf16 probabilities).  They live at function scope
  // because of a hardware rule the compiler cannot apply to asm: an MFMA goes on reading its source
  // registers for a while after it has issued, so nothing may be written to them for the next few MFMAs
  // (measured: exponentials landing in a K operand two instructions after its last score MFMA corrupted
  // that MFMA's result).  hold() marks a register as still in use at the point where it is written: the
  // allocator cannot hand it to another value before that.  Every asm MFMA's source is held until at
  // least four MFMAs after the instruction that reads it last, across step boundaries too.
  bf16x8 va[2][4], pb0[2], pb1[2];
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    const __bf16 zero = (__bf16)0.0f;
    va[1][2][e] = zero; va[1][3][e] = zero; pb0[1][e] = zero; pb1[1][e] = zero;
  }
  acc_zero(pb0[1]);
  auto hold = [&](const bf16x8& x) { asm volatile("" : : "v"(x)); };
  auto settle_acc = [&]() {   // (the operands of the last PV MFMAs stay put meanwhile)
    asm volatile("s_nop 15\n\ts_nop 15" : : "v"(va[1][2]), "v"(va[1][3]), "v"(pb0[1]), "v"(pb1[1]) : MLRA_ACC_CLOBBERS);
  };
  // Moves the reference maximum of head tile nt up by d >= 0 (per lane: 0 for heads that keep theirs):
  // the history (Z, l) is weighted down by 2^-d, and the scores of the next tile, which the matrix pipe
  // has already produced relative to the old reference, are shifted.  (Rare; call settle_acc first.)
  auto rescale = [&](auto nt_tag, float d, f32x16& next_scores) {
    constexpr int nt = decltype(nt_tag)::value;
    const float alpha = __builtin_amdgcn_exp2f(-d);
    acc_scale<16 * (0 + nt), 16>(alpha);
    acc_scale<16 * (2 + nt), 16>(alpha);
    acc_scale<16 * (4 + nt), 16>(alpha);
    acc_scale<16 * (6 + nt), 16>(alpha);
    acc_scale<128 + 4 * nt, 1>(alpha);
    asm volatile("s_nop 7" : : : MLRA_ACC_CLOBBERS);   // the register writes above precede the next MFMA that reads them
    const float dh = GLA ? 0.5f * d : d;
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      next_scores[i] -= d;
      negm[nt][i] -= dh;
    }
    m_run[nt] += d;
    asm volatile("s_nop 7" : "+v"(negm[nt]));   // written just now, read by the next step's first score MFMA
  };
  // P^T = 2^score for two consecutive accumulator rows of a head tile (the scores are already relative to
  // the reference maximum) and their rounding to bf16 into the PV B operand: two pieces, so that the
  // rounding can sit one MFMA after the exponentials it consumes.
  auto prob_exp = [&](const f32x16& sv, int r, float& p0, float& p1) {
    p0 = __builtin_amdgcn_exp2f(sv[r]);
    p1 = __builtin_amdgcn_exp2f(sv[r + 1]);
    asm volatile("" : "+v"(p0), "+v"(p1));   // computed here, not sunk to the first use
  };
  // Row sums and Z^T += V^T P^T on the fixed accumulation registers (see acc_pv_mfma).  A tile is read and
  // written only by its own MFMAs (eight MFMAs apart); the A operand comes from LDS reads that the compiler
  // waits for (it sees the register dependence), the B operand from conversions issued at least eight
  // MFMAs earlier.
  auto row_sum_mfma = [&](int nt, const bf16x8& pt) {
    if (nt == 0) acc_row_sum_mfma<0>(row_sel, pt); else acc_row_sum_mfma<1>(row_sel, pt);
  };
  auto pv_mfma = [&](int mt, int nt, const bf16x8& vt, const bf16x8& pt) {
    switch (2 * mt + nt) {   // (a constant once the step is unrolled)
      case 0: acc_pv_mfma<0>(vt, pt); break;
      case 1: acc_pv_mfma<1>(vt, pt); break;
      case 2: acc_pv_mfma<2>(vt, pt); break;
      case 3: acc_pv_mfma<3>(vt, pt); break;
      case 4: acc_pv_mfma<4>(vt, pt); break;
      case 5: acc_pv_mfma<5>(vt, pt); break;
      case 6: acc_pv_mfma<6>(vt, pt); break;
      default: acc_pv_mfma<7>(vt, pt); break;
    }
  };
  // S^T += K Q^T for one 32-token x 32-head tile and 16 channels.  asm, so that the register classes are
  // fixed: the K operand and the scores in ordinary registers, the query operand in the accumulation file
  // (left to itself the allocator spreads LDS results over both files and then has no accumulation
  // registers left for the queries).  score_first starts a tile's chain from minus the reference maximum.
  // The scores are next read eight or more MFMAs after the chain's last instruction (column maxima) and a
  // whole step later (exponentials), so no wait is needed here; the GLA form, which stores them to LDS at
  // once, waits explicitly.
  auto score_mfma = [&](f32x16& acc, const bf16x8& kt, const bf16x8& qt) {
    asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(acc) : "v"(kt), "a"(qt));
  };
  auto score_first = [&](f32x16& acc, const bf16x8& kt, const bf16x8& qt, const f32x16& init) {
    asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %3" : "=&v"(acc) : "v"(kt), "a"(qt), "v"(init));
  };
  auto prob_pack = [&](int r, float p0, float p1, bf16x8 (&pb)[2]) {
    bf16x2 pp = {(__bf16)p0, (__bf16)p1};
    asm volatile("" : "+v"(pp));
    pb[r >> 3][r & 7] = pp[0];
    pb[r >> 3][(r & 7) + 1] = pp[1];
  };
  auto mask_tail = [&](f32x16& sv) {
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int tok = tw * 32 + (r >> 2) * 8 + g * 4 + (r & 3);
      if (tok >= nvalid_last) sv[r] = -INFINITY;
    }
  };

  // ---- prologue: every stage gets a tile; scores and column maxima of tile 0; K operands of tile 1 ----
  bf16x8 qreg[2][12];
  issue_last_tile();
  for (int jj = 1; jj < STAGES - kQStages && jj < ntiles; ++jj) issue_tile();
  if (GLA && tid < 4) ((float*)(smem + STAGES * kStageB))[tid] = 0.f;   // the zeros some RoPE reads below take
  // queries landed (they are older than the tile loads; vector-memory operations retire in order) ...
  if (ntiles >= STAGES - kQStages) wait_vmcnt<kLoadsTile * (STAGES - kQStages)>(); else wait_vmcnt<0>();
  __builtin_amdgcn_s_barrier();   // ... in every wave's share
  // The factor tau * log2(e) goes into the queries, once, so that the matrix pipe delivers scores in the
  // log2 domain: each query element is multiplied in fp32 and rounded to bf16 again (queries that arrive
  // already multiplied, scale_log2 == 1, go straight from LDS into the accumulation registers).
  const bool q_ready = sc == 1.0f;
#pragma unroll
  for (int nt = 0; nt < 2; ++nt) {
    const int row = hw * 64 + nt * 32 + c32;                       // q_abs row of this lane's head column
    const int rrow = PAIRED ? nt * 32 + c32 : row;                 // its RoPE row
    unsigned qaddr[12];
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) qaddr[ks] = q_lds + row * (kDcb * 2) + (((2 * ks + g) ^ (row & 15)) << 4);
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      const unsigned addr = q_lds + kHeadsWG * (kDcb * 2) + rrow * (kDr * 2) + (((2 * ks + g) ^ ((rrow >> 1) & 7)) << 4);
      // GLA: the RoPE channels are split between the two waves whose partial scores are added, so that
      // the RoPE term is counted once; the other wave's channels are read from 16 bytes of zeros
      qaddr[8 + ks] = (!GLA || (ks >> 1) == hw) ? addr : lds_base + STAGES * kStageB;
    }
    bf16x8 raw[12];
#pragma unroll
    for (int ks = 0; ks < 12; ++ks) raw[ks] = *(lds_bf16x8_ptr)(size_t)qaddr[ks];
    if (!q_ready) {
#pragma unroll
      for (int ks = 0; ks < 12; ++ks)
#pragma unroll
        for (int e = 0; e < 8; ++e) raw[ks][e] = (__bf16)((float)raw[ks][e] * sc);
    }
#pragma unroll
    for (int ks = 0; ks < 12; ++ks) {
      asm volatile("" : "+a"(raw[ks]));   // into the accumulation file, where the score MFMAs read it
      qreg[nt][ks] = raw[ks];
    }
  }
  // every wave has its queries in registers before the stages under them are refilled
  __builtin_amdgcn_s_barrier();
  for (int jj = STAGES - kQStages; jj < STAGES && jj < ntiles; ++jj) issue_tile();
  if (ntiles >= STAGES) wait_vmcnt<kLoadsTile * (STAGES - 2)>(); else wait_vmcnt<0>();
  __builtin_amdgcn_s_barrier();   // tiles 0 and 1 landed for every wave
  f32x16 sa0, sa1, sb0, sb1;
  bf16x8 ka[12];
  {
    load_k(0, ka);
#pragma unroll
    for (int i = 0; i < 16; ++i) { sa0[i] = 0.f; sa1[i] = 0.f; }
#pragma unroll
    for (int ks = 0; ks < 12; ++ks) {
      sa0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka[ks], qreg[0][ks], sa0, 0, 0, 0);
      sa1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka[ks], qreg[1][ks], sa1, 0, 0, 0);
      if (ks == 1) asm volatile("" : : "v"(ka[0]));   // see the main loop
    }
    // the maxima read the accumulators through asm, which the compiler's MFMA hazard bookkeeping does
    // not see: let the last score MFMA retire first
    asm volatile("s_nop 15\n\ts_nop 15" : "+v"(sa0), "+v"(sa1));
    if (GLA) {   // add the partner's partial scores of tile 0 (as in the main loop)
      f32x4* const xb = (f32x4*)(smem + STAGES * kStageB);
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        xb[(wave * 8 + i) * 64 + lane] = f32x4{sa0[4 * i], sa0[4 * i + 1], sa0[4 * i + 2], sa0[4 * i + 3]};
        xb[(wave * 8 + 4 + i) * 64 + lane] = f32x4{sa1[4 * i], sa1[4 * i + 1], sa1[4 * i + 2], sa1[4 * i + 3]};
      }
      __syncthreads();
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        f32x4 x0 = xb[((wave ^ 1) * 8 + i) * 64 + lane], x1 = xb[((wave ^ 1) * 8 + 4 + i) * 64 + lane];
        asm volatile("" : "+v"(x0), "+v"(x1));
#pragma unroll
        for (int e = 0; e < 4; ++e) { sa0[4 * i + e] += x0[e]; sa1[4 * i + e] += x1[e]; }
      }
      __syncthreads();
    }
    float mx0, mx1;
    col_max2(sa0, sa1, mx0, mx1);
    m_run[0] = mx0;
    m_run[1] = mx1;
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      sa0[i] -= mx0;
      sa1[i] -= mx1;
      negm[0][i] = GLA ? -0.5f * mx0 : -mx0;
      negm[1][i] = GLA ? -0.5f * mx1 : -mx1;
    }
    // Rows past the end of the ragged tile hold copies of its last valid row: their scores equal a valid
    // score, so the maxima above were right without a mask (and finite even for a wave none of whose rows
    // exists); their probabilities are what has to vanish.
    if (nvalid_last < kTile) { mask_tail(sa0); mask_tail(sa1); }
    __builtin_amdgcn_sched_barrier(0);
    load_k((1 % STAGES) * kStageB, ka);   // (a stale stage if the chunk has a single tile: those scores are never used)
  }

  // ---- main loop, software-pipelined over tiles; every MFMA is followed by about six issue slots of
  // other work, which is what the matrix pipe hides.  Step j:
  //   block A: scores of tile j+1 (n0, n1; K operands were fetched during the previous step) on the
  //            matrix pipe  ||  probabilities of tile j from its scores (c0, c1) and the LDS transpose
  //            reads of V(j) on the other pipes;
  //   block B: Z += V(j)^T P(j)^T on the matrix pipe  ||  wait for tile j+2 + workgroup barrier, loads of
  //            tile j+STAGES into the stage tile j leaves, K operands of tile j+2, column maxima of
  //            tile j+1.
  // The barrier says two things: tile j+2 is visible to every wave, and every wave has finished its LDS
  // reads of tile j (V, this step) and tile j+1 (K, previous step).  (Tiles are counted in processing
  // order: tile 0 is the chunk's last one.)  Issuing steps load a tile that exists and is full, so they are
  // straight-line code; the last STAGES steps of a chunk issue nothing.  sched_barrier(0) pins the
  // interleaving. ----
  // (the ring position is kept as a byte offset: no multiplication per step.  A step's loads go into the
  // stage of the tile it consumes, tile j + STAGES into the stage of tile j.)
  unsigned st_cur = 0;
  auto step = [&](auto issue_tag, int j, f32x16& c0, f32x16& c1, f32x16& n0, f32x16& n1) {
    constexpr bool ISSUE = decltype(issue_tag)::value;   // tile j + STAGES exists (and is a full one)
    const bool has_next = j + 1 < ntiles;
    const unsigned st_k2 = (st_cur + 2 * kStageB >= STAGES * kStageB) ? st_cur + 2 * kStageB - STAGES * kStageB
                                                                       : st_cur + 2 * kStageB;   // stage of tile j+2

    __builtin_amdgcn_sched_barrier(0);
    // ---- block A: 24 score MFMAs; the first of each head tile starts from minus the reference maximum.
    // MFMA i < 16 carries the exponentials of probability pair i (pairs 0..7: head tile 0, 8..15: head
    // tile 1) and the bf16 rounding of pair i-1; MFMA 16+q carries the LDS transpose reads of V operand q.
    // (Measured: moving the roundings behind the MFMAs of the transpose reads instead costs 25 cycles per tile.)
    float pr[4];
#pragma unroll
    for (int i = 0; i < 24; ++i) {
      const int ks = i >> 1;
      if (i == 0) score_first(n0, ka[0], qreg[0][0], negm[0]);
      else if (i == 1) score_first(n1, ka[0], qreg[1][0], negm[1]);
      else if ((i & 1) == 0) score_mfma(n0, ka[ks], qreg[0][ks]);
      else score_mfma(n1, ka[ks], qreg[1][ks]);
      // sources of earlier MFMAs that may be reused from here on (see hold above): the PV operands of the
      // previous step's last MFMAs, and each K operand four MFMAs after the pair that read it
      if (i == 3) { hold(va[1][2]); hold(va[1][3]); hold(pb0[1]); hold(pb1[1]); }
      if (i >= 5 && (i & 1) == 1) hold(ka[(i >> 1) - 2]);
      if (i < 16) {
        if (i < 8) prob_exp(c0, 2 * i, pr[2 * (i & 1)], pr[2 * (i & 1) + 1]);
        else prob_exp(c1, 2 * (i - 8), pr[2 * (i & 1)], pr[2 * (i & 1) + 1]);
      }
      if (i >= 1 && i <= 16) {
        const int pi = i - 1;   // the pair whose exponentials went out behind the previous MFMA
        if (pi < 8) prob_pack(2 * pi, pr[2 * (pi & 1)], pr[2 * (pi & 1) + 1], pb0);
        else prob_pack(2 * (pi - 8), pr[2 * (pi & 1)], pr[2 * (pi & 1) + 1], pb1);
      }
      if (i >= 16) {
        const int q = i - 16;
        load_v_part(st_cur, q >> 2, q & 3, va);
      }
      __builtin_amdgcn_sched_barrier(0);
    }

    // GLA: this wave's partial scores of tile j+1 go to the exchange buffer (complete only now: the
    // stores wait for the last score MFMA); the partner's are added behind MFMAs 2..5 below
    f32x4* const xbuf = (f32x4*)(smem + STAGES * kStageB);   // [4 waves][8][64 lanes] x 16 bytes
    if (GLA) {
      asm volatile("s_nop 15\n\ts_nop 15" : "+v"(n0), "+v"(n1));   // the last score MFMAs have retired
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        xbuf[(wave * 8 + i) * 64 + lane] = f32x4{n0[4 * i], n0[4 * i + 1], n0[4 * i + 2], n0[4 * i + 3]};
        xbuf[(wave * 8 + 4 + i) * 64 + lane] = f32x4{n1[4 * i], n1[4 * i + 1], n1[4 * i + 2], n1[4 * i + 3]};
      }
    }
    // ---- block B: 16 MFMAs (m = 0..15: ss = m / 8, mt = (m / 2) % 4, nt = m % 2)
    float mx0 = 0.f, mx1 = 0.f;
    bool need_any = false;
#pragma unroll
    for (int m = 0; m < 16; ++m) {
      const int ss = m >> 3, mt = (m >> 1) & 3;
      if ((m & 1) == 0) pv_mfma(mt, 0, va[ss][mt], pb0[ss]);
      else pv_mfma(mt, 1, va[ss][mt], pb1[ss]);
      if (m == 0 || m == 8) {
        row_sum_mfma(0, pb0[ss]);
        row_sum_mfma(1, pb1[ss]);
      }
      // (the address arithmetic of this step's loads does not depend on the barrier: it goes in front of it,
      // where it overlaps with the wait for the slowest wave.  The bookkeeping for the next step's loads issues
      // a scalar load of the next page id; while that is in flight every wait for an LDS read has to be a wait
      // for everything, so it goes at the end of the step, where the next wait is one for everything anyway:
      // measured 1745 cycles per tile there against 1785 behind the barrier and 1800 in front of it.)
      if (m == 0 && ISSUE) issue_begin(st_cur);
      if (m == 14 && ISSUE && kLoadsTile <= 6) issue_end();
      if (m == 1) {
        // this wave's LDS reads of V(j) have returned (so has everything older) before it tells the
        // others that the stage may be overwritten
        // (while tiles are still being issued, STAGES - 3 of them may stay in flight behind tile j+2; the
        // last steps of a chunk simply wait for everything that is left)
        if (ISSUE) wait_vm_lgkm<kLoadsTile * (STAGES - 3)>(); else wait_vm_lgkm<0>();
        __builtin_amdgcn_s_barrier();
      }
      // (a compute unit takes about 64 bytes of vector-memory requests per cycle, and its four waves issue
      // their loads behind the same MFMAs: one 1 KiB load per wave behind every second MFMA stays below
      // that rate, two behind one MFMA wait on each other for four MFMAs' time.  The forms with ten loads
      // per tile have no slots to spare and put one behind every MFMA.)
      // (the loads sit behind the odd MFMAs: the even ones carry the column maxima)
      if (kLoadsTile <= 6) {
        if (ISSUE && m >= 3 && (m & 1) == 1 && (m - 3) / 2 < kLoadsTile) issue_full_part((m - 3) / 2);
      } else {
        if (ISSUE && m >= 2 && m < 2 + kLoadsTile) issue_full_part(m - 2);
        if (ISSUE && m == 2 + kLoadsTile) issue_end();
      }
      // (the last K read is three MFMAs from the end of the step: the first wait of the next step, which
      // covers every LDS read because a scalar load is in flight, then finds them all returned)
      if (GLA && m >= 2 && m <= 5) {
        // partner = the wave with the other channel half and the same token half (the barrier behind MFMA 1
        // made its stores visible); after MFMA 5 every wave has its sums and the buffer may be rewritten
        const f32x4* px = xbuf + ((wave ^ 1) * 8 + 2 * (m - 2)) * 64 + lane;
        f32x4 x0 = px[0], x1 = px[64];
        asm volatile("" : "+v"(x0), "+v"(x1));   // ordinary registers (the additions below cannot read the other file)
        f32x16& dst = (m < 4) ? n0 : n1;
        const int r0 = 8 * ((m - 2) & 1);
#pragma unroll
        for (int e = 0; e < 4; ++e) { dst[r0 + e] += x0[e]; dst[r0 + 4 + e] += x1[e]; }
        if (m == 5) __builtin_amdgcn_s_barrier();
      }
      if (m == 1) hold(ka[10]);
      if (m == 3) hold(ka[11]);
      if (m >= 5 && m <= 11 && (m & 1) == 1) hold(va[0][(m - 5) >> 1]);   // last read by MFMA m - 4
      if (m == 13) hold(va[1][0]);
      if (m == 15) hold(va[1][1]);
      if (m == 10) hold(pb0[0]);
      if (m == 11) hold(pb1[0]);
      if (m >= 2 && m <= 13) load_k_part(st_k2, m - 2, ka);
      // (the score chains ended four MFMAs and a barrier before MFMA 2; in the GLA form the partner's partial
      // scores are added behind MFMAs 2..5 first)
      constexpr int kMaxAt = GLA ? 6 : 2;
      if (m == kMaxAt) mx0 = max8(n0[0], n0, 0);
      if (m == kMaxAt + 2) mx0 = max8(mx0, n0, 8);
      if (m == kMaxAt + 4) mx1 = max8(n1[0], n1, 0);
      if (m == kMaxAt + 6) mx1 = max8(mx1, n1, 8);
      if (m == kMaxAt + 8) {
        cross_max(mx0, mx1);
        // (one comparison on the larger of the two maxima decides the common case, here rather than at the
        // end of the step so that the branch there finds its condition ready)
        float mx_both;
        asm("v_max_f32 %0, %1, %2" : "=v"(mx_both) : "v"(mx0), "v"(mx1));
        need_any = __any(mx_both > kLazy);
      }
      __builtin_amdgcn_sched_barrier(0);
    }
    // the maxima are relative to the reference: it moves only when a head's scores outgrow it by 2^kLazy
    // (an issuing step always has a next tile)
    if (__builtin_expect((ISSUE || has_next) && need_any, 0)) {
      const bool need0 = mx0 > kLazy, need1 = mx1 > kLazy;
      settle_acc();
      rescale(std::integral_constant<int, 0>{}, need0 ? mx0 : 0.f, n0);
      rescale(std::integral_constant<int, 1>{}, need1 ? mx1 : 0.f, n1);
    }
    st_cur = (st_cur + kStageB == STAGES * kStageB) ? 0 : st_cur + kStageB;
  };
  {
    const std::integral_constant<bool, true> issuing;
    const std::integral_constant<bool, false> draining;
    // steps 0 .. ntiles - STAGES - 1 issue a tile each, the last STAGES steps only drain the pipeline
    const int n_issue = ntiles > STAGES ? ntiles - STAGES : 0;
    int j = 0;
    for (; j + 4 <= n_issue; j += 4) {   // (four steps per trip: the taken branch at the end costs a refetch)
      step(issuing, j, sa0, sa1, sb0, sb1);
      step(issuing, j + 1, sb0, sb1, sa0, sa1);
      step(issuing, j + 2, sa0, sa1, sb0, sb1);
      step(issuing, j + 3, sb0, sb1, sa0, sa1);
    }
    for (; j + 2 <= n_issue; j += 2) {
      step(issuing, j, sa0, sa1, sb0, sb1);
      step(issuing, j + 1, sb0, sb1, sa0, sa1);
    }
    if (j < n_issue) {   // an odd number of issuing steps: one more, then the score registers trade places
      step(issuing, j, sa0, sa1, sb0, sb1);
      ++j;
#pragma unroll
      for (int i = 0; i < 16; ++i) { sa0[i] = sb0[i]; sa1[i] = sb1[i]; }
    }
    for (; j < ntiles; j += 2) {
      step(draining, j, sa0, sa1, sb0, sb1);
      if (j + 1 < ntiles) step(draining, j + 1, sb0, sb1, sa0, sa1);
    }
  }

  // ---- merge the two token halves of each head half through LDS, write the chunk's partial ----
  {
  settle_acc();   // the last PV MFMAs have retired before ordinary code reads the accumulators
  // (the lane's indices are derived again from a thread id the compiler cannot connect to the first one:
  // otherwise it keeps a dozen of them alive across the main loop, spilled to scratch memory)
  int tid_again = threadIdx.x;
  asm volatile("" : "+v"(tid_again));
  const int tid = tid_again, wave = tid >> 6, lane = tid & 63, hw = wave & 1, tw = wave >> 1, g = lane >> 5,
            c32 = lane & 31;
  const int blk = (PAIRED && !GLA) ? blk0 + hw : blk0;
  const int wave_head0 = PAIRED ? hgrp * 64 : hgrp * kHeadsWG + hw * 64;
  float l_run[2];
  l_run[0] = acc_read<128>();   // (already summed over both token halves of the wave)
  l_run[1] = acc_read<132>();
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
  float m_out[2], l_out[2], w_mine[2];
#pragma unroll
  for (int nt = 0; nt < 2; ++nt) {
    const float mp = mbuf[(wave ^ 2) * 64 + nt * 32 + c32];
    const float lp = lbuf[(wave ^ 2) * 64 + nt * 32 + c32];
    const float ms = fmaxf(m_run[nt], mp);
    const float w_own = __builtin_amdgcn_exp2f(m_run[nt] - ms);
    const float w_par = __builtin_amdgcn_exp2f(mp - ms);
    m_out[nt] = ms;
    l_out[nt] = l_run[nt] * w_own + lp * w_par;
    w_mine[nt] = w_own;
  }
  // this wave's Z^T, four registers at a time, weighted for the merge of the two token halves
  auto z4 = [&](auto nt_tag, auto mt_tag, auto r4_tag) {
    constexpr int nt = decltype(nt_tag)::value;
    f32x4 v = acc_read4<decltype(mt_tag)::value, nt, decltype(r4_tag)::value>();
    const float w = w_mine[nt];
    return f32x4{v[0] * w, v[1] * w, v[2] * w, v[3] * w};
  };
  // (compile-time loops over head tile, channel tile and register quad: the register names are immediates)
  auto for_each_quad = [&](auto&& fn) {
    auto quads = [&](auto nt_tag, auto mt_tag) {
      fn(nt_tag, mt_tag, std::integral_constant<int, 0>{});
      fn(nt_tag, mt_tag, std::integral_constant<int, 1>{});
      fn(nt_tag, mt_tag, std::integral_constant<int, 2>{});
      fn(nt_tag, mt_tag, std::integral_constant<int, 3>{});
    };
    auto tiles = [&](auto nt_tag) {
      quads(nt_tag, std::integral_constant<int, 0>{});
      quads(nt_tag, std::integral_constant<int, 1>{});
      quads(nt_tag, std::integral_constant<int, 2>{});
      quads(nt_tag, std::integral_constant<int, 3>{});
    };
    tiles(std::integral_constant<int, 0>{});
    tiles(std::integral_constant<int, 1>{});
  };
  auto zrow = [&](int nt, int mt, int r4) {
    return zbuf + (hw * 64 + nt * 32 + c32) * kZPitch + mt * 32 + r4 * 8 + g * 4;
  };
  if (tw == 1) {
    for_each_quad([&](auto nt_tag, auto mt_tag, auto r4_tag) {
      *(f32x4*)zrow(decltype(nt_tag)::value, decltype(mt_tag)::value, decltype(r4_tag)::value) = z4(nt_tag, mt_tag, r4_tag);
    });
  }
  __syncthreads();
  if (tw == 0) {
    for_each_quad([&](auto nt_tag, auto mt_tag, auto r4_tag) {
      f32x4* const row = (f32x4*)zrow(decltype(nt_tag)::value, decltype(mt_tag)::value, decltype(r4_tag)::value);
      const f32x4 own = z4(nt_tag, mt_tag, r4_tag);
      f32x4 v = *row;
      v[0] += own[0];
      v[1] += own[1];
      v[2] += own[2];
      v[3] += own[3];
      *row = v;
    });
    // (bf16 rows: 1 / l of the row's head goes into the padding behind its 128 channels)
    if (p.rows_bf16 && g == 0) {
#pragma unroll
      for (int nt = 0; nt < 2; ++nt)
        zbuf[(hw * 64 + nt * 32 + c32) * kZPitch + kDcb] = l_out[nt] > 0.f ? 1.f / l_out[nt] : 0.f;
    }
  }
  __syncthreads();
  // zbuf row hl = hw * 64 + (head inside the wave's 64): plain form, 128 heads of one block; PAIRED, 64
  // heads of block blk0 then the same 64 heads of block blk0 + 1
  // (GLA: rows 64..127 are channels 128..255 of the same 64 heads of the one block)
  constexpr int kZRow = GLA ? 2 * kDcb : kDcb;   // channels of one partial row in the workspace
  if (p.rows_bf16) {
    // The chunk's partial leaves normalised: z * (1 / l) rounded to bf16, with (m, l) beside it in fp32.  A
    // convex combination of cache rows is no larger than they are, so bf16 holds it as well as it holds
    // the cache; with one chunk per sequence the row is already what the up-projection consumes, with
    // several the merge weighs the rows by 2^(m_k - m*) l_k.  Half the bytes of fp32 partials.
    bf16_t* zn = (bf16_t*)p.part_z;
    for (int idx = tid; idx < kHeadsWG * (kDcb / 8); idx += 256) {
      const int hl = idx / (kDcb / 8), f8 = idx % (kDcb / 8);
      const int row_blk = (PAIRED && !GLA) ? blk0 + (hl >> 6) : blk0;
      const int row_head = PAIRED ? hgrp * 64 + (hl & 63) : hgrp * kHeadsWG + hl;
      const size_t row_unit = ((size_t)seq * p.n_blocks + row_blk) * p.n_splits + split;
      if (row_head < p.h) {
        const float inv = zbuf[hl * kZPitch + kDcb];
        const f32x4 lo = *(const f32x4*)(zbuf + hl * kZPitch + f8 * 8), hi = *(const f32x4*)(zbuf + hl * kZPitch + f8 * 8 + 4);
        bf16x8 packed;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          packed[e] = (__bf16)(inv * lo[e]);
          packed[4 + e] = (__bf16)(inv * hi[e]);
        }
        *(bf16x8*)(zn + (row_unit * p.h + row_head) * kZRow + (GLA ? (hl >> 6) * kDcb : 0) + f8 * 8) = packed;
      }
    }
  } else {
    // (for the generic merge kernel, which takes shapes whose tables do not fit the MFMA epilogue's LDS: fp32, not normalised)
    for (int idx = tid; idx < kHeadsWG * (kDcb / 4); idx += 256) {
      const int hl = idx / (kDcb / 4), f4 = idx % (kDcb / 4);
      const int row_blk = (PAIRED && !GLA) ? blk0 + (hl >> 6) : blk0;
      const int row_head = PAIRED ? hgrp * 64 + (hl & 63) : hgrp * kHeadsWG + hl;
      const size_t row_unit = ((size_t)seq * p.n_blocks + row_blk) * p.n_splits + split;
      if (row_head < p.h)
        *(f32x4*)(p.part_z + (row_unit * p.h + row_head) * kZRow + (GLA ? (hl >> 6) * kDcb : 0) + f4 * 4) =
            *(const f32x4*)(zbuf + hl * kZPitch + f4 * 4);
    }
  }
  const size_t unit = ((size_t)seq * p.n_blocks + blk) * p.n_splits + split;
  if (tw == 0 && g == 0 && !(GLA && hw == 1)) {   // (GLA: both channel halves hold the same m and l)
#pragma unroll
    for (int nt = 0; nt < 2; ++nt) {
      const int head = wave_head0 + nt * 32 + c32;
      if (head < p.h) {
        p.part_ml[(unit * p.h + head) * 2 + 0] = m_out[nt];
        p.part_ml[(unit * p.h + head) * 2 + 1] = l_out[nt];
      }
    }
  }
  }
}

constexpr int kStages = 6;         // plain form: 6 x 24 KiB
constexpr int kStagesPaired = 4;   // PAIRED form: 4 x 40 KiB = all 160 KiB of LDS

}  // namespace

// Fills a.chunk_tab (workspace) with per-sequence chunk lengths, see plan_chunks_kernel.
int launch_plan_chunks(const DecodeArgs& a) {
  if (!a.chunk_tab || !a.unit_tab || a.plan.target_chunks <= 0) return MLRA_ERR_SHAPE;
  if (a.plan.n_splits > 1023 || a.batch > 2048) return MLRA_ERR_SHAPE;
  plan_chunks_kernel<<<1, 256, 3 * a.batch * sizeof(int32_t), a.stream>>>(
      a.seq_lens, a.chunk_tab, a.unit_tab, a.batch, a.plan.target_chunks, a.plan.n_splits, 128,
      a.plan.single_if_uniform ? 1 : 0);
  return check_launch();
}

// Fills a.seq_order (workspace) with the sequence ids in dispatch order (see seq_order_kernel).
// MLRA_ERR_SHAPE (and nothing enqueued) when the batch is outside what the O(batch^2) rank sort is meant for.
int launch_seq_order(const DecodeArgs& a) {
  const int group = a.q_group > 1 ? a.q_group : 1;
  if (!a.seq_order || a.batch <= 1 || a.batch > 8192 || a.batch % group != 0) return MLRA_ERR_SHAPE;
  const int n_seqs = a.batch / group;
  seq_order_kernel<<<(n_seqs + 255) / 256, 256, n_seqs * sizeof(int32_t), a.stream>>>(a.seq_lens, a.seq_order, n_seqs,
                                                                                     group);
  return check_launch();
}

// (several query tokens per sequence: the order is what brings a sequence's queries together, so it is
// wanted even when one round of workgroups covers the launch)
static bool want_seq_order(const DecodeArgs& a, long long n_wg) {
  return !a.balanced && (n_wg > device_cu_count() || a.q_group > 1);
}

// Pages of 16 or 32 tokens (a wave's 16 rows of a tile never straddle a page), or whole tiles.
static bool page_size_ok(int page_size) { return page_size == 16 || page_size == 32 || page_size % kTile == 0; }
// (the kernels form page id x bytes-per-page from 32-bit factors)
static bool page_bytes_ok(const DecodeArgs& a) { return (long long)a.n_blocks * a.page_size * a.d_cb * 2 < (1LL << 32); }

bool decode_mfma_supported(const DecodeArgs& a) {
  // (the query rows are addressed with 32-bit byte offsets from q_abs / q_rope)
  return a.dtype == MLRA_BF16 && a.d_cb == kDcb && a.d_r == kDr && page_size_ok(a.page_size) && page_bytes_ok(a) &&
         a.plan.chunk_tokens % kTile == 0 &&
         (long long)a.batch * a.n_blocks * a.h * (kDcb * 2) < (1LL << 32) &&
         (long long)a.batch * a.h * a.groups * (kDr * 2) < (1LL << 32);
}

// Blocks that serve at most 64 heads in their last 128-head group leave half of the plain form's waves
// idle; with an even number of blocks the PAIRED form runs two blocks per workgroup instead.
bool decode_mfma_paired(int h, int n_blocks) { return n_blocks % 2 == 0 && (h - 1) % kHeadsWG < 64; }

// GLA-2 shape: latent heads of 256 channels (Section 2.3); 64 heads per workgroup.
bool decode_gla_supported(const DecodeArgs& a) {
  return a.dtype == MLRA_BF16 && a.d_cb == 2 * kDcb && a.d_r == kDr && page_size_ok(a.page_size) && page_bytes_ok(a) &&
         a.plan.chunk_tokens % kTile == 0 &&
         (long long)a.batch * a.n_blocks * a.h * (4 * kDcb) < (1LL << 32) &&
         (long long)a.batch * a.h * a.groups * (kDr * 2) < (1LL << 32);
}

int launch_decode_gla(const DecodeArgs& a) {
  static PerDeviceSetup setup;
  int setup_dev = -1;
  constexpr int kStagesGla = 3;
  const int lds = kStagesGla * (2 * kLatBytes + kRopeBytes) + 4 * 8 * 64 * 16;   // stages + score exchange
  if (setup.needed(&setup_dev)) {
    if (hipFuncSetAttribute((const void*)decode_mfma_kernel<kStagesGla, 2>,
                            hipFuncAttributeMaxDynamicSharedMemorySize, lds) != hipSuccess)
      return MLRA_ERR_LAUNCH;
    setup.done(setup_dev);
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
  p.groups = a.groups;
  p.n_splits = a.plan.n_splits;
  p.chunk = a.plan.chunk_tokens;
  p.batch = a.batch;
  p.scale_log2 = softmax_scale_log2(a.softmax_scale);
  p.rows_bf16 = a.rows_bf16 ? 1 : 0;
  p.chunk_tab = a.balanced ? a.chunk_tab : nullptr;
  p.unit_tab = a.balanced ? a.unit_tab : nullptr;
  p.seq_order = nullptr;
  const long long n_wg = (long long)a.plan.n_splits * a.n_blocks * ((a.h + 63) / 64) * a.batch;
  if (n_wg <= 0 || n_wg > 0x7fffffffLL) return MLRA_ERR_SHAPE;
  if (want_seq_order(a, n_wg) && launch_seq_order(a) == MLRA_OK) p.seq_order = a.seq_order;
  MLRA_LAUNCH_TIMED(a.t_main, (decode_mfma_kernel<kStagesGla, 2>), dim3((unsigned)n_wg), dim3(256), lds, a.stream, p);
  return check_launch();
}

int launch_decode_mfma(const DecodeArgs& a) {
  static PerDeviceSetup setup;
  int setup_dev = -1;
  const bool paired = decode_mfma_paired(a.h, a.n_blocks);
  const int lds = paired ? kStagesPaired * (2 * kLatBytes + kRopeBytes) : kStages * kStageBytes;
  if (setup.needed(&setup_dev)) {
    if (hipFuncSetAttribute((const void*)decode_mfma_kernel<kStages, 0>,
                            hipFuncAttributeMaxDynamicSharedMemorySize, kStages * kStageBytes) != hipSuccess ||
        hipFuncSetAttribute((const void*)decode_mfma_kernel<kStagesPaired, 1>,
                            hipFuncAttributeMaxDynamicSharedMemorySize,
                            kStagesPaired * (2 * kLatBytes + kRopeBytes)) != hipSuccess)
      return MLRA_ERR_LAUNCH;
    setup.done(setup_dev);
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
  p.groups = a.groups;
  p.n_splits = a.plan.n_splits;
  p.chunk = a.plan.chunk_tokens;
  p.batch = a.batch;
  p.scale_log2 = softmax_scale_log2(a.softmax_scale);
  p.rows_bf16 = a.rows_bf16 ? 1 : 0;
  const int n_hg = paired ? (a.h + 63) / 64 : (a.h + kHeadsWG - 1) / kHeadsWG;
  const long long n_wg = (long long)a.plan.n_splits * (paired ? a.n_blocks / 2 : a.n_blocks) * n_hg * a.batch;
  if (n_wg <= 0 || n_wg > 0x7fffffffLL) return MLRA_ERR_SHAPE;
  // more than one round of workgroups (one per CU at a time): longest sequences first
  p.seq_order = nullptr;
  p.chunk_tab = a.balanced ? a.chunk_tab : nullptr;
  p.unit_tab = a.balanced ? a.unit_tab : nullptr;
  if (want_seq_order(a, n_wg) && launch_seq_order(a) == MLRA_OK) p.seq_order = a.seq_order;
  if (paired)
    MLRA_LAUNCH_TIMED(a.t_main, (decode_mfma_kernel<kStagesPaired, 1>), dim3((unsigned)n_wg), dim3(256), lds, a.stream, p);
  else
    MLRA_LAUNCH_TIMED(a.t_main, (decode_mfma_kernel<kStages, 0>), dim3((unsigned)n_wg), dim3(256), lds, a.stream, p);
  return check_launch();
}

}  // namespace mlra
