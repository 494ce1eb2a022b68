/*
 * libmlra -- decode-step attention of Multi-Head Low-Rank Attention (MLRA) for AMD MI355X (gfx950).
 *
 * C ABI.  Every buffer is a DEVICE pointer owned by the caller unless a comment says "host".
 * The library enqueues kernels on the given HIP stream (hipStream_t passed as void*, NULL = the
 * default stream) and returns without synchronising.  It allocates nothing; scratch memory is a
 * caller-provided workspace.  No call throws; each returns
 * an mlra_status.  Errors that the host can see (null pointer, unsupported shape or dtype, a
 * workspace that is too small, a failed launch) return a negative status and enqueue nothing.
 * Device-side preconditions are the caller's: page ids in [0, num_pages), seq_lens[b] <=
 * max_pages_per_seq * page_size, positions[b] inside the pages mapped for sequence b.
 *
 * Notation follows the paper: n context length, h query heads, d_h head dim, d_r = d_h^R the
 * partial-RoPE dim, d_c the KV latent dim cut into n_blocks channel blocks of d_cb = d_c/n_blocks
 * (Section 2.1 "Block Multiplications"), tau = 1/sqrt(d_h + d_r) the softmax scale.
 * MLRA-4 is n_blocks = 4; one device's share of 4-way tensor parallelism is n_blocks = 1 with that
 * block's pool and weights (closing paragraph of Section 3.2: the branches are independent up to a final sum).
 *
 * Layouts (row-major, last index fastest):
 *   latent pool  [num_pages][n_blocks][page_size][d_cb]   C^KV, channel block b of a token in plane b
 *   rope pool    [num_pages][page_size][d_r]              K^RoPE, already rotated, shared by all heads
 *   page_table   [batch][max_pages_per_seq] int32         logical page -> physical page
 *   seq_lens     [batch] int32                            valid tokens, including the newest one
 *   w_uk, w_uv   [n_blocks][d_cb][h*d_h]                  the paper's W^UK, W^UV in R^{d_c x (h d_h)},
 *                                                         i.e. row block b, head i in columns [i d_h,(i+1) d_h)
 */
#ifndef MLRA_H_
#define MLRA_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#if defined(__GNUC__)
#define MLRA_API __attribute__((visibility("default")))
#else
#define MLRA_API
#endif

typedef enum {
  MLRA_OK = 0,
  MLRA_ERR_NULL = -1,      /* a required pointer is NULL                         */
  MLRA_ERR_SHAPE = -2,     /* a dimension is non-positive or not supported        */
  MLRA_ERR_DTYPE = -3,     /* unknown or unsupported element type                 */
  MLRA_ERR_WORKSPACE = -4, /* workspace missing or smaller than required          */
  MLRA_ERR_LAUNCH = -5     /* the HIP runtime refused a launch or a query         */
} mlra_status;

typedef enum { MLRA_BF16 = 0, MLRA_F32 = 1 } mlra_dtype;

/* Paged latent KV cache (Section 2.1: both C^KV and K^RoPE are cached; per token d_c + d_r
 * elements, Table 1 column "KV Cache").  A contiguous cache is the identity page table. */
typedef struct mlra_cache {
  void* latent;              /* device [num_pages][n_blocks][page_size][d_cb] */
  void* rope;                /* device [num_pages][page_size][d_r]            */
  const int32_t* page_table; /* device [batch][max_pages_per_seq]             */
  const int32_t* seq_lens;   /* device [batch]                                */
  int32_t num_pages;
  int32_t page_size;
  int32_t max_pages_per_seq;
  int32_t n_blocks;
  int32_t d_cb;
  int32_t d_r;
  int32_t dtype;             /* mlra_dtype of both pools                      */
} mlra_cache;

/* Human-readable text for a status (host pointer to a static string). */
MLRA_API const char* mlra_strerror(int status);

/* Stores the newest token's cache row of every sequence (Section 2.1: C^KV and K^RoPE of each token
 * are cached).  Row b goes to logical slot positions[b] of sequence b; positions[b] < 0 skips the
 * sequence.  Values are converted from src_dtype to the cache dtype with round-to-nearest-even.
 * RMSNorm, the alpha_kv scaling of Eq. (9) and RoPE happen upstream and are not applied here.
 *   c_kv_new   [batch][n_blocks*d_cb]  blocks side by side, block b in columns [b d_cb,(b+1) d_cb)
 *   k_rope_new [batch][d_r]
 *   positions  [batch] int32 (device) */
MLRA_API int mlra_append_kv(const mlra_cache* cache, int32_t batch, const void* c_kv_new, const void* k_rope_new,
                   int32_t src_dtype, const int32_t* positions, void* stream);

/* Step 1 of the absorbed decode (Section 2.1 "Query-Side Weight Absorption"), per block:
 *   q_abs[s][b][i][:] = W^UK_(b),(i) q_nope[s][i][:]      (einsum "hp,hpc->hc", c = d_cb)
 *   q_nope [batch][h][d_h], w_uk [n_blocks][d_cb][h*d_h], q_abs [batch][n_blocks][h][d_cb];
 * all three have element type dtype.  Accumulation is fp32. */
MLRA_API int mlra_absorb_q(int32_t batch, int32_t h, int32_t d_h, int32_t n_blocks, int32_t d_cb,
                  const void* q_nope, const void* w_uk, void* q_abs, int32_t dtype, void* stream);

/* The same with the softmax scale folded into the queries (Eq. (5): both score terms carry the factor tau,
 * so it may be applied to the queries once instead of to every score):
 *   q_abs[s][b][i][:]   = tau log2(e) * W^UK_(b),(i) q_nope[s][i][:]   (multiplied in fp32, rounded once)
 *   q_rope_out[s][i][:] = tau log2(e) * q_rope[s][i][:]                [batch][h][d_r], may alias q_rope
 * with tau = softmax_scale > 0.  The decode entry points take such queries with
 * softmax_scale = MLRA_SCALE_FOLDED: the scores then leave the matrix pipe in the log2 domain and the decode
 * kernel skips its own multiplication of the queries.  Outputs and lse are those of the unfolded calls up
 * to the rounding of the queries.  One launch on `stream`; errors as mlra_absorb_q (+ MLRA_ERR_SHAPE for
 * softmax_scale <= 0 or d_r <= 0). */
#define MLRA_SCALE_FOLDED 0.0f
MLRA_API int mlra_absorb_q_folded(int32_t batch, int32_t h, int32_t d_h, int32_t n_blocks, int32_t d_cb, int32_t d_r,
                         const void* q_nope, const void* w_uk, const void* q_rope, float softmax_scale,
                         void* q_abs, void* q_rope_out, int32_t dtype, void* stream);

/* Bytes of workspace mlra_decode_attn / mla_decode_attn need for these sizes on the current device
 * (0 on invalid sizes).  max_seq_len is max_pages_per_seq * page_size of the cache passed later. */
MLRA_API size_t mlra_decode_workspace_bytes(int32_t batch, int32_t h, int32_t n_blocks, int32_t d_cb,
                                   int32_t max_seq_len);

/* Steps 2 and 3 of the absorbed decode, per block, and the block sum (Eq. (1) applied to each block;
 * Eq. (5); output rescale of Eq. (10)).  For sequence s, head i:
 *   score_b[t] = softmax_scale * ( q_abs[s][b][i] . C_(b)[t] + q_rope[s][i] . K^RoPE[t] ),  t < seq_lens[s]
 *   z_b        = sum_t Softmax(score_b)[t] C_(b)[t]
 *   out[s][i]  = out_scale * sum_b z_b W^UV_(b),(i)
 * The single decode query attends to all seq_lens[s] cached rows (its own row included; append first).
 * seq_lens[s] == 0 gives a zero output row and lse = -inf.
 *   q_abs  [batch][n_blocks][h][d_cb], q_rope [batch][h][d_r], w_uv [n_blocks][d_cb][h*d_h]: cache dtype
 *   out    [batch][h][d_h] of out_dtype
 *   lse    optional [batch][n_blocks][h] fp32: natural-log sum of exp(score_b); may be NULL
 *   workspace: at least mlra_decode_workspace_bytes(batch, h, n_blocks, d_cb,
 *              max_pages_per_seq*page_size) bytes, 256-byte aligned; contents are overwritten.
 *   softmax_scale: tau > 0, or MLRA_SCALE_FOLDED when q_abs and q_rope come from mlra_absorb_q_folded
 *              (they then carry tau log2(e) and the scores are not scaled again).
 * Context is split into chunks processed by independent workgroups whose partial (max, sum, z) are
 * merged with a log-sum-exp merge; results are deterministic (no atomics). */
MLRA_API int mlra_decode_attn(const mlra_cache* cache, int32_t batch, int32_t h, int32_t d_h, const void* q_abs,
                     const void* q_rope, const void* w_uv, float softmax_scale, float out_scale, void* out,
                     int32_t out_dtype, float* lse, void* workspace, size_t workspace_bytes, void* stream);

/* mlra_decode_attn for callers that cannot allocate device memory or pass a workspace (code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc): same arguments without the
 * workspace, same kernels, same results.  The scratch memory is a fixed array of
 * MLRA_STATIC_SCRATCH_BYTES inside the library's device image (each GPU the library runs on holds its
 * own copy until the process ends); the call allocates and frees nothing.  Shapes whose
 * mlra_decode_workspace_bytes exceeds MLRA_STATIC_SCRATCH_BYTES return MLRA_ERR_WORKSPACE and enqueue
 * nothing (the five benchmark configurations need at most 32.6 MiB).  All calls on one GPU share that
 * GPU's array: calls that may overlap on one GPU (different streams, different threads) race on it and
 * must be serialised by the caller; calls on one stream are ordered and safe.  The first call on a
 * device looks up the array's address (hipGetSymbolAddress), later calls reuse it. */
#define MLRA_STATIC_SCRATCH_BYTES (40u << 20)
MLRA_API int mlra_decode_attn_static(const mlra_cache* cache, int32_t batch, int32_t h, int32_t d_h, const void* q_abs,
                            const void* q_rope, const void* w_uv, float softmax_scale, float out_scale, void* out,
                            int32_t out_dtype, float* lse, void* stream);

/* Gated attention output (Appendix E, "Gated Attention": O^attn = Attention(H') . G with
 * G = sigma(H W^G) in R^{h d_h}): mlra_decode_attn with its output multiplied elementwise by
 *   gate [batch][h][d_h] of the cache dtype, the values of G (the nonlinearity is applied upstream).
 * The product is taken in fp32 before the output is rounded. */
MLRA_API int mlra_decode_attn_gated(const mlra_cache* cache, int32_t batch, int32_t h, int32_t d_h, const void* q_abs,
                           const void* q_rope, const void* w_uv, const void* gate, float softmax_scale,
                           float out_scale, void* out, int32_t out_dtype, float* lse, void* workspace,
                           size_t workspace_bytes, void* stream);

/* Several query tokens per sequence (multi-token prediction / speculative decoding): the causal tail of
 * Eq. (5).  The q_len newest rows of every sequence are already cached (seq_lens counts them); query j
 * of sequence s sits at row seq_lens[s] - q_len + j and attends to rows 0 .. seq_lens[s] - q_len + j
 * (Section 2.1: a position attends to its prefix).  A query whose prefix is empty gives a zero row.
 *   q_abs [batch][q_len][n_blocks][h][d_cb]   (mlra_absorb_q with batch*q_len rows produces this)
 *   q_rope [batch][q_len][h][d_r], out [batch][q_len][h][d_h], lse optional [batch][q_len][n_blocks][h]
 * Everything else as mlra_decode_attn.  The q_len queries of a sequence run as q_len decode units over the
 * same pages, dispatched so that they share one XCD's L2 (the sequence's rows leave HBM once); workspace from
 * mlra_decode_multi_workspace_bytes (max_pages_per_seq as in the cache passed later). */
MLRA_API size_t mlra_decode_multi_workspace_bytes(int32_t batch, int32_t q_len, int32_t h, int32_t n_blocks,
                                         int32_t d_cb, int32_t page_size, int32_t max_pages_per_seq);
MLRA_API int mlra_decode_attn_multi(const mlra_cache* cache, int32_t batch, int32_t q_len, int32_t h, int32_t d_h,
                           const void* q_abs, const void* q_rope, const void* w_uv, float softmax_scale,
                           float out_scale, void* out, int32_t out_dtype, float* lse, void* workspace,
                           size_t workspace_bytes, void* stream);

/* MLA decode (Section 2.1, three-step algorithm): the same computation with one latent block of
 * d_c channels.  Requires cache->n_blocks == 1; out_scale is 1. */
MLRA_API int mla_decode_attn(const mlra_cache* cache, int32_t batch, int32_t h, int32_t d_h, const void* q_abs,
                    const void* q_rope, const void* w_uv, float softmax_scale, void* out, int32_t out_dtype,
                    float* lse, void* workspace, size_t workspace_bytes, void* stream);

/* MLRA-2 (Eq. (6)) on the same cache.  Heads are cut into two groups by the map gamma of Section 2.3
 * (gamma(i) = 0 for i < h/2, else 1; i_bar = i - gamma(i) h/2) and the latent blocks likewise: group g
 * owns blocks [g n_blocks/2, (g+1) n_blocks/2), i.e. blocks 2g and 2g+1 of the paper's four.  A block
 * serves only the h/2 heads of its group and a head's output is the sum over its group's blocks:
 *   out[s][i] = out_scale * sum_{b in group gamma(i)} Softmax(score_b) C_(b) W^UV_b,(i_bar)
 * with score_b as in mlra_decode_attn.  Everything indexed by (block, head) therefore holds h/2 heads
 * per block:
 *   w_uk, w_uv [n_blocks][d_cb][(h/2)*d_h]   blocks 2g, 2g+1 stacked = the group matrix W^(g),UK / W^(g),UV
 *                                            in R^{2 d_cb x (h/2) d_h}; head i in columns [i_bar d_h, +d_h)
 *   q_abs      [batch][n_blocks][h/2][d_cb]  row i_bar of block b belongs to head i_bar + gamma h/2
 *   lse        [batch][n_blocks][h/2]
 *   q_nope [batch][h][d_h], q_rope [batch][h][d_r], out [batch][h][d_h] keep all h heads in order.
 * n_blocks and h must be even.  With n_blocks = 2 (one block of 2 d_h channels per group) the same call
 * computes GLA-2 (Eq. (3)).  mlra_append_kv is shared.  Argument conventions, workspace rules and error
 * behaviour are those of mlra_absorb_q / mlra_decode_workspace_bytes / mlra_decode_attn. */
MLRA_API int mlra2_absorb_q(int32_t batch, int32_t h, int32_t d_h, int32_t n_blocks, int32_t d_cb,
                   const void* q_nope, const void* w_uk, void* q_abs, int32_t dtype, void* stream);
/* (as mlra_absorb_q_folded, for the two head groups of Eq. (6); pass softmax_scale = MLRA_SCALE_FOLDED to
 * mlra2_decode_attn) */
MLRA_API int mlra2_absorb_q_folded(int32_t batch, int32_t h, int32_t d_h, int32_t n_blocks, int32_t d_cb, int32_t d_r,
                          const void* q_nope, const void* w_uk, const void* q_rope, float softmax_scale,
                          void* q_abs, void* q_rope_out, int32_t dtype, void* stream);
MLRA_API size_t mlra2_decode_workspace_bytes(int32_t batch, int32_t h, int32_t n_blocks, int32_t d_cb,
                                    int32_t max_seq_len);
MLRA_API int mlra2_decode_attn(const mlra_cache* cache, int32_t batch, int32_t h, int32_t d_h, const void* q_abs,
                      const void* q_rope, const void* w_uv, float softmax_scale, float out_scale, void* out,
                      int32_t out_dtype, float* lse, void* workspace, size_t workspace_bytes, void* stream);

/* Pre-attention of the newest token of every sequence (Section 2.1 and Appendix C, subsection "Multi-Head Latent Attention (MLA)", which MLRA keeps from
 * MLA; scaling factors of Eq. (9)).  With x = hidden[s] and t = positions[s]:
 *   C^Q  = alpha_q  RMSNorm(x W^DQ)      q_nope[s][i] = (C^Q W^UQ)[i d_h : (i+1) d_h]
 *   C^KV = alpha_kv RMSNorm(x W^DKV)     q_rope[s][i] = RoPE((C^Q W^QR)[i d_r : (i+1) d_r], t)
 *   K^RoPE = RoPE(x W^KR, t)
 * and C^KV (cut into the cache's n_blocks channel blocks) and K^RoPE are stored at logical slot t of
 * sequence s, exactly where mlra_append_kv would put them (t < 0: queries only, nothing is cached).
 * RMSNorm(v) = gain * v / sqrt(mean(v^2) + eps) over the whole latent; gain pointers may be NULL (= 1).
 * RoPE rotates the 2-D blocks [2l, 2l+1] by t * rope_base^(-2l/d_r) (Appendix B, proof of the RoPE
 * theorem; the frequencies are the usual ones, the paper leaves them open).  C^Q is rounded to dtype
 * before the up-projections; accumulation is fp32.  All matrices are row-major with the paper's shapes:
 *   w_dq [d][d_cq], w_dkv [d][n_blocks*d_cb], w_kr [d][d_r], w_uq [d_cq][h*d_h], w_qr [d_cq][h*d_r],
 *   gain_q [d_cq], gain_kv [n_blocks*d_cb]: device, element type dtype (as hidden, q_nope, q_rope).
 * Follow with mlra_absorb_q (or mlra2_absorb_q) on q_nope and the decode entry point. */
typedef struct mlra_pre_weights {
  const void* w_dq;
  const void* w_dkv;
  const void* w_kr;
  const void* w_uq;
  const void* w_qr;
  const void* gain_q;   /* may be NULL */
  const void* gain_kv;  /* may be NULL */
  int32_t d;            /* hidden size */
  int32_t d_cq;         /* query latent dim d_c' */
  int32_t h;
  int32_t d_h;
  int32_t dtype;        /* mlra_dtype of hidden, weights, gains, q_nope, q_rope */
  float alpha_q;        /* Eq. (9): sqrt(d / d_c') */
  float alpha_kv;       /* Eq. (9): sqrt(4 d / d_c) for MLRA */
  float eps;
  float rope_base;
} mlra_pre_weights;

/* Workspace bytes for mlra_pre_attention on the current device (0 on invalid sizes). */
MLRA_API size_t mlra_pre_attention_workspace_bytes(int32_t batch, int32_t d, int32_t d_cq, int32_t n_blocks,
                                          int32_t d_cb, int32_t d_r, int32_t h, int32_t d_h, int32_t dtype);
/*   hidden [batch][d], positions [batch] int32 (device), q_nope [batch][h][d_h], q_rope [batch][h][d_r];
 *   workspace: 256-byte aligned, contents overwritten.  Errors as for the other entry points; d_h and
 *   d_r must be even and d_r <= 256. */
MLRA_API int mlra_pre_attention(const mlra_cache* cache, const mlra_pre_weights* weights, int32_t batch,
                       const void* hidden, const int32_t* positions, void* q_nope, void* q_rope,
                       void* workspace, size_t workspace_bytes, void* stream);

/* Workspace bytes for gqa_decode_attn (0 on invalid sizes). */
MLRA_API size_t gqa_decode_workspace_bytes(int32_t batch, int32_t h, int32_t d_h, int32_t max_seq_len);

/* GQA decode (Appendix C, "MQA and GQA"): query head i reads KV head floor(i / (h/g)).
 *   out[s][i] = Softmax(softmax_scale * q[s][i] . K[t][j])_t V[t][j],  j = floor(i*g/h), t < seq_lens[s]
 *   k_pool, v_pool [num_pages][g][page_size][d_h] of dtype; q [batch][h][d_h] of dtype
 *   page_table [batch][max_pages_per_seq], seq_lens [batch]; out [batch][h][d_h] of out_dtype. */
MLRA_API int gqa_decode_attn(const void* k_pool, const void* v_pool, const int32_t* page_table, const int32_t* seq_lens,
                    int32_t num_pages, int32_t page_size, int32_t max_pages_per_seq, int32_t batch, int32_t h,
                    int32_t g, int32_t d_h, int32_t dtype, const void* q, float softmax_scale, void* out,
                    int32_t out_dtype, void* workspace, size_t workspace_bytes, void* stream);

/* Measurement aid (host-side state, not thread-safe).  Between begin and end, every mlra_decode_attn /
 * mla_decode_attn call records, for at most max_calls calls, the start and the end of its main decode
 * kernel and of its merge + up-projection epilogue kernel into HIP events: the kernel's own execution
 * interval on the bf16 fast paths (what a kernel trace reports as its duration; planning kernels that
 * precede the decode kernel are not part of it), stream markers around the kernel on the generic paths.
 * mlra_kernel_timing_end waits for those events, stores the average duration in milliseconds of the two
 * kernels and the number of calls measured into the given HOST pointers, and releases the events.
 * begin allocates host event objects; neither call belongs in a latency-critical loop. */
MLRA_API int mlra_kernel_timing_begin(int32_t max_calls);
MLRA_API int mlra_kernel_timing_end(double* main_kernel_ms, double* epilogue_kernel_ms, int32_t* calls);

/* Measurement probes (not part of the decode path).
 * mlra_probe_stream_read: a plain streaming read of `bytes` bytes (device pointer, 16-byte aligned) by
 *   `workgroups` workgroups of 256 threads; the XOR of the data is folded into sink[workgroup] (device,
 *   `workgroups` dwords, owned by the caller) so that the reads are real.  Timed by the caller, it gives the
 *   streaming-read ceiling of the machine the benchmark runs on, to set beside the 8 TB/s nameplate.
 * mlra_probe_shader_clock: one wavefront counts shader cycles against the 100 MHz constant counter for about
 *   spin_us microseconds and stores {cycles, 10 ns ticks} into out[0..1] (device, two int64): launched on a
 *   second stream while other kernels run, it reads the shader clock the chip sustains under that load. */
MLRA_API int mlra_probe_stream_read(const void* src, size_t bytes, uint32_t* sink, int32_t workgroups, void* stream);
MLRA_API int mlra_probe_shader_clock(long long* out, int32_t spin_us, void* stream);

/* Introspection aid (host logic only, touches no device memory and enqueues nothing): which kernels and
 * which context split a decode call of this shape takes.  Arguments as for the decode entry points: h is
 * the total number of query heads, groups is 1 for mlra_decode_attn / mla_decode_attn and 2 for
 * mlra2_decode_attn, dtype the cache dtype, max_seq_len = max_pages_per_seq * page_size.  info is a HOST
 * array of 6 values:
 *   [0] decode kernel: 0 generic, 1 MFMA plain form, 2 MFMA PAIRED form (two blocks per workgroup),
 *       3 MFMA GLA form (256-channel latent heads), 4 MFMA MLA kernel (one 512-channel latent)
 *   [1] chunk slots per (sequence, block)     [2] uniform chunk length in tokens
 *   [3] > 0: chunk lengths may follow the sequence lengths (planning kernel), with this many chunks per block
 *       as the target                          [4] 1: a batch of nearly equal lengths is then left uncut
 *   [5] 1: the merge + up-projection epilogue runs on MFMA, 0: generic
 * Returns MLRA_OK, or MLRA_ERR_NULL / MLRA_ERR_SHAPE / MLRA_ERR_DTYPE as the decode entry points would. */
MLRA_API int mlra_decode_plan_info(int32_t batch, int32_t h, int32_t d_h, int32_t groups, int32_t n_blocks, int32_t d_cb,
                                   int32_t d_r, int32_t page_size, int32_t max_seq_len, int32_t dtype, int32_t* info);

#ifdef __cplusplus
}
#endif
#endif /* MLRA_H_ */
