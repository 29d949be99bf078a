/*
 * semipd.h - C ABI of the semi-PD hot path on one MI355X (gfx950).
 *
 * What the library is: the prefill worker's and the decode worker's attention
 * step, running at the same time on disjoint sets of compute units of ONE GPU,
 * over ONE paged KV-cache pool shared by both (paper: System Design, "Overview",
 * "Prefill and Decode Workers", "Computational Resource Controller", "Unified
 * Memory Manager").  The paper partitions SMs between two processes with MPS;
 * here the two phases are two HIP streams created with disjoint CU masks.
 *
 * Conventions
 *  - Every call returns an int status (SPD_OK or a negative SPD_E*), never throws,
 *    and leaves all library state unchanged when it fails: pool, block tables, operation
 *    numbers, and the partition (a step adopts a staged partition only once nothing but a
 *    HIP call can still fail).  SPD_EHIP is the exception: a failing HIP call may leave
 *    work of the step enqueued and its reservations made.
 *  - Every device tensor handed to a step (q, k, v, latent, out, k_new, v_new, the dense side
 *    of spd_kv_write / spd_kv_gather) must start on a 16-byte boundary: the kernels move 16
 *    bytes per lane.  SPD_EINVAL otherwise.
 *  - "device" pointers are HIP device addresses owned by the caller (the library
 *    never frees them); "host" pointers are ordinary host memory read during the
 *    call only.  Tensors are dense row-major bf16 unless stated otherwise.
 *  - Steps are asynchronous: they enqueue work on the calling phase's current
 *    stream and return.  Use spd_phase_sync / spd_phase_query to wait.
 *  - One thread may drive the prefill phase while another drives the decode
 *    phase (the paper's two asynchronous workers).  spd_kv_* may be called from
 *    both at once.  Two threads must not drive the SAME phase concurrently.
 */
#ifndef SEMIPD_H
#define SEMIPD_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct spd_ctx spd_ctx;   /* device, partition state, per-phase streams and staging   */
typedef struct spd_pool spd_pool; /* unified KV pool: pages + allocator + block tables        */

enum {
  SPD_OK = 0,
  SPD_EINVAL = -1, /* bad argument (null pointer, non-positive size, unsupported shape)     */
  SPD_ENOMEM = -2, /* pool exhausted: fewer free blocks than the call needs                 */
  SPD_ENOENT = -3, /* unknown request id                                                    */
  SPD_EHIP = -5,   /* a HIP call failed; spd_last_hip_error() has its code                  */
  SPD_ESTATE = -6, /* call not valid in this state (e.g. a step on a host-only context)     */
  SPD_ETOOBIG = -7 /* spd_decode_step_noalloc: the batch needs more than its fixed scratch   */
};

enum { SPD_PHASE_PREFILL = 0, SPD_PHASE_DECODE = 1 };

typedef enum { SPD_KV_GQA = 0, SPD_KV_MLA_LATENT = 1, SPD_KV_MLA_LATENT_FP8 = 2 } spd_kv_kind;

/* ------------------------------------------------------------------ context */

/* Create a context on HIP device `device` (>= 0).  device == -1 creates a host-only
 * context: allocator, block tables and the partition state machine work, no GPU is
 * touched, and every call that would launch work returns SPD_ESTATE.
 * The initial partition is (all CUs, all CUs): both phases may use the whole chip,
 * the paper's (100, 100) setting ("Computational Resource Controller"). */
int spd_ctx_create(int device, spd_ctx** out);
int spd_ctx_destroy(spd_ctx* ctx);

/* CU count, XCD count and the granularity (in CUs) to which partition sizes are rounded
 * (one CU in each of the four shader arrays of every XCD: an XCD deals its workgroups to its
 * shader arrays in turn, so CUs beyond a whole such row add no throughput).  A host-only
 * context reports MI355X's 256 / 8 / 32. */
int spd_device_info(spd_ctx* ctx, int* total_cus, int* xcds, int* cu_granularity);

/* ------------------------------------------------------------------ unified KV pool
 * Paper: "Unified Memory Manager" - one paged store for the KV cache of both workers,
 * accessed through per-request block tables.  The pool memory belongs to the caller
 * and must outlive the pool object; it survives every spd_set_partition (the paper's
 * resident process that keeps weights and KV cache across worker switches).
 *
 * Page geometry.  GQA: a page holds page_tokens tokens of K [n_kv_heads, dim_k] and
 * V [n_kv_heads, dim_v]; page_tokens must be a multiple of 16; dim_k == dim_v in {64, 128}.
 * MLA latent: a page holds page_tokens rows of dim_k (= 576) values, n_kv_heads = 1,
 * dim_v = 512 is the number of leading dims that act as values; page_tokens % 32 == 0.
 * MLA latent, FP8 (paper, Evaluation "Model": DeepSeek-V3 is served with FP8 precision; the format is
 * this library's reading): the same geometry, but a cached row keeps its 512 leading entries as OCP
 * FP8 E4M3 codes with one fp32 scale per block of 128 entries (scale = largest magnitude of the block
 * / 448, or 1 for an all-zero block; code = E4M3(clamp(x / scale, -448, 448)), nearest even, division
 * and scale in fp32) and its 64 rope entries in bf16: 656 bytes per token instead of 1152.  Every call
 * takes and returns the same bf16 tensors as for a bf16 latent pool: rows are quantised on their way
 * into the pages, spd_kv_gather hands back decode(code) * scale rounded to bf16, and the decode step
 * attends over exactly those dequantised rows.  RoPE inside the decode step is not offered on such a
 * pool (SPD_EINVAL).
 * The byte layout inside a page is private to the library (it is arranged for the
 * decode kernel's matrix-core operand order); read or write pages only through
 * spd_kv_write / spd_kv_gather / the steps. */
typedef struct {
  int32_t kind;        /* spd_kv_kind */
  int32_t page_tokens; /* P */
  int32_t n_kv_heads;
  int32_t dim_k;
  int32_t dim_v;
  int64_t num_pages;
} spd_pool_desc;

/* Bytes a pool of this geometry needs. */
int spd_pool_bytes(const spd_pool_desc* desc, uint64_t* bytes_out);
/* dev_mem: device pointer, 256-byte aligned, `bytes` >= spd_pool_bytes.  With a host-only
 * context dev_mem may be NULL.  The pool starts with every page free. */
int spd_pool_create(spd_ctx* ctx, void* dev_mem, uint64_t bytes, const spd_pool_desc* desc, spd_pool** out);
int spd_pool_destroy(spd_pool* pool);
/* total pages, free pages, live requests, number of successful mutating operations so far. */
int spd_pool_stats(spd_pool* pool, int64_t* total, int64_t* free_pages, int64_t* live_reqs, uint64_t* op_seq);

/* Atomic block allocation (paper: "Unified Memory Manager", the query / get / update of the
 * memory utilisation done under one lock so that the two asynchronous workers cannot
 * interleave).  Thread-safe.  Policy (the paper fixes none; this is the library's contract):
 * the free list is a stack whose first pops are 0, 1, 2, ...; reserve grows request `req_id`'s
 * block table to ceil(n_tokens_total / P) blocks (creating the request if new; never shrinks);
 * all-or-nothing: SPD_ENOMEM and no change if too few blocks are free.  free returns every
 * block of the request, pushed back last-to-first, and forgets the request.
 * Lifetime rule of free: the blocks can be handed out again by the very next reserve, on either
 * worker, so a request may be freed only after every step that was given its id (prefill step,
 * decode step, spd_kv_write, spd_kv_gather; the decode worker's steps too) has finished on the
 * GPU - after spd_phase_sync, or spd_phase_query reporting done, of the phases that used it.
 * The library checks it: while such a step may still be running, free returns SPD_ESTATE and
 * changes nothing (it never waits).  Work the caller enqueues itself on a phase's stream is
 * the caller's to order.
 * op_seq_out (nullable) receives the operation's position (1, 2, ...) in the pool's
 * linearised order of successful mutating calls; failed calls consume no number. */
int spd_kv_reserve(spd_pool* pool, uint64_t req_id, int32_t n_tokens_total, uint64_t* op_seq_out);
int spd_kv_free(spd_pool* pool, uint64_t req_id, uint64_t* op_seq_out);
/* Copy the request's block table (physical page ids, logical order) to host `out[cap]`;
 * *n_out = its length (also when cap is too small, in which case SPD_EINVAL is returned). */
int spd_kv_block_table(spd_pool* pool, uint64_t req_id, int32_t* out, int32_t cap, int32_t* n_out);
/* Copy the free stack, bottom to top (the next reserve pops out[n-1]), to host `out[cap]`. */
int spd_kv_free_list(spd_pool* pool, int32_t* out, int64_t cap, int64_t* n_out);

/* Write n_tokens rows into request `req_id`'s pages at logical positions
 * [start_pos, start_pos + n_tokens); blocks must already be reserved (SPD_EINVAL if not).
 * GQA: k device [n_tokens, n_kv_heads, dim_k], v device [n_tokens, n_kv_heads, dim_v].
 * MLA: k device [n_tokens, dim_k] latent rows, v must be NULL.
 * Enqueued on `phase`'s current stream (paper, "Prefill and Decode Workers": the K, V
 * projections of a request are written into the KV cache). */
int spd_kv_write(spd_ctx* ctx, spd_pool* pool, int phase, uint64_t req_id, int32_t start_pos,
                 int32_t n_tokens, const void* k, const void* v);
/* Inverse of spd_kv_write: logical rows [0, n_tokens) of the request to dense device
 * buffers of the same shapes (v_out NULL for MLA).  For tests and migration. */
int spd_kv_gather(spd_ctx* ctx, spd_pool* pool, int phase, uint64_t req_id, int32_t n_tokens,
                  void* k_out, void* v_out);

/* ------------------------------------------------------------------ the allocator across processes
 * Paper, "Unified Memory Manager" and "Computational Resource Controller": the two workers are two
 * PROCESSES over one KV cache that a resident process keeps; an allocation is atomic across them.  The
 * calls below keep the allocator state itself - free stack, block tables, utilisation, operation
 * numbers - in a POSIX shared-memory segment `name` (must start with '/') under a process-shared
 * mutex inside the segment, so that every worker process that opens the segment allocates from the
 * same pool with the same policy and results as spd_kv_reserve / spd_kv_free above (free list a stack
 * whose first pops are 0, 1, 2, ...; all-or-nothing; blocks returned last to first; one operation
 * number per successful mutating call, in the order the calls took the lock).  Host logic only: no GPU
 * is touched, the pages themselves are not part of the segment.  At most max_requests requests are
 * live at a time (SPD_ENOMEM beyond, nothing changes).  create fails with SPD_ESTATE if the name
 * exists; open with SPD_ENOENT if it does not, SPD_ESTATE if it is not a complete pool segment.
 * close unmaps (the segment lives on); unlink removes the name.  If a process dies inside a call
 * the next caller finds the lock abandoned and every later call returns SPD_ESTATE: the state can no
 * longer be trusted. */
typedef struct spd_shm_pool spd_shm_pool;
int spd_shm_pool_create(const char* name, int64_t num_pages, int32_t page_tokens, int32_t max_requests,
                        spd_shm_pool** out);
int spd_shm_pool_open(const char* name, spd_shm_pool** out);
int spd_shm_pool_close(spd_shm_pool* pool);
int spd_shm_pool_unlink(const char* name);
int spd_shm_pool_stats(spd_shm_pool* pool, int64_t* total, int64_t* free_pages, int64_t* live_reqs, uint64_t* op_seq);
int spd_shm_kv_reserve(spd_shm_pool* pool, uint64_t req_id, int32_t n_tokens_total, uint64_t* op_seq_out);
int spd_shm_kv_free(spd_shm_pool* pool, uint64_t req_id, uint64_t* op_seq_out);
int spd_shm_kv_block_table(spd_shm_pool* pool, uint64_t req_id, int32_t* out, int32_t cap, int32_t* n_out);
int spd_shm_kv_free_list(spd_shm_pool* pool, int32_t* out, int64_t cap, int64_t* n_out);

/* ------------------------------------------------------------------ the two steps */

/* Prefill step (paper, Background "LLM Processing Phases" and "Prefill and Decode
 * Workers": the prefill iteration processes the whole prompt and writes its K, V into the
 * cache).  For each request r (rows cu_seqlens[r] .. cu_seqlens[r+1] of the packed batch) and
 * query head h (KV head h / (n_q_heads / n_kv_heads)):
 *     out[i, h, :] = sum_{j <= i} softmax_j(scale * q[i, h, :] . k[j, g, :]) * v[j, g, :]
 * and the request's rows are written to its pages at positions 0 .. len-1; the step reserves
 * ceil(len / P) blocks per request first (all requests or none: SPD_ENOMEM changes nothing).
 *   q   device [T, n_q_heads, dim_qk]    k device [T, n_kv_heads, dim_qk]
 *   v   device [T, n_kv_heads, dim_v]    out device [T, n_q_heads, dim_v]
 * GQA pool: n_kv_heads / dim_qk / dim_v are the pool's.  MLA pool: k, v are the un-absorbed
 * per-head tensors (n_kv_heads == n_q_heads, dim_qk 192, dim_v 128) and `latent` device
 * [T, 576] is what is written to the pages; latent must be NULL for a GQA pool.
 * Zero-length requests are SPD_EINVAL; scale must be positive and finite (the running maximum
 * of the scores is taken before scaling).
 *
 * Chunked prefill (paper, Evaluation "Baselines": the chunked-prefill variants): with
 * prefix_lens non-NULL (GQA pools only) request r already has prefix_lens[r] >= 0 tokens in its
 * pages and the rows given are the next piece of its prompt, at positions prefix .. prefix+len-1:
 *     out[i, h, :] = sum_{j <= prefix + i} softmax_j(scale * q[i, h, :] . K_r[j, g, :]) * V_r[j, g, :]
 * where K_r, V_r are the cached rows followed by the piece's own.  The step reserves blocks for
 * prefix + len tokens, writes the new rows to the pages, gathers each request's rows
 * 0 .. prefix+len-1 through its block table into a library workspace and attends over that.  A
 * request with prefix > 0 must exist with at least prefix tokens reserved (else SPD_ENOENT /
 * SPD_EINVAL).
 *
 * With `rope` non-NULL (GQA pools only; spd_rope_config is declared further down; paper, Evaluation
 * "Implementation based on DistServe": the RoPE kernel) q and k are the vectors BEFORE the rotary
 * embedding and the step rotates them itself, IN PLACE (q and k hold the rotated vectors afterwards,
 * as after spd_rope_qk), row i of request r by position prefix_lens[r] + i: the keys on their way
 * into the pages, in the launch that writes the pages (so K crosses memory once for rotation and
 * page write together), the queries in a pass of their own before the attention.  The rotating range
 * must fit the head (rotary_offset + rotary_dim <= dim_qk; multiples of 8 and 16), else SPD_EINVAL. */
struct spd_rope_config;
typedef struct {
  int32_t n_req;
  const uint64_t* req_ids;   /* host [n_req] */
  const int32_t* cu_seqlens; /* host [n_req + 1], cu_seqlens[0] == 0 */
  const void* q;
  const void* k;
  const void* v;
  const void* latent;
  void* out;
  int32_t n_q_heads;
  int32_t n_kv_heads;
  int32_t dim_qk;
  int32_t dim_v;
  float scale;
  const int32_t* prefix_lens; /* host [n_req] or NULL (no cached prefix) */
  const struct spd_rope_config* rope; /* NULL, or: q and k are given before RoPE and rotated by the step */
} spd_prefill_batch;
int spd_prefill_step(spd_ctx* ctx, spd_pool* pool, const spd_prefill_batch* batch);

/* Decode step (paper, Background: the decode phase produces the next token from the last
 * token and the KV cache, and appends the new key / value; "Unified Memory Manager": the
 * cache is read through the block table, and the decode worker allocates inside the paged
 * attention computation).  For each request b with context n = ctx_lens[b] >= 1 and head h:
 *     out[b, h, :] = sum_{t < n} softmax_t(scale * q[b, h, :] . K_b[t, g, :]) * V_b[t, g, :]
 * where K_b, V_b are the request's cached rows found through its block table.  If k_new is
 * non-NULL the step first reserves blocks for n tokens and writes k_new[b], v_new[b] at
 * position n - 1 (so n counts the token being decoded); if NULL it attends only.
 *   GQA: q device [B, n_q_heads, dim_k], k_new/v_new device [B, n_kv_heads, dim_k/dim_v],
 *        out device [B, n_q_heads, dim_v].
 *   MLA: q device [B, n_q_heads, 576] (absorbed query), k_new device [B, 576] latent rows,
 *        v_new NULL, out device [B, n_q_heads, 512];
 *        s[h,t] = scale * q[b,h,:] . c_t,  out[b,h,:] = sum_t softmax_t(s[h,:]) * c_t[0:512].
 * n_q_heads must be a multiple of n_kv_heads with at most 16 query heads per KV head; scale
 * must be positive and finite.
 * With `rope` non-NULL (declared further down; paper, Evaluation "Implementation based on
 * DistServe": the RoPE kernel) q and k_new are the vectors BEFORE the rotary embedding: the step
 * rotates request b's query and new key by position ctx_lens[b] - 1, the query into a library
 * workspace (the caller's q, k_new are left as they are), the key straight into the page, in the one
 * launch that appends; the attention then reads the rotated query.  The rotating range must fit the
 * head (rotary_offset + rotary_dim <= dim_k; multiples of 8 and 16) or the call is SPD_EINVAL. */
typedef struct {
  int32_t n_req;
  const uint64_t* req_ids; /* host [n_req] */
  const int32_t* ctx_lens; /* host [n_req] */
  const void* q;
  const void* k_new;
  const void* v_new;
  void* out;
  int32_t n_q_heads;
  float scale;
  const struct spd_rope_config* rope; /* NULL, or: q and k_new are given before RoPE (see below) */
} spd_decode_batch;
int spd_decode_step(spd_ctx* ctx, spd_pool* pool, const spd_decode_batch* batch);

/* The decode step for callers that cannot allocate device memory: code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc.  Same arguments, same kernels and bit-identical
 * results as spd_decode_step, but the call allocates and frees nothing on the device or in pinned
 * memory (no hipMalloc / hipHostMalloc / hipFree, no event or stream creation): the device twin of
 * the step's metadata (context lengths, block tables, work items, append descriptors, RoPE
 * frequencies) and the workspace (split-K partials, rotated queries) lie in a static device array of
 * 33 MiB that every GPU the library runs on holds from the library's load to the end of the process
 * (its address is resolved once per device in spd_ctx_create), and the pinned staging ring is the one
 * spd_ctx_create made.  Limits (spd_noalloc_limits): 256 KiB of metadata per step, i.e.
 * 4 n_req (1 + pages of the longest context) + 8 work items + 32 n_req (append) bytes, and 32 MiB of
 * workspace, i.e. 4 n_req n_q_heads chunks (dim_v + 2) + 2 n_req n_q_heads dim_k (rope) bytes, where
 * chunks is the split-K count the library picks (about 6 workgroups per compute unit of the decode
 * share).  A batch beyond either limit is refused with SPD_ETOOBIG and nothing is enqueued.  Kernel
 * timing (spd_set_kernel_timing) is not recorded for these steps.
 * The array is shared by every context and every call on that GPU and keeps the last call's contents
 * (nothing in it has to start at zero: each step writes every partial it later reads).  Steps of one
 * decode phase run in stream order and may follow one another freely, also mixed with spd_decode_step;
 * calls on the same GPU from two contexts, or from two processes' worth of streams, that overlap in
 * time race on the array and must be serialised by the caller. */
int spd_decode_step_noalloc(spd_ctx* ctx, spd_pool* pool, const spd_decode_batch* batch);
/* The two limits above, in bytes (either pointer may be NULL). */
int spd_noalloc_limits(uint64_t* metadata_bytes, uint64_t* workspace_bytes);

/* ------------------------------------------------------------------ the step before attention */

/* Rotary position embedding (paper, Evaluation, "Implementation based on DistServe": the RoPE
 * kernel, modified for the Llama-3.1 models).  The paper gives no formula; this is the published
 * definition.  Every head vector x of a token at position p is rotated pairwise, pair i
 * (0 <= i < rotary_dim / 2) by the angle p * w_i:
 *     x'_a = x_a cos(p w_i) - x_b sin(p w_i),    x'_b = x_b cos(p w_i) + x_a sin(p w_i)
 * with (a, b) = (off + i, off + i + rotary_dim / 2), or (off + 2i, off + 2i + 1) if `interleaved`,
 * off = rotary_offset; the other entries of the head pass through.  w_i = theta^(-2i / rotary_dim);
 * with factor != 1 the Llama-3.1 scaling is applied to it: with wavelength L = 2 pi / w_i,
 *     L < original_max_pos / high_freq_factor : unchanged
 *     L > original_max_pos / low_freq_factor  : w_i / factor
 *     otherwise: s = (original_max_pos / L - low_freq_factor) / (high_freq_factor - low_freq_factor),
 *                w_i' = (1 - s) w_i / factor + s w_i.
 * Angles are formed in fp64, the rotation in fp32, the result rounded to bf16 (nearest even). */
typedef struct spd_rope_config {
  double theta;             /* > 0, e.g. 500000 (Llama-3) */
  double factor;            /* >= 1; 1 = no frequency scaling (the three fields below are then unused) */
  double low_freq_factor;   /* > 0 */
  double high_freq_factor;  /* > low_freq_factor */
  int32_t original_max_pos; /* > 0 */
  int32_t rotary_dim;       /* rotating entries per head: positive, a multiple of 16 for spd_rope_qk */
  int32_t rotary_offset;    /* first rotating entry of a head: >= 0, a multiple of 8 for spd_rope_qk */
  int32_t interleaved;      /* 0: pairs (i, i + rotary_dim/2); else pairs (2i, 2i + 1) */
} spd_rope_config;
/* Host only: writes the rotary_dim / 2 frequencies w_i (scaled if factor != 1) to out[0 .. cap). */
int spd_rope_inv_freq(const spd_rope_config* cfg, double* out, int32_t cap);
/* Rotates, in place, q device [n_tokens, n_q_heads, dim] and k device [n_tokens, n_kv_heads, dim]
 * (bf16, 16-byte aligned; either may be NULL), token t by positions[t] (host [n_tokens], >= 0).
 * dim must be a multiple of 8 and rotary_offset + rotary_dim <= dim.  Enqueued on `phase`'s current
 * stream, i.e. on that phase's compute units, before the step that consumes q and k (for a decode
 * step the new token's position is ctx_len - 1; k_new goes to the pages rotated).  The positions
 * are copied before the call returns.  SPD_EINVAL on any violated condition, nothing enqueued. */
int spd_rope_qk(spd_ctx* ctx, int phase, const spd_rope_config* cfg, const int32_t* positions, int32_t n_tokens,
                void* q, int32_t n_q_heads, void* k, int32_t n_kv_heads, int32_t dim);

/* ------------------------------------------------------------------ the step after attention */

/* First step of the gated FFN (paper, Evaluation, "Implementation based on DistServe": the first
 * two GEMMs of the gated FFN are fused into one).  The paper gives no formula; this is the
 * published gated (SwiGLU) FFN of the Llama models:
 *     g = x W_gate^T,  u = x W_up^T,  out = silu(g) * u,  silu(z) = z / (1 + exp(-z))
 * computed as ONE product of x with the joint matrix [2 inter, hidden], whose rows
 * 64 b .. 64 b + 31 are rows 32 b .. 32 b + 31 of W_gate and rows 64 b + 32 .. 64 b + 63 the rows
 * with the same numbers of W_up (so that a gate column and its up column meet in one wave), with the
 * activation applied to the fp32 accumulators and one rounding to bf16 (nearest even) at the end.
 * w_gu holds the joint matrix in PACKED form (spd_ffn_pack_gate_up writes it): tiles of 256 joint
 * rows x 32 hidden entries (16 KiB), tile (tn, ks) at byte ((tn * hidden / 32) + ks) * 16384; inside
 * a tile joint row 256 tn + r keeps 64 bytes at r * 64, and its 16-byte piece number s (0..3)
 * holds the hidden entries 32 ks + 8 (s ^ ((r >> 2) & 3)) .. + 7.  (The order of a tile in the
 * kernel's LDS stage: a weight load is 1 KiB of consecutive bytes, and a batch of a few tokens,
 * which is bound by reading the weights once, streams them.)
 * x device [n_tokens, hidden] row-major, w_gu device 2 * inter * hidden elements as above, out device
 * [n_tokens, inter] row-major, bf16; x and w_gu 16-byte aligned; hidden a multiple of 32, inter a
 * multiple of 128; n_tokens >= 0 (0: nothing is enqueued).  Enqueued on `phase`'s current stream,
 * i.e. on that phase's compute units; the buffers belong to the caller and must stay valid until the
 * stream has run the call.  SPD_EINVAL on any violated condition, nothing enqueued. */
int spd_ffn_gate_up(spd_ctx* ctx, int phase, const void* x, const void* w_gu, void* out, int32_t n_tokens,
                    int32_t hidden, int32_t inter);
/* Writes the packed joint matrix w_gu (device, 2 * inter * hidden elements, layout above) from
 * w_gate, w_up device [inter, hidden] row-major (bf16, 16-byte aligned, same conditions on hidden
 * and inter; a permutation of 16-byte pieces, done once per layer at load time).  Enqueued on
 * `phase`'s current stream. */
int spd_ffn_pack_gate_up(spd_ctx* ctx, int phase, const void* w_gate, const void* w_up, void* w_gu, int32_t hidden,
                         int32_t inter);

/* A decode worker inside the library (paper, System Design, "Prefill and Decode Workers": the
 * decode worker runs its iterations asynchronously beside the prefill worker).  Starts a host
 * thread that calls spd_decode_step on batches[0], batches[1], ... batches[n_batches-1],
 * batches[0], ... back to back (each call blocks only when four of its steps are already in
 * flight) until it is stopped, at least once.  The batch descriptors, the arrays they point to and the pool
 * must stay valid and unchanged until spd_decode_worker_stop returns; no other thread may drive
 * the decode phase meanwhile.  Stop joins the thread and reports the number of steps it issued
 * and the first failing status (SPD_OK if none; the worker ends at the first failure).  The
 * issued steps may still be running on the GPU: use spd_phase_sync to wait for them. */
typedef struct spd_worker spd_worker;
int spd_decode_worker_start(spd_ctx* ctx, spd_pool* pool, const spd_decode_batch* const* batches, int32_t n_batches,
                            spd_worker** out);
int spd_decode_worker_stop(spd_worker* w, int64_t* steps_issued, int* status);
/* Decode steps the running worker has issued so far (a counter read, no synchronisation). */
int spd_decode_worker_steps(spd_worker* w, int64_t* steps_issued);

/* Block the calling thread until everything enqueued so far by `phase` has finished. */
int spd_phase_sync(spd_ctx* ctx, int phase);
/* *done = 1 if everything enqueued so far by `phase` has finished, else 0.  Never blocks. */
int spd_phase_query(spd_ctx* ctx, int phase, int* done);
/* Make `phase`'s future work wait (on the GPU, not the host) for everything `other` has
 * enqueued so far - e.g. a decode step that reads pages a prefill step has just written. */
int spd_phase_wait_for(spd_ctx* ctx, int phase, int other);
/* The phase's current hipStream_t, for callers that enqueue their own work or events. */
int spd_phase_stream(spd_ctx* ctx, int phase, void** hip_stream_out);

/* ------------------------------------------------------------------ partition
 * Paper, "Computational Resource Controller": a configuration (x, y) gives x % of the
 * compute units to prefill and y % to decode; x + y may exceed 100 (the two then compete);
 * a new (x, y) is prepared first and adopted late (delayed switching), and each worker
 * adopts it at its own iteration boundary without waiting for the other (asynchronous
 * switching).  Here (x, y) are CU counts.  Each is rounded to the nearest multiple of the
 * granularity, at least one granule, at most all CUs; if the two requested counts sum to no more
 * than the total (disjoint shares) and the rounded ones would overlap, decode gets what prefill
 * leaves.  Prefill takes CUs from the low end of
 * the mask, decode from the high end; they overlap only when the counts sum above the total.
 * The call prepares (creates or re-uses) the two CU-masked streams and stages them as
 * pending; it never blocks on GPU work and never touches the pool.  Each phase switches to
 * its pending stream at the start of its next step; the new stream waits on the GPU for the
 * old stream's last work of that phase, so steps of one phase stay ordered. */
int spd_set_partition(spd_ctx* ctx, int prefill_cus, int decode_cus);
/* Active and pending CU counts per phase (pending == active when nothing is staged). */
int spd_get_partition(spd_ctx* ctx, int* prefill_active, int* decode_active, int* prefill_pending,
                      int* decode_pending);
/* The CU mask (one bit per CU, 32 per word) of the phase's ACTIVE stream to host words[cap]. */
int spd_phase_cu_mask(spd_ctx* ctx, int phase, uint32_t* words, int32_t cap, int32_t* n_words);
/* Pure function: masks for a (prefill_cus, decode_cus) request on a device with total_cus CUs
 * and the given granularity; writes ceil(total_cus / 32) words to each of host
 * prefill_words / decode_words and the rounded counts to *p_out / *d_out. */
int spd_partition_masks(int total_cus, int granularity, int prefill_cus, int decode_cus,
                        uint32_t* prefill_words, uint32_t* decode_words, int* p_out, int* d_out);

/* ------------------------------------------------------------- SLO-aware partition adjuster
 * Paper, "Dynamic Adjusting Method": Algorithm 1 (SLO-aware adjusting algorithm) with the
 * latency models of Eq. 4, TTFT_x = a1 / (x - lambda) + b1 and TPOT_y = a2 / y + b2, learned
 * online from observed latencies (Eq. 1-3 give their shape).  Host logic only: the caller feeds
 * latencies, asks once per iteration for the partition to use, and passes a changed answer to
 * spd_set_partition (shares are percentages of the GPU's CUs).
 *
 * Where the printed algorithm is broken or silent this library: increments the step counter once
 * per loop pass; starts x', y' as the normalised current shares 100 x / (x + y), 100 y / (x + y);
 * tests "both SLOs fail: keep the partition" first; lowers the other share instead when a share
 * would pass 100, never below one step; takes the nearest-rank percentile of the window's
 * samples; fits by ordinary least squares over the latest `history` (share, latency) points, one
 * per window, with lambda from the integer grid 0 .. min(x) - 1 (smallest squared error; a larger
 * lambda must win by more than 1e-12 (1 + error)); and uses Eq. 1 alone (b = 0, lambda = 0,
 * a = latency * share of the latest point) while all points of a phase sit at one share.
 * Points are kept at the raw share (x0, y0) and the models are evaluated at the normalised share, as the
 * printed algorithm does.  Where the shares overlap (x + y > 100, e.g. the initial (100, 100)) a model
 * fitted at share 100 is therefore asked about share 50 and predicts about twice the observed latency:
 * the phase that fails its objective then takes all max_step steps of its first adjustment, and since a
 * share cannot pass 100 the other phase's share is lowered instead ((100, 100) -> (100, 60) with the
 * defaults).  From the second window on the fit has two shares and follows the data.
 */
typedef struct spd_ctrl spd_ctrl;
typedef struct spd_ctrl_config {
  double slo_ttft;      /* S^p: TTFT objective, any time unit (the unit of the observations)     */
  double slo_tpot;      /* S^d: TPOT objective                                                   */
  double p_slo;         /* percentile of the objectives, 0 < p <= 100 (the paper uses 90)        */
  int32_t window_size;  /* adjust every window_size iterations (> 0)                             */
  int32_t max_step;     /* at most this many steps per adjustment (> 0)                          */
  int32_t step_size;    /* percentage points per step, 1 .. 50                                   */
  int32_t history;      /* (share, latency) points kept per phase for the fit (>= 1)             */
} spd_ctrl_config;
/* SPD_EINVAL on a null pointer or a field outside the ranges above. */
int spd_ctrl_create(const spd_ctrl_config* cfg, spd_ctrl** out);
int spd_ctrl_destroy(spd_ctrl* c);
/* One observed latency (finite, >= 0) into the current window.  Callable from the prefill and
 * the decode thread at once. */
int spd_ctrl_observe_ttft(spd_ctrl* c, double latency);
int spd_ctrl_observe_tpot(spd_ctrl* c, double latency);
/* Algorithm 1 for iteration `iter` (>= 0) under the current partition (x0, y0), each within
 * step_size .. 100: writes the partition to use from now on to *x, *y (equal to x0, y0 when
 * iter is not a multiple of window_size, when a window is empty, or when nothing has to move).
 * Closing a window clears its samples. */
int spd_ctrl_step(spd_ctrl* c, int64_t iter, int32_t x0, int32_t y0, int32_t* x, int32_t* y);
/* The current model to host out[5] = {a1, lambda, b1, a2, b2} (zeros before the first window). */
int spd_ctrl_model(spd_ctrl* c, double* out);

/* ===================================================================================
 * MEASUREMENT AND DEBUG AIDS.  Nothing below is part of the hot path's interface: no step
 * needs these calls, they change no result, and a serving loop never makes them.  They are
 * exported for the benchmark, the profiles and the tests of the partition.
 * =================================================================================== */

/* Two environment variables, read once by spd_ctx_create (never by a step), override choices
 * the library otherwise makes itself:
 *   SPD_PREFILL_PERSISTENT=0|1  launch the prefill kernel with one workgroup per work item (0) or
 *                               with one persistent workgroup per compute unit (1) regardless of
 *                               the partition;
 *   SPD_DECODE_CHUNK_TILES=n    fix the split-K chunk of the decode kernels to n 16-token tiles. */

/* With timing on, each step is bracketed by HIP events (spd_phase_last_ms)
 * and, separately, so are its attention kernel(s) (not the
 * block-table upload or the page write) with HIP events on the phase's stream; the last
 * 256 steps are kept.  spd_phase_kernel_ms waits for the phase, writes the durations
 * (milliseconds, oldest first) of the steps recorded since the last call to host out[cap]
 * and their number to *n_out.  Off by default (each record costs a few microseconds). */
int spd_set_kernel_timing(spd_ctx* ctx, int on);
int spd_phase_kernel_ms(spd_ctx* ctx, int phase, float* out, int32_t cap, int32_t* n_out);
/* GPU time of the phase's most recent step in milliseconds (waits for that step).  Steps are
 * timed only while timing is on (spd_set_kernel_timing); otherwise SPD_ESTATE. */
int spd_phase_last_ms(spd_ctx* ctx, int phase, float* ms);

/* A plain device-to-device copy kernel (16 bytes per lane, grid-stride) of `bytes` (a
 * multiple of 16; src, dst 16-byte aligned) from src to dst on the phase's current stream.
 * Its known traffic calibrates hardware byte counters. */
int spd_phase_copy(spd_ctx* ctx, int phase, void* dst, const void* src, uint64_t bytes);

/* A read-only streaming kernel over `bytes` (a multiple of 16) of device memory at src
 * (16-byte aligned) on the phase's current stream: eight independent 16-byte loads in flight
 * per lane, nothing written.  Its speed on a masked stream is the read ceiling of that CU
 * share, the yardstick for the decode kernels (which read every cached byte once and write
 * almost nothing). */
int spd_phase_read(spd_ctx* ctx, int phase, const void* src, uint64_t bytes);

/* The same, read the way the attention kernels fetch their tiles: two workgroups per compute
 * unit, every wave streaming a contiguous part of the buffer with load instructions that write
 * straight into LDS, 16 KiB in flight per wave.  On a share of the chip this reads faster than
 * the register loads above; the yardstick is the faster of the two. */
int spd_phase_read_lds(spd_ctx* ctx, int phase, const void* src, uint64_t bytes);

/* One wave, on the caller's stream `hip_stream` (a hipStream_t; null: the default stream), runs
 * 64 * iters dependent integer adds and writes to device dev_out[3] (8-byte aligned): the time
 * that took in ticks of the constant 100 MHz counter, in ticks of the shader cycle counter,
 * and the chain's result.  Run beside the two phases it shows the clock the chip holds under
 * that load (cycle ticks / constant ticks x 100 MHz).  1 <= iters <= 2^32. */
int spd_clock_probe(spd_ctx* ctx, void* hip_stream, uint64_t iters, uint64_t* dev_out);

/* Does matrix work overlap vector work inside one wave, or only between the waves of a SIMD?  One workgroup
 * on `hip_stream` (null: the default stream) writes to device dev_out[8] (8-byte aligned), in hundredths of
 * a shader cycle per loop iteration: [0] one 32x32x16 bf16 MFMA per iteration, [1] eight independent vector
 * instructions (four v_exp_f32, four v_fma_f32), [2] the MFMA followed by those eight, all three from one
 * wave alone; [3] the MFMA loop again while another wave of the same SIMD runs the vector loop beside it,
 * [4] that other wave's vector loop.  If [2] is about [0] + [1] while [3] and [4] stay about [0] and [1], an
 * MFMA holds the wave that issued it and the two kinds of work overlap only between waves. */
int spd_issue_probe(spd_ctx* ctx, void* hip_stream, uint64_t* dev_out);

/* Run a tiny kernel of `n_blocks` workgroups on the phase's current stream and
 * report, to host ids[cap], the distinct hardware (XCD << 16 | SE << 8 | CU) ids that ran
 * them; used to check that a masked stream stays on its CUs. */
int spd_phase_probe_cus(spd_ctx* ctx, int phase, int32_t n_blocks, int32_t* ids, int32_t cap, int32_t* n_ids);


/* ------------------------------------------------------------------ errors */
const char* spd_strerror(int status);
/* The hipError_t of the most recent SPD_EHIP on this thread (0 if none). */
int spd_last_hip_error(void);

#ifdef __cplusplus
}
#endif
#endif /* SEMIPD_H */
