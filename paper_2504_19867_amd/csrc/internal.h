// Internal declarations shared by the host side and the kernels of libsemipd.
// Not part of the public ABI (see include/semipd.h).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <map>
#include <atomic>
#include <mutex>
#include <unordered_map>
#include <vector>

#include "semipd.h"

namespace spd {

// ---------------------------------------------------------------------------------------------
// Page layout in HBM.
//
// Tokens are grouped in tiles of 16 (TILE_T).  A GQA page holds, for every KV head g, a
// contiguous "head region" of P/16 tiles; each tile is a K part followed by a V part:
//
//   K part (16 tokens x dk):  [chunk c = d/8][token t][8 dims]
//       A wave that loads "chunk 4s + lane/16, token lane%16" with one 16-byte load per lane
//       reads 1 KiB contiguous and gets exactly the A operand of v_mfma_f32_16x16x32_bf16
//       (row = token, 8 consecutive contraction elements per lane) for k-step s.
//   V part (16 tokens x dv):  [d/32][token quad t/4][d%16][(d/16)%2][t%4]
//       One 16-byte load per lane at "(blk2*4 + lane/16)*16 + lane%16" is again 1 KiB
//       contiguous and holds the A operands (row = d, 4 consecutive tokens per lane) of two
//       v_mfma_f32_16x16x16_bf16 for the value blocks 2*blk2 and 2*blk2 + 1.
//
// An MLA latent page keeps the natural order: P rows of 576 dims.  Its decode kernel stages rows
// through LDS and reads them back in both operand orders (kernels_decode_mla.hip).
// ---------------------------------------------------------------------------------------------
constexpr int TILE_T = 16;
// FP8 latent pages: a cached row is 512 E4M3 codes, 4 fp32 scales (one per 128 entries) and 64 bf16 rope entries
constexpr int FP8_ROW_BYTES = 512 + 16 + 128;

struct PoolGeom {
  int kind, P, Hkv, dk, dv;
  int tiles_per_page;
  uint32_t tile_k_bytes, tile_v_bytes, tile_bytes, head_bytes;
  uint64_t page_bytes;
};

__host__ __device__ inline uint32_t k_elem_offset(int t16, int d) { return ((d >> 3) * 16 + t16) * 8 + (d & 7); }
__host__ __device__ inline uint32_t v_elem_offset(int t16, int d) {
  return (((((d >> 5) * 4 + (t16 >> 2)) * 16 + (d & 15)) * 2 + ((d >> 4) & 1)) * 4) + (t16 & 3);
}

inline PoolGeom make_geom(const spd_pool_desc& d) {
  PoolGeom g{};
  g.kind = d.kind; g.P = d.page_tokens; g.Hkv = d.n_kv_heads; g.dk = d.dim_k; g.dv = d.dim_v;
  g.tiles_per_page = d.page_tokens / TILE_T;
  g.tile_k_bytes = d.kind == SPD_KV_MLA_LATENT_FP8 ? TILE_T * FP8_ROW_BYTES : TILE_T * d.dim_k * 2;
  g.tile_v_bytes = d.kind == SPD_KV_GQA ? TILE_T * d.dim_v * 2 : 0;
  g.tile_bytes = g.tile_k_bytes + g.tile_v_bytes;
  g.head_bytes = g.tiles_per_page * g.tile_bytes;
  g.page_bytes = (uint64_t)g.head_bytes * d.n_kv_heads;
  return g;
}

// One 16-token tile's worth of rows to copy between a dense [rows, heads, dim] tensor and a page.
struct TileDesc {
  int32_t src_row;   // row of the dense tensor that maps to token t_begin of the tile
  int32_t page;      // physical page id
  int32_t sub;       // tile index inside the page
  int32_t t_begin;   // first token slot (0..15) touched
  int32_t t_end;     // one past the last token slot touched
  int32_t pad[3];    // pad[0]: logical position of the tile's token slot 0 in its request
};

// Prefill work item = one workgroup: one tile of query rows of one request, for a group of query
// heads that share a KV head.  len == 0 marks a padding item (the workgroup exits at once).
struct PrefillWork {
  int32_t row0;      // first packed row of the request's queries (and outputs)
  int32_t len;       // number of query rows of the request in this step
  int32_t q_tile;    // tile index inside those rows (tile height depends on the head grouping)
  int32_t head0;     // first query head of the workgroup's head group
  int32_t kv_row0;   // first row of the request's keys / values in the K, V tensors the kernel reads
  int32_t q_off;     // position of query row 0 in the request = number of cached tokens before it
};

// The entry point that allocates nothing keeps its device-side working memory in one static device
// array (noalloc.hip): four metadata twins (one per slot of the decode phase's staging ring), then the
// split-K partials and the rotated queries.
constexpr size_t NOALLOC_STAGE_BYTES = 256u << 10;
constexpr size_t NOALLOC_WS_BYTES = 32u << 20;
constexpr size_t SCRATCH_BYTES = 4 * NOALLOC_STAGE_BYTES + NOALLOC_WS_BYTES;

extern thread_local int g_last_hip_error;
inline int hip_fail(hipError_t e) { g_last_hip_error = (int)e; return SPD_EHIP; }
#define SPD_HIP(expr) do { hipError_t _e = (expr); if (_e != hipSuccess) return ::spd::hip_fail(_e); } while (0)

}  // namespace spd

// ------------------------------------------------------------------------------------------ objects
// A request's block table, and for each phase the number of the last step of that phase that took the table
// (0: none): spd_kv_free refuses while such a step may still be running on the GPU.
struct spd_req_table : std::vector<int32_t> {
  uint64_t last_use[2] = {0, 0};
};

struct spd_pool {
  spd_ctx* ctx;
  spd_pool_desc desc;
  spd::PoolGeom geom;
  char* base;
  uint64_t bytes;
  std::mutex mu;                                  // the "lock on memory utilisation"
  std::vector<int32_t> free_stack;                // top = back()
  int64_t used = 0;
  uint64_t op_seq = 0;
  std::unordered_map<uint64_t, spd_req_table> tables;
};

struct spd_stage {          // pinned host buffer + device twin, reused round-robin per phase
  char* host = nullptr;
  char* dev = nullptr;
  size_t cap = 0;
  char* dev_static = nullptr;   // this slot's metadata twin inside the static scratch array (decode phase)
  hipEvent_t done = nullptr;          // recorded behind the last kernel of the step that used the slot
  bool in_flight = false;
  std::atomic<uint64_t> seq{0};       // number of that step (stored after the event has been recorded)
};

struct spd_phase_state {
  hipStream_t stream = nullptr;        // active
  int active_cus = 0;
  hipStream_t pending_stream = nullptr;
  int pending_cus = 0;
  bool has_pending = false;
  std::vector<uint32_t> active_mask, pending_mask;
  spd_stage ring[4];
  int ring_pos = 0;
  std::atomic<uint64_t> issue_seq{0};  // steps (ring commits) of this phase so far; the next step's number is this + 1
  std::atomic<uint64_t> done_seq{0};   // a step number known to have finished on the GPU (steps of a phase finish in order)
  hipEvent_t ev_start = nullptr, ev_end = nullptr, ev_switch = nullptr, ev_cross = nullptr;
  bool timed = false;
  char* workspace = nullptr;           // split-K partials (decode)
  size_t ws_cap = 0;
  // workspaces outgrown, with the number of the last step that may still read them: freed once that step has
  // finished (looked at when the workspace grows again, in spd_phase_sync and when the context goes)
  std::vector<std::pair<char*, uint64_t>> ws_retired;
  std::mutex ws_mu;                    // the list above (a step's thread against another thread's spd_phase_sync)
  // last split-K chunk choice of the MLA decode (re-derived when the batch has changed by more than a little)
  int ck_B = 0, ck_cus = 0, ck_chunk = 0;
  int64_t ck_sum = 0;
  hipEvent_t kev[256][2] = {};         // kernel timing ring (measurement aid)
  uint64_t kev_count = 0, kev_read = 0;
};

struct spd_ctx {
  int device = -1;                     // -1: host only
  int total_cus = 256, xcds = 8, granularity = 32;
  std::mutex part_mu;                  // partition state (set_partition vs step entry)
  std::map<std::vector<uint32_t>, hipStream_t> stream_cache;
  spd_phase_state phase[2];
  bool kernel_timing = false;
  int env_prefill_persistent = -1;     // SPD_PREFILL_PERSISTENT as read by spd_ctx_create (-1: not set)
  int env_decode_chunk_tiles = 0;      // SPD_DECODE_CHUNK_TILES as read by spd_ctx_create (0: not set)
  char* scratch = nullptr;             // this device's copy of the static scratch array (noalloc.hip)
};

namespace spd {
// host helpers (ctx.cpp)
int phase_enter(spd_ctx* ctx, int phase, hipStream_t* stream_out);   // adopt pending stream
// may_alloc = false: SPD_ETOOBIG instead of growing the slot's buffers
int stage_acquire(spd_ctx* ctx, int phase, size_t bytes, spd_stage** out, bool may_alloc = true);
int scratch_resolve(int device, char** out);   // noalloc.hip: address of `device`'s copy of the scratch array
// copy = false: the caller has already launched a kernel that copies host -> dev (see launch_kv_write)
// dev: the device twin to copy to (null: the slot's own st->dev)
int stage_commit(spd_ctx* ctx, int phase, spd_stage* st, size_t bytes, hipStream_t stream, bool copy = true,
                 char* dev = nullptr);
int stage_host_as_device(spd_stage* st, void** out);   // device-readable address of the pinned host buffer
int stage_copy(spd_stage* st, size_t bytes, hipStream_t stream, char* dev = nullptr);   // host buffer -> device twin
// true if step number `seq` of `phase` has finished on the GPU (any thread may ask)
bool phase_step_done(spd_ctx* ctx, int phase, uint64_t seq);
int workspace_reserve(spd_ctx* ctx, int phase, size_t bytes, char** out);
int kernel_timing_mark(spd_ctx* ctx, int phase, int which, hipStream_t stream);   // which: 0 begin, 1 end
// rope.cpp: SPD_OK if the configuration is well-formed; the frequency table (rotary_dim / 2 doubles)
int rope_config_check(const spd_rope_config* c);
void rope_frequencies(const spd_rope_config* c, double* out);

// kernel launchers (kernels_*.hip); all enqueue on `stream` and return the launch status
// d_tiles may be device-readable pinned host memory.  With copy_dst non-null the same launch also
// copies copy_bytes (rounded up to 16) from copy_src to copy_dst.
// With rope_w non-null (device or device-readable pinned: rot / 2 frequencies) the key rows are rotated on the way
// (position = TileDesc.pad[0] + token slot), into the pages and in place in k; only where kv_write_can_rotate.
hipError_t launch_kv_write(const PoolGeom& g, char* pool_base, const TileDesc* d_tiles, int n_tiles,
                           const void* k, const void* v, hipStream_t stream, void* copy_dst = nullptr,
                           const void* copy_src = nullptr, uint64_t copy_bytes = 0, const double* rope_w = nullptr,
                           int rot = 0, int rot_off = 0, bool interleaved = false);
bool kv_write_can_rotate(const PoolGeom& g);
hipError_t launch_kv_gather(const PoolGeom& g, const char* pool_base, const TileDesc* d_tiles, int n_tiles,
                            void* k_out, void* v_out, hipStream_t stream);
// FP8 latent pools (kernels_kv_fp8.hip): quantising page write of dense [rows, 576] bf16 latent rows (with the same
// optional metadata copy as launch_kv_write), and the gather that hands back the dequantised rows
hipError_t launch_kv_write_fp8(const PoolGeom& g, char* pool_base, const TileDesc* d_tiles, int n_tiles, const void* latent,
                               hipStream_t stream, void* copy_dst = nullptr, const void* copy_src = nullptr,
                               uint64_t copy_bytes = 0);
hipError_t launch_kv_gather_fp8(const PoolGeom& g, const char* pool_base, const TileDesc* d_tiles, int n_tiles, void* out,
                                hipStream_t stream);
hipError_t launch_decode_gqa(const PoolGeom& g, const char* pool_base, const void* q, void* out,
                             const int32_t* d_ctx_lens, const int32_t* d_block_tables, int bt_stride,
                             const void* d_items, int n_items, int B, int H, float scale, int chunk_tiles,
                             int max_chunks, float* ws_o, float* ws_ml, hipStream_t stream);
hipError_t launch_decode_mla(const PoolGeom& g, const char* pool_base, const void* q, void* out,
                             const int32_t* d_ctx_lens, const int32_t* d_block_tables, int bt_stride,
                             const void* d_items, int n_items, int B, int H, float scale, int chunk_steps,
                             int max_chunks, float* ws_o, float* ws_ml, hipStream_t stream, bool fp8 = false);
int decode_mla_step_tokens();
// one workgroup per chain: workgroup b computes the items d_work[d_chain[b]] .. d_work[d_chain[b + 1] - 1]
hipError_t launch_prefill(const void* q, const void* k, const void* v, void* out, const PrefillWork* d_work,
                          const int32_t* d_chain, int n_blocks, int H, int Hkv, int dqk, int dv, float scale,
                          hipStream_t stream);
// x [T, K], w_gu [2 I, K] (joint gate/up rows in blocks of 32 + 32), out [T, I], all bf16 in device memory;
// K a multiple of 32, I a multiple of 128
hipError_t launch_ffn_gate_up(const void* x, const void* w_gu, void* out, int T, int K, int I, int xcds, int cus,
                              hipStream_t stream);
hipError_t launch_ffn_pack(const void* w_gate, const void* w_up, void* w_gu, int K, int I, hipStream_t stream);
// d_pos, d_w may be device-readable pinned host memory
hipError_t launch_rope(void* q, int n_q_heads, void* k, int n_kv_heads, int dim, int rot, int off, bool interleaved,
                       int n_tokens, const int32_t* d_pos, const double* d_w, hipStream_t stream);
// decode step with RoPE: rotated query copy + rotated key (and value) appended to the page, one launch
hipError_t launch_rope_append(const PoolGeom& g, char* pool_base, const TileDesc* d_descs, const int32_t* d_ctx_lens, int B,
                              const void* q, void* q_out, int Hq, int dq, const void* k_new, const void* v_new, int rot,
                              int off, bool interleaved, const double* d_w, hipStream_t stream);
hipError_t launch_probe(int32_t* d_ids, int n_blocks, hipStream_t stream);
hipError_t launch_copy(void* dst, const void* src, uint64_t bytes, int cus, hipStream_t stream);
hipError_t launch_read(const void* src, uint64_t bytes, int cus, uint32_t* sink, hipStream_t stream);
hipError_t launch_read_lds(const void* src, uint64_t bytes, int cus, uint32_t* sink, hipStream_t stream);
hipError_t launch_clock_probe(uint64_t iters, uint64_t* d_out, hipStream_t stream);
hipError_t launch_issue_probe(uint64_t* d_out, hipStream_t stream);
bool prefill_shape_supported(int dqk, int dv);
int prefill_heads_per_block(int group);   // query heads of one KV head that share a workgroup
int prefill_block_m(int group);           // query rows per workgroup
}  // namespace spd
