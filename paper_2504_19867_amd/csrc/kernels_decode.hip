// Decode step, GQA: paged attention of one query row per request over the unified pool.
//
// Paper, Background "LLM Processing Phases" (decode produces the next token from the last
// token and the KV cache) and "Unified Memory Manager" (the cache is read through the block
// table).  For request b, query head h (KV head g = h / G):
//     out[b,h,:] = sum_{t<n} softmax_t(scale * q[b,h,:] . K[t,g,:]) * V[t,g,:]
//
// The step is bandwidth-bound: every K, V byte of the batch is read exactly once.  One
// workgroup (4 waves) owns one (request, KV head, chunk of the context) and serves all G
// query heads of the group from the same bytes.  Each wave streams whole 16-token tiles from
// HBM straight into matrix-core operand registers (the page layout is arranged so that every
// 16-byte-per-lane load of a wave is 1 KiB contiguous, see internal.h), keeps an online
// softmax per query in registers, and double-buffers the next two tiles while it works.
// The matrix cores are used because G query rows share each key (G*2*d flops per 2*d bytes):
// for G = 8 the fp32 vector units of a partial CU share cannot keep up with HBM.
//   S^T[key, query] = K_tile[16 x d] . Q^T[d x 16]       v_mfma_f32_16x16x32_bf16, d/32 steps
//   O^T[dim, query] += V_tile^T[16 x 16] . P^T[16 x 16]  v_mfma_f32_16x16x16_bf16, d/16 blocks
// Long contexts are split into chunks (split-K); partial (max, sum, O) triples go to a
// workspace and a small second kernel merges them.
#include "internal.h"

namespace spd {

typedef unsigned short bf16_t;
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef short s16x4 __attribute__((ext_vector_type(4)));

typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));

// two floats -> two bf16 (round to nearest even), packed low / high
__device__ inline uint32_t pack_bf16_rne(float a, float b) {
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(f32x2{a, b}, bf16x2));
}
__device__ inline bf16_t to_bf16_rne(float a) { return (bf16_t)(pack_bf16_rne(a, 0.f) & 0xffffu); }

template <int D>
struct TileFrag {          // two 16-token tiles, K and V parts, in operand order
  uint4 k[2][D / 32];
  uint4 v[2][D / 32];
};

// A 16-byte load of data that is read exactly once (KV pages in a decode step): marked non-temporal,
// so that the stream does not push the prefill partition's K/V tiles, which ARE re-read, out of the L2
// the two partitions share.
__device__ inline uint4 load_once(const uint4* p) {
  typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
  const u32x4 r = __builtin_nontemporal_load((const u32x4*)p);
  return uint4{r.x, r.y, r.z, r.w};
}

template <int D>
__device__ inline void load_step(TileFrag<D>& f, const char* __restrict__ pool, uint64_t page_bytes,
                                 uint32_t tile_bytes, int tiles_per_page, const int32_t* __restrict__ bt_row,
                                 uint64_t head_off, int tile, int n_tiles, int lane) {
#pragma unroll
  for (int u = 0; u < 2; ++u) {
    int t = tile + u;
    t = t < n_tiles ? t : n_tiles - 1;            // an out-of-range tile re-reads the last one; it is masked later
    const int page = bt_row[t / tiles_per_page];
    const char* p = pool + (uint64_t)page * page_bytes + head_off + (uint64_t)(t % tiles_per_page) * tile_bytes;
    const uint4* kp = (const uint4*)p + lane;
    const uint4* vp = (const uint4*)(p + TILE_T * D * 2) + lane;
#pragma unroll
    for (int s = 0; s < D / 32; ++s) f.k[u][s] = load_once(kp + s * 64);
#pragma unroll
    for (int s = 0; s < D / 32; ++s) f.v[u][s] = load_once(vp + s * 64);
  }
}

template <int D>
__device__ inline void compute_step(const TileFrag<D>& f, const bf16x8 (&qf)[D / 32], f32x4 (&O)[D / 16], float& m,
                                    float& l, int tile, int n_tiles, int n, float c, int c4) {
  f32x4 S[2];
#pragma unroll
  for (int u = 0; u < 2; ++u) {
    S[u] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int s = 0; s < D / 32; ++s)
      S[u] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, f.k[u][s]), qf[s], S[u], 0, 0, 0);
  }
  // lane holds, for query (lane % 16), the keys tile*16 + 4*c4 + i of each tile
  const bool tail = (tile + 2) * TILE_T > n;
  if (tail) {
#pragma unroll
    for (int u = 0; u < 2; ++u)
#pragma unroll
      for (int i = 0; i < 4; ++i)
        if ((tile + u) * TILE_T + 4 * c4 + i >= n) S[u][i] = -INFINITY;
  }
  float mx = fmaxf(fmaxf(fmaxf(S[0][0], S[0][1]), fmaxf(S[0][2], S[0][3])),
                   fmaxf(fmaxf(S[1][0], S[1][1]), fmaxf(S[1][2], S[1][3])));
  mx = fmaxf(mx, __shfl_xor(mx, 16));
  mx = fmaxf(mx, __shfl_xor(mx, 32));
  const float m_new = fmaxf(m, mx);
  const float alpha = __builtin_amdgcn_exp2f((m - m_new) * c);
  const float mc = m_new * c;
  float psum = 0.f;
  uint2 pb[2];
#pragma unroll
  for (int u = 0; u < 2; ++u) {
    float p[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      p[i] = __builtin_amdgcn_exp2f(S[u][i] * c - mc);
      psum += p[i];
    }
    pb[u].x = pack_bf16_rne(p[0], p[1]);
    pb[u].y = pack_bf16_rne(p[2], p[3]);
  }
  l = l * alpha + psum;
  m = m_new;
#pragma unroll
  for (int blk = 0; blk < D / 16; ++blk) O[blk] *= alpha;
#pragma unroll
  for (int u = 0; u < 2; ++u) {
    int t = tile + u;
    t = t < n_tiles ? t : n_tiles - 1;
    const bool vtail = (t + 1) * TILE_T > n;      // tile holds slots past the context: their bytes are arbitrary
#pragma unroll
    for (int b2 = 0; b2 < D / 32; ++b2) {
      uint4 v = f.v[u][b2];
      if (vtail) {
        const int t0 = t * TILE_T + 4 * c4;
        const uint32_t m01 = (t0 + 0 < n ? 0x0000ffffu : 0u) | (t0 + 1 < n ? 0xffff0000u : 0u);
        const uint32_t m23 = (t0 + 2 < n ? 0x0000ffffu : 0u) | (t0 + 3 < n ? 0xffff0000u : 0u);
        v.x &= m01; v.y &= m23; v.z &= m01; v.w &= m23;
      }
      const s16x4 a0 = __builtin_bit_cast(s16x4, uint2{v.x, v.y});
      const s16x4 a1 = __builtin_bit_cast(s16x4, uint2{v.z, v.w});
      const s16x4 pv = __builtin_bit_cast(s16x4, pb[u]);
      O[2 * b2] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(a0, pv, O[2 * b2], 0, 0, 0);
      O[2 * b2 + 1] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(a1, pv, O[2 * b2 + 1], 0, 0, 0);
    }
  }
}

// grid (n_items * n_kv_heads), block 256; workgroup i serves KV head i % n_kv_heads of work item
// i / n_kv_heads = (request, chunk).  Heads vary fastest so that the round-robin placement of
// workgroups on the 8 XCDs gives every XCD the same mix of long and short chunks.
template <int D>
__global__ __launch_bounds__(256, 2) void decode_gqa_kernel(
    const char* __restrict__ pool, uint64_t page_bytes, uint32_t head_bytes, uint32_t tile_bytes, int tiles_per_page,
    const bf16_t* __restrict__ q, bf16_t* __restrict__ out, const int32_t* __restrict__ ctx_lens,
    const int32_t* __restrict__ bt, int bt_stride, const int2* __restrict__ items, int Hkv, int H, int G,
    float c /* scale * log2(e) */, int chunk_tiles, int max_chunks, float* __restrict__ ws_o,
    float* __restrict__ ws_ml) {
  const int2 item = items[blockIdx.x / Hkv];
  const int b = item.x, chunk = item.y, g = blockIdx.x % Hkv;
  const int n = ctx_lens[b];
  const int n_tiles = (n + TILE_T - 1) / TILE_T;
  const int tile0 = chunk * chunk_tiles;
  if (tile0 >= n_tiles) return;
  const int tile1 = min(n_tiles, tile0 + chunk_tiles);
  const int n_steps = (tile1 - tile0 + 1) >> 1;
  const int n_chunks = (n_tiles + chunk_tiles - 1) / chunk_tiles;
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // wave-uniform: page ids become scalar loads
  const int col = lane & 15, c4 = lane >> 4;

  bf16x8 qf[D / 32];
#pragma unroll
  for (int s = 0; s < D / 32; ++s) {
    uint4 raw = uint4{0, 0, 0, 0};
    if (col < G) raw = *(const uint4*)(q + ((size_t)b * H + g * G + col) * D + 8 * (4 * s + c4));
    qf[s] = __builtin_bit_cast(bf16x8, raw);
  }

  f32x4 O[D / 16];
#pragma unroll
  for (int i = 0; i < D / 16; ++i) O[i] = f32x4{0.f, 0.f, 0.f, 0.f};
  float m = -INFINITY, l = 0.f;

  const int32_t* bt_row = bt + (size_t)b * bt_stride;
  const uint64_t head_off = (uint64_t)g * head_bytes;
  // Software pipeline over this wave's steps j = wave, wave + 4, ...: the loads of the next step
  // are in flight while the current one is consumed.  The steady-state loop body has no branch,
  // so the compiler can wait for exactly the older buffer (vmcnt = loads of the newer one).
#define SPD_LOAD(F, J) load_step<D>(F, pool, page_bytes, tile_bytes, tiles_per_page, bt_row, head_off, tile0 + 2 * (J), n_tiles, lane)
#define SPD_COMP(F, J) compute_step<D>(F, qf, O, m, l, tile0 + 2 * (J), n_tiles, n, c, c4)
  TileFrag<D> fa, fb;
  int j = wave;
  if (j < n_steps) {
    SPD_LOAD(fa, j);
    while (j + 8 < n_steps) {
      SPD_LOAD(fb, j + 4);
      SPD_COMP(fa, j);
      SPD_LOAD(fa, j + 8);
      SPD_COMP(fb, j + 4);
      j += 8;
    }
    if (j + 4 < n_steps) {
      SPD_LOAD(fb, j + 4);
      SPD_COMP(fa, j);
      SPD_COMP(fb, j + 4);
    } else {
      SPD_COMP(fa, j);
    }
  }
#undef SPD_LOAD
#undef SPD_COMP
  l += __shfl_xor(l, 16);
  l += __shfl_xor(l, 32);

  // merge the four waves' (m, l, O) through LDS
  __shared__ float sm_o[4][16][D + 4];
  __shared__ float sm_m[4][16], sm_l[4][16];
#pragma unroll
  for (int blk = 0; blk < D / 16; ++blk)
    *(f32x4*)&sm_o[wave][col][16 * blk + 4 * c4] = O[blk];
  if (c4 == 0) { sm_m[wave][col] = m; sm_l[wave][col] = l; }
  __syncthreads();
  for (int idx = threadIdx.x; idx < G * D; idx += 256) {
    const int qh = idx / D, d = idx % D;
    const float m_tot = fmaxf(fmaxf(sm_m[0][qh], sm_m[1][qh]), fmaxf(sm_m[2][qh], sm_m[3][qh]));
    float l_tot = 0.f, o = 0.f;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
      const float wgt = __builtin_amdgcn_exp2f((sm_m[w][qh] - m_tot) * c);
      l_tot += sm_l[w][qh] * wgt;
      o += sm_o[w][qh][d] * wgt;
    }
    const size_t head = (size_t)b * H + g * G + qh;
    if (n_chunks == 1) {
      out[head * D + d] = to_bf16_rne(o / l_tot);
    } else {
      const size_t slot = head * max_chunks + chunk;
      ws_o[slot * D + d] = o;
      if (d == 0) { ws_ml[slot * 2] = m_tot * c; ws_ml[slot * 2 + 1] = l_tot; }
    }
  }
}

// grid (ceil(H / (512 / D)), B), block 128: merge the chunks of (request, head) pairs; D / 4 threads per head, four
// output dims each.
template <int D>
__global__ __launch_bounds__(128) void decode_combine_kernel(bf16_t* __restrict__ out, const int32_t* __restrict__ ctx_lens,
                                                            int H, int chunk_tiles, int max_chunks,
                                                            const float* __restrict__ ws_o,
                                                            const float* __restrict__ ws_ml) {
  constexpr int TPH = D / 4;                       // threads per head
  const int h = blockIdx.x * (128 / TPH) + threadIdx.x / TPH, b = blockIdx.y, d = 4 * (threadIdx.x % TPH);
  const int n_tiles = (ctx_lens[b] + TILE_T - 1) / TILE_T;
  const int n_chunks = (n_tiles + chunk_tiles - 1) / chunk_tiles;
  if (n_chunks <= 1 || h >= H) return;            // one chunk: written directly by the attention kernel
  const size_t slot0 = ((size_t)b * H + h) * max_chunks;
  float m_tot = -INFINITY;
  for (int ck = 0; ck < n_chunks; ++ck) m_tot = fmaxf(m_tot, ws_ml[(slot0 + ck) * 2]);
  float l_tot = 0.f;
  f32x4 o = f32x4{0.f, 0.f, 0.f, 0.f};
  for (int ck = 0; ck < n_chunks; ++ck) {
    const float wgt = __builtin_amdgcn_exp2f(ws_ml[(slot0 + ck) * 2] - m_tot);
    l_tot += ws_ml[(slot0 + ck) * 2 + 1] * wgt;
    o += *(const f32x4*)(ws_o + (slot0 + ck) * D + d) * wgt;
  }
  uint2 pk;
  pk.x = pack_bf16_rne(o[0] / l_tot, o[1] / l_tot);
  pk.y = pack_bf16_rne(o[2] / l_tot, o[3] / l_tot);
  *(uint2*)(out + ((size_t)b * H + h) * D + d) = pk;
}

template <int D>
static hipError_t launch_decode_gqa_t(const PoolGeom& g, const char* pool_base, const void* q, void* out,
                                      const int32_t* d_ctx_lens, const int32_t* d_bt, int bt_stride,
                                      const int2* d_items, int n_items, int B, int H, float scale, int chunk_tiles,
                                      int max_chunks, float* ws_o, float* ws_ml, hipStream_t stream) {
  const float c = scale * 1.4426950408889634f;
  hipLaunchKernelGGL(decode_gqa_kernel<D>, dim3((unsigned)n_items * g.Hkv), dim3(256), 0, stream, pool_base,
                     g.page_bytes, g.head_bytes, g.tile_bytes, g.tiles_per_page, (const bf16_t*)q, (bf16_t*)out, d_ctx_lens,
                     d_bt, bt_stride, d_items, g.Hkv, H, H / g.Hkv, c, chunk_tiles, max_chunks, ws_o, ws_ml);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess || max_chunks <= 1) return e;
  hipLaunchKernelGGL(decode_combine_kernel<D>, dim3((unsigned)(H + 512 / D - 1) / (512 / D), B), dim3(128), 0, stream, (bf16_t*)out, d_ctx_lens, H, chunk_tiles,
                     max_chunks, ws_o, ws_ml);
  return hipGetLastError();
}

hipError_t launch_decode_gqa(const PoolGeom& g, const char* pool_base, const void* q, void* out,
                             const int32_t* d_ctx_lens, const int32_t* d_block_tables, int bt_stride,
                             const void* d_items, int n_items, int B, int H, float scale, int chunk_tiles,
                             int max_chunks, float* ws_o, float* ws_ml, hipStream_t stream) {
  if (g.dk == 128)
    return launch_decode_gqa_t<128>(g, pool_base, q, out, d_ctx_lens, d_block_tables, bt_stride, (const int2*)d_items,
                                    n_items, B, H, scale, chunk_tiles, max_chunks, ws_o, ws_ml, stream);
  if (g.dk == 64)
    return launch_decode_gqa_t<64>(g, pool_base, q, out, d_ctx_lens, d_block_tables, bt_stride, (const int2*)d_items,
                                   n_items, B, H, scale, chunk_tiles, max_chunks, ws_o, ws_ml, stream);
  return hipErrorInvalidValue;
}

}  // namespace spd
