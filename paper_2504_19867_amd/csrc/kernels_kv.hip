// Page write / gather kernels and the CU-id probe.
//
// Paper, "Prefill and Decode Workers": the K, V projections of a request are written into
// the KV cache during prefill and the cache is updated at every decode iteration.  These
// kernels move rows between dense [rows, heads, dim] tensors and the library's page layout
// (internal.h); they are pure copies, bit-exact.
#include "internal.h"

#include <algorithm>

namespace spd {

typedef unsigned short bf16_t;

// 16-byte accesses of data that passes through once (rows on their way into pages, pages on their
// way out): marked non-temporal, so that these streams leave the L2's contents to the attention kernels.
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
__device__ inline uint4 load_once(const void* p) {
  const u32x4 r = __builtin_nontemporal_load((const u32x4*)p);
  return uint4{r.x, r.y, r.z, r.w};
}
__device__ inline void store_once(void* p, uint4 v) { __builtin_nontemporal_store(u32x4{v.x, v.y, v.z, v.w}, (u32x4*)p); }

// grid (n_tiles + copy_cols, n_kv_heads), block 256.  One workgroup copies the touched token slots
// of one 16-token tile of one KV head.  The descriptors may lie in pinned host memory (one read
// per workgroup).  Workgroups past n_tiles copy copy_n16 16-byte pieces copy_src -> copy_dst
// instead: the step's metadata rides along in the same launch.
__global__ __launch_bounds__(256) void kv_write_kernel(char* __restrict__ base, uint64_t page_bytes,
                                                       uint32_t head_bytes, uint32_t tile_bytes,
                                                       uint32_t tile_k_bytes, const TileDesc* __restrict__ descs,
                                                       const bf16_t* __restrict__ k, const bf16_t* __restrict__ v,
                                                       int Hkv, int dk, int dv, int natural, int n_tiles,
                                                       uint4* __restrict__ copy_dst, const uint4* __restrict__ copy_src,
                                                       uint64_t copy_n16) {
  if ((int)blockIdx.x >= n_tiles) {
    const uint64_t blk = (uint64_t)(blockIdx.x - n_tiles) * gridDim.y + blockIdx.y;
    const uint64_t stride = (uint64_t)(gridDim.x - n_tiles) * gridDim.y * blockDim.x;
    for (uint64_t i = blk * blockDim.x + threadIdx.x; i < copy_n16; i += stride) copy_dst[i] = copy_src[i];
    return;
  }
  const TileDesc d = descs[blockIdx.x];
  const int g = blockIdx.y;
  char* tile = base + (uint64_t)d.page * page_bytes + (uint64_t)g * head_bytes + (uint64_t)d.sub * tile_bytes;
  // K part: [chunk][token][8 dims] (GQA) or natural [token][dim] rows (MLA latent), one 16-byte
  // piece per (chunk, token).  For the GQA order the pieces cross LDS so that both the row reads
  // (consecutive chunks of a token) and the page writes (consecutive tokens of a chunk) are contiguous.
  const int k_items = (dk >> 3) * TILE_T;
  if (natural) {
    for (int i = threadIdx.x; i < k_items; i += blockDim.x) {
      const int t = i / (dk >> 3), c = i % (dk >> 3);
      if (t >= d.t_begin && t < d.t_end)
        *(uint4*)(tile + (size_t)t * dk * 2 + (size_t)c * 16) =
            *(const uint4*)(k + ((size_t)(d.src_row + t - d.t_begin) * Hkv + g) * dk + c * 8);
    }
  }
  // V part: [d/32][token quad][d%16][(d/16)%2][4 tokens], one 16-byte piece per (d/32, quad, d%16).
  // The tile's rows go through LDS (16-byte loads of 8 dims, [token][dim]) and come out transposed.
  __shared__ uint4 ks[TILE_T][32 + 1];              // dk <= 256: 32 pieces per token, one of padding
  __shared__ bf16_t vs[TILE_T][256 + 8];            // dv <= 256; 8 elements of padding per row
  bf16_t* vt = (bf16_t*)(tile + tile_k_bytes);
  const int pieces = v ? (dv >> 3) * TILE_T : 0;
  // all row reads of the workgroup (K and V) are issued before anything waits for them
  for (int i = threadIdx.x; i < max(natural ? 0 : k_items, pieces); i += blockDim.x) {
    uint4 kr = uint4{0, 0, 0, 0}, vr = uint4{0, 0, 0, 0};
    const int tk = i / (dk >> 3), ck = i % (dk >> 3);
    const bool k_ok = !natural && i < k_items && tk >= d.t_begin && tk < d.t_end;
    if (k_ok) kr = *(const uint4*)(k + ((size_t)(d.src_row + tk - d.t_begin) * Hkv + g) * dk + ck * 8);
    const int tv = i / max(dv >> 3, 1), cv = i % max(dv >> 3, 1);
    const bool v_ok = i < pieces && tv >= d.t_begin && tv < d.t_end;
    if (v_ok) vr = *(const uint4*)(v + ((size_t)(d.src_row + tv - d.t_begin) * Hkv + g) * dv + cv * 8);
    if (k_ok) ks[tk][ck] = kr;
    if (v_ok) *(uint4*)&vs[tv][cv * 8] = vr;
  }
  __syncthreads();
  if (!natural) {
    for (int i = threadIdx.x; i < k_items; i += blockDim.x) {
      const int t = i & 15, c = i >> 4;
      if (t >= d.t_begin && t < d.t_end) *(uint4*)(tile + ((size_t)(c * 16 + t) << 4)) = ks[t][c];
    }
  }
  if (v == nullptr) return;
  const int v_items = (dv >> 5) * 64;
  for (int i = threadIdx.x; i < v_items; i += blockDim.x) {
    const int m = i & 15, c4 = (i >> 4) & 3, blk2 = i >> 6;
    bf16_t vals[8];
    bool all = true;
#pragma unroll
    for (int par = 0; par < 2; ++par)
#pragma unroll
      for (int tt = 0; tt < 4; ++tt) {
        const int t = 4 * c4 + tt, dd = 32 * blk2 + 16 * par + m;
        const bool ok = t >= d.t_begin && t < d.t_end;
        all = all && ok;
        vals[par * 4 + tt] = ok ? vs[t][dd] : (bf16_t)0;
      }
    bf16_t* dst = vt + ((size_t)((blk2 * 4 + c4) * 16 + m) << 3);
    if (all) {
      uint4 pk;
      pk.x = vals[0] | ((uint32_t)vals[1] << 16);
      pk.y = vals[2] | ((uint32_t)vals[3] << 16);
      pk.z = vals[4] | ((uint32_t)vals[5] << 16);
      pk.w = vals[6] | ((uint32_t)vals[7] << 16);
      *(uint4*)dst = pk;
    } else {
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const int t = 4 * c4 + (e & 3);
        if (t >= d.t_begin && t < d.t_end) dst[e] = vals[e];
      }
    }
  }
}

// The same page write for GQA pools with dk, dv <= 128, one workgroup per 16-token tile and group of
// up to HG KV heads: the descriptor (possibly in pinned host memory) is fetched once per group
// instead of once per head, and the row reads of all the group's heads are in flight together
// before the first head goes through LDS.  grid (n_tiles + copy_cols, ceil(Hkv / HG)), block 256.
// With ROPE the key rows are rotated on the way (rotary position embedding, token position = pos0 of the tile's
// descriptor + token slot; same arithmetic as rope_kernel: fp64 angle reduced to [-pi, pi], fp32 rotation, one
// rounding to bf16): the rotated piece goes to the page and back to the caller's k row, which the attention
// kernel of the same step reads.  A piece's partner (the other half of its pairs, in the half layout) is found
// in the LDS copy of the raw row.
struct RopeFuse {
  const double* w;        // [rot / 2] frequencies
  bf16_t* k_rw;           // the k tensor again, writable
  int rot, off;           // rotating entries per head, first rotating entry (multiples of 16 and 8)
  int interleaved;
};

__device__ inline float kv_bf_lo(uint32_t w) { return __builtin_bit_cast(float, w << 16); }
__device__ inline float kv_bf_hi(uint32_t w) { return __builtin_bit_cast(float, w & 0xffff0000u); }
__device__ inline uint32_t kv_pack_bf16(float a, float b) {
  typedef float f32x2_ __attribute__((ext_vector_type(2)));
  typedef __bf16 bf16x2_ __attribute__((ext_vector_type(2)));
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(f32x2_{a, b}, bf16x2_));
}

template <int HG, bool ROPE>
__global__ __launch_bounds__(256) void kv_write_heads_kernel(char* __restrict__ base, uint64_t page_bytes, uint32_t head_bytes,
                                                             uint32_t tile_bytes, uint32_t tile_k_bytes,
                                                             const TileDesc* __restrict__ descs, const bf16_t* __restrict__ k,
                                                             const bf16_t* __restrict__ v, int Hkv, int dk, int dv, int n_tiles,
                                                             uint4* __restrict__ copy_dst, const uint4* __restrict__ copy_src,
                                                             uint64_t copy_n16, RopeFuse rp) {
  if ((int)blockIdx.x >= n_tiles) {
    const uint64_t blk = (uint64_t)(blockIdx.x - n_tiles) * gridDim.y + blockIdx.y;
    const uint64_t stride = (uint64_t)(gridDim.x - n_tiles) * gridDim.y * blockDim.x;
    for (uint64_t i = blk * blockDim.x + threadIdx.x; i < copy_n16; i += stride) copy_dst[i] = copy_src[i];
    return;
  }
  __shared__ uint4 ks[TILE_T][16 + 1];              // dk <= 128: 16 pieces per token, one of padding
  __shared__ bf16_t vs[TILE_T][128 + 8];            // dv <= 128; 8 elements of padding per row
  const TileDesc d = descs[blockIdx.x];
  const int g0 = blockIdx.y * HG, ng = min(HG, Hkv - g0);
  const int i = threadIdx.x;
  const int ck_n = dk >> 3, cv_n = dv >> 3;         // 16-byte pieces per K row, per V row
  const int tk = i / ck_n, ck = i % ck_n, tv = i / cv_n, cv = i % cv_n;
  const bool k_ok = i < ck_n * TILE_T && tk >= d.t_begin && tk < d.t_end;
  const bool v_ok = i < cv_n * TILE_T && tv >= d.t_begin && tv < d.t_end;
  uint4 kr[HG], vr[HG];
#pragma unroll
  for (int g = 0; g < HG; ++g) {
    kr[g] = vr[g] = uint4{0, 0, 0, 0};
    if (g < ng && k_ok) kr[g] = load_once(k + ((size_t)(d.src_row + tk - d.t_begin) * Hkv + g0 + g) * dk + ck * 8);
    if (g < ng && v_ok) vr[g] = load_once(v + ((size_t)(d.src_row + tv - d.t_begin) * Hkv + g0 + g) * dv + cv * 8);
  }
  const int v_items = (dv >> 5) * 64;
  // the piece this thread carries to the page: token slot t_out, piece c_out of the row
  const int t_out = i & 15, c_out = i >> 4;
  const bool out_ok = i < ck_n * TILE_T && t_out >= d.t_begin && t_out < d.t_end;
  float cs[8], sn[8];
  int partner = -1;                                  // half layout: the piece that holds the other entry of each pair
  bool rotates = false, second = false;
  if constexpr (ROPE) {
    const int e0 = 8 * c_out - rp.off;               // the piece's first entry, counted from the rotating range's start
    rotates = out_ok && e0 >= 0 && e0 < rp.rot;
    if (rotates) {
      const int half = rp.rot >> 1;
      second = !rp.interleaved && e0 >= half;
      partner = rp.interleaved ? c_out : (second ? c_out - (half >> 3) : c_out + (half >> 3));
      const int pair0 = rp.interleaved ? (e0 >> 1) : (second ? e0 - half : e0);
      const double p = (double)(d.pad[0] + t_out);
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        if (rp.interleaved && j >= 4) break;
        const double turns = p * rp.w[pair0 + j] * 0.15915494309189535;   // angle / 2 pi
        const float r = (float)((turns - __builtin_rint(turns)) * 6.283185307179586);
        sincosf(r, &sn[j], &cs[j]);
      }
    }
  }
#pragma unroll
  for (int g = 0; g < HG; ++g) {
    if (g >= ng) break;
    char* tile = base + (uint64_t)d.page * page_bytes + (uint64_t)(g0 + g) * head_bytes + (uint64_t)d.sub * tile_bytes;
    if (k_ok) ks[tk][ck] = kr[g];
    if (v_ok) *(uint4*)&vs[tv][cv * 8] = vr[g];
    __syncthreads();
    // K part [chunk][token][8 dims]
    if (out_ok) {
      uint4 piece = ks[t_out][c_out];
      if constexpr (ROPE) {
        if (rotates) {
          uint32_t x[4] = {piece.x, piece.y, piece.z, piece.w};
          if (rp.interleaved) {                       // word j holds pair j: low half a, high half b
#pragma unroll
            for (int j = 0; j < 4; ++j) {
              const float xa = kv_bf_lo(x[j]), xb = kv_bf_hi(x[j]);
              x[j] = kv_pack_bf16(xa * cs[j] - xb * sn[j], xb * cs[j] + xa * sn[j]);
            }
          } else {
            const uint4 other = ks[t_out][partner];
            const uint32_t y[4] = {other.x, other.y, other.z, other.w};
#pragma unroll
            for (int j = 0; j < 4; ++j) {
              const float m0 = kv_bf_lo(x[j]), m1 = kv_bf_hi(x[j]), o0 = kv_bf_lo(y[j]), o1 = kv_bf_hi(y[j]);
              // first half: mine is a (a cos - b sin); second half: mine is b (b cos + a sin)
              x[j] = second ? kv_pack_bf16(m0 * cs[2 * j] + o0 * sn[2 * j], m1 * cs[2 * j + 1] + o1 * sn[2 * j + 1])
                            : kv_pack_bf16(m0 * cs[2 * j] - o0 * sn[2 * j], m1 * cs[2 * j + 1] - o1 * sn[2 * j + 1]);
            }
          }
          piece = uint4{x[0], x[1], x[2], x[3]};
          *(uint4*)(rp.k_rw + ((size_t)(d.src_row + t_out - d.t_begin) * Hkv + g0 + g) * dk + c_out * 8) = piece;
        }
      }
      store_once(tile + ((size_t)(c_out * 16 + t_out) << 4), piece);
    }
    // V part [d/32][token quad][d%16][(d/16)%2][4 tokens]
    if (i < v_items) {
      bf16_t* vt = (bf16_t*)(tile + tile_k_bytes);
      const int m = i & 15, c4 = (i >> 4) & 3, blk2 = i >> 6;
      bf16_t vals[8];
      bool all = true;
#pragma unroll
      for (int par = 0; par < 2; ++par)
#pragma unroll
        for (int tt = 0; tt < 4; ++tt) {
          const int t = 4 * c4 + tt, dd = 32 * blk2 + 16 * par + m;
          const bool ok = t >= d.t_begin && t < d.t_end;
          all = all && ok;
          vals[par * 4 + tt] = ok ? vs[t][dd] : (bf16_t)0;
        }
      bf16_t* dst = vt + ((size_t)((blk2 * 4 + c4) * 16 + m) << 3);
      if (all) {
        uint4 pk;
        pk.x = vals[0] | ((uint32_t)vals[1] << 16);
        pk.y = vals[2] | ((uint32_t)vals[3] << 16);
        pk.z = vals[4] | ((uint32_t)vals[5] << 16);
        pk.w = vals[6] | ((uint32_t)vals[7] << 16);
        store_once(dst, pk);
      } else {
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const int t = 4 * c4 + (e & 3);
          if (t >= d.t_begin && t < d.t_end) dst[e] = vals[e];
        }
      }
    }
    __syncthreads();
  }
}

// Inverse of kv_write_kernel, with the same 16-byte pieces: K pieces go straight back to their rows,
// the V tile is un-transposed through LDS and leaves as 16-byte row pieces.
__global__ __launch_bounds__(256) void kv_gather_kernel(const char* __restrict__ base, uint64_t page_bytes,
                                                        uint32_t head_bytes, uint32_t tile_bytes,
                                                        uint32_t tile_k_bytes, const TileDesc* __restrict__ descs,
                                                        bf16_t* __restrict__ k_out, bf16_t* __restrict__ v_out,
                                                        int Hkv, int dk, int dv, int natural) {
  const TileDesc d = descs[blockIdx.x];
  const int g = blockIdx.y;
  const char* tile = base + (uint64_t)d.page * page_bytes + (uint64_t)g * head_bytes + (uint64_t)d.sub * tile_bytes;
  const int k_items = (dk >> 3) * TILE_T;
  for (int i = threadIdx.x; i < k_items; i += blockDim.x) {
    const int t = i & 15, c = i >> 4;
    if (t >= d.t_begin && t < d.t_end) {
      const size_t off = natural ? (size_t)t * dk * 2 + (size_t)c * 16 : ((size_t)(c * 16 + t) << 4);
      *(uint4*)(k_out + ((size_t)(d.src_row + t - d.t_begin) * Hkv + g) * dk + c * 8) = load_once(tile + off);
    }
  }
  if (v_out == nullptr) return;
  __shared__ bf16_t vs[TILE_T][256 + 8];            // dv <= 256; 8 elements of padding per row
  const bf16_t* vt = (const bf16_t*)(tile + tile_k_bytes);
  const int v_items = (dv >> 5) * 64;               // 16-byte pieces of the tile: (d/32, token quad, d%16)
  for (int i = threadIdx.x; i < v_items; i += blockDim.x) {
    const int m = i & 15, c4 = (i >> 4) & 3, blk2 = i >> 6;
    const uint4 pk = load_once(vt + ((size_t)((blk2 * 4 + c4) * 16 + m) << 3));
    const uint32_t w[4] = {pk.x, pk.y, pk.z, pk.w};
#pragma unroll
    for (int e = 0; e < 8; ++e) {                   // element e = (d/16)%2 * 4 + token%4
      const int par = e >> 2, tt = e & 3;
      vs[4 * c4 + tt][32 * blk2 + 16 * par + m] = (bf16_t)(w[e >> 1] >> (16 * (e & 1)));
    }
  }
  __syncthreads();
  const int pieces = (dv >> 3) * TILE_T;
  for (int i = threadIdx.x; i < pieces; i += blockDim.x) {
    const int t = i / (dv >> 3), c = i % (dv >> 3);
    if (t >= d.t_begin && t < d.t_end)
      *(uint4*)(v_out + ((size_t)(d.src_row + t - d.t_begin) * Hkv + g) * dv + c * 8) = *(const uint4*)&vs[t][c * 8];
  }
}

// Each workgroup reports which XCD / shader engine / CU it ran on (hardware id registers).
__global__ void probe_kernel(int32_t* __restrict__ ids) {
  if (threadIdx.x == 0) {
    // s_getreg_b32: simm16 = (size-1) << 11 | offset << 6 | register id
    const uint32_t hw_id = __builtin_amdgcn_s_getreg((31 << 11) | 4);    // HW_REG_HW_ID
    const uint32_t xcc = __builtin_amdgcn_s_getreg((3 << 11) | 20);      // HW_REG_XCC_ID, bits 3:0
    const uint32_t cu = (hw_id >> 8) & 0xf, sh = (hw_id >> 12) & 0x1, se = (hw_id >> 13) & 0x7;
    ids[blockIdx.x] = (int32_t)((xcc << 16) | (se << 8) | (sh << 4) | cu);
  }
  // keep the workgroup resident for a moment so that the launch spreads over the allowed CUs
  const uint64_t t0 = __builtin_readcyclecounter();
  while (__builtin_readcyclecounter() - t0 < 20000) {
  }
}

// Plain streaming copy, 16 bytes per lane, grid-stride.
__global__ __launch_bounds__(256) void copy_kernel(uint4* __restrict__ dst, const uint4* __restrict__ src, uint64_t n16) {
  const uint64_t stride = (uint64_t)gridDim.x * blockDim.x;
  for (uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += stride) dst[i] = src[i];
}

// Read-only stream: every lane keeps eight independent 16-byte loads in flight, grid-stride over n16 pieces; what is
// read is folded into one word that is stored only if it equals a value it cannot practically take, so the loads stay
// and nothing is written.
__global__ __launch_bounds__(256) void read_kernel(const uint4* __restrict__ src, uint64_t n16, uint32_t* __restrict__ sink) {
  const uint64_t stride = (uint64_t)gridDim.x * blockDim.x;
  uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
  uint32_t acc = 0;
  for (; i + 7 * stride < n16; i += 8 * stride) {
    uint4 r[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) r[j] = load_once(src + i + j * stride);
#pragma unroll
    for (int j = 0; j < 8; ++j) acc ^= r[j].x ^ r[j].y ^ r[j].z ^ r[j].w;
  }
  for (; i < n16; i += stride) {
    const uint4 r = load_once(src + i);
    acc ^= r.x ^ r.y ^ r.z ^ r.w;
  }
  if (acc == 0x9e3779b9u && sink) sink[0] = acc;
}

// The same stream taken through LDS: every wave reads a contiguous part of the buffer with 1 KiB load instructions
// that write straight into its 16 KiB of LDS (as the attention kernels' tile loads do), up to 16 of them in flight;
// what is left over at the end goes the way of read_kernel.  Two workgroups per compute unit.
__global__ __launch_bounds__(256, 2) void read_lds_kernel(const uint4* __restrict__ src, uint64_t n16, uint32_t* __restrict__ sink) {
  __shared__ __attribute__((aligned(1024))) char lds[4 * 16384];
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
  const uint64_t waves = (uint64_t)gridDim.x * 4, gw = (uint64_t)blockIdx.x * 4 + wave;
  const uint64_t inst = n16 / 64 / waves;                   // 1 KiB instructions per wave
  const uint4* p = src + gw * inst * 64 + lane;
  const uint32_t base = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char*)lds + (uint32_t)wave * 16384;
  for (uint64_t i = 0; i < inst; ++i) {
    const uint32_t dst = base + (uint32_t)(i & 15) * 1024;
    asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, off nt\n\ts_waitcnt vmcnt(15)" ::"s"(dst), "v"(p + i * 64) : "memory");
  }
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  uint32_t acc = *(const uint32_t*)(lds + wave * 16384 + lane * 4);
  for (uint64_t i = waves * inst * 64 + (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += (uint64_t)gridDim.x * blockDim.x) {
    const uint4 r = load_once(src + i);
    acc ^= r.x ^ r.y ^ r.z ^ r.w;
  }
  if (acc == 0x9e3779b9u && sink) sink[0] = acc;
}

hipError_t launch_read_lds(const void* src, uint64_t bytes, int cus, uint32_t* sink, hipStream_t stream) {
  hipLaunchKernelGGL(read_lds_kernel, dim3((unsigned)cus * 2), dim3(256), 0, stream, (const uint4*)src, bytes / 16, sink);
  return hipGetLastError();
}

hipError_t launch_read(const void* src, uint64_t bytes, int cus, uint32_t* sink, hipStream_t stream) {
  hipLaunchKernelGGL(read_kernel, dim3((unsigned)cus * 8), dim3(256), 0, stream, (const uint4*)src, bytes / 16, sink);
  return hipGetLastError();
}

// One wave runs a chain of `iters` dependent integer adds (each waits for the one before: a fixed number of shader
// clock cycles whatever else the chip is doing) and reports how long that took on the constant-rate 100 MHz counter
// and on the shader cycle counter.  out[0] = constant-rate ticks, out[1] = cycle-counter ticks, out[2] = the chain's
// result (keeps it alive).
__global__ __launch_bounds__(64) void clock_probe_kernel(uint64_t iters, uint64_t* __restrict__ out) {
  uint32_t x = (uint32_t)threadIdx.x;
  const uint64_t w0 = wall_clock64();
  const uint64_t c0 = __builtin_readcyclecounter();
  for (uint64_t i = 0; i < iters; ++i) {
#pragma unroll
    for (int j = 0; j < 64; ++j) asm volatile("v_add_u32 %0, %0, %1" : "+v"(x) : "v"(x));
  }
  const uint64_t c1 = __builtin_readcyclecounter();
  const uint64_t w1 = wall_clock64();
  if (threadIdx.x == 0) {
    out[0] = w1 - w0;
    out[1] = c1 - c0;
    out[2] = x;
  }
}

hipError_t launch_clock_probe(uint64_t iters, uint64_t* d_out, hipStream_t stream) {
  hipLaunchKernelGGL(clock_probe_kernel, dim3(1), dim3(64), 0, stream, iters, d_out);
  return hipGetLastError();
}

// Does matrix work overlap vector work inside one wave, or only between waves?  One workgroup of five waves: waves 0
// and 4 share a SIMD, the other three idle.  Wave 0 times (shader cycles per iteration, 256 iterations each)
//   out[0]: one 32x32x16 bf16 MFMA per iteration (four accumulators in rotation),
//   out[1]: eight independent vector instructions per iteration (four v_exp_f32, four v_fma_f32),
//   out[2]: the MFMA followed by the same eight vector instructions,
// then, after a barrier, out[3]: its MFMA loop again while wave 4 runs the vector loop beside it (out[4]: wave 4's
// cycles per iteration in that phase).  out[5] keeps the results alive.
__global__ __launch_bounds__(320) void issue_probe_kernel(uint64_t* __restrict__ out) {
  typedef float f32x16_ __attribute__((ext_vector_type(16)));
  typedef __bf16 bf16x8_ __attribute__((ext_vector_type(8)));
  const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
  constexpr int N = 256;
  f32x16_ acc[4];
  for (int i = 0; i < 4; ++i)
    for (int e = 0; e < 16; ++e) acc[i][e] = 0.f;
  const uint4 araw = uint4{0x3f803f80u, 0x3f803f80u, 0x3f803f80u, 0x3f803f80u};
  const bf16x8_ a = __builtin_bit_cast(bf16x8_, araw);
  float x[8];
  for (int j = 0; j < 8; ++j) x[j] = 0.001f * (float)(threadIdx.x + j);
  auto valu8 = [&]() {
    asm volatile("v_exp_f32 %0, %0\n\tv_exp_f32 %1, %1\n\tv_exp_f32 %2, %2\n\tv_exp_f32 %3, %3\n\t"
                 "v_fma_f32 %4, %4, %4, %4\n\tv_fma_f32 %5, %5, %5, %5\n\tv_fma_f32 %6, %6, %6, %6\n\tv_fma_f32 %7, %7, %7, %7"
                 : "+v"(x[0]), "+v"(x[1]), "+v"(x[2]), "+v"(x[3]), "+v"(x[4]), "+v"(x[5]), "+v"(x[6]), "+v"(x[7]));
  };
  auto mfma1 = [&](int i) { acc[i & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, a, acc[i & 3], 0, 0, 0); };
  uint64_t t[6] = {0, 0, 0, 0, 0, 0};
  if (wave == 0) {
    uint64_t t0 = __builtin_readcyclecounter();
#pragma unroll 4
    for (int i = 0; i < N; ++i) { mfma1(i); __builtin_amdgcn_sched_barrier(0); }
    asm volatile("s_nop 7\n\ts_nop 7\n\ts_nop 7" ::: "memory");
    t[0] = __builtin_readcyclecounter() - t0;
    t0 = __builtin_readcyclecounter();
#pragma unroll 4
    for (int i = 0; i < N; ++i) { valu8(); __builtin_amdgcn_sched_barrier(0); }
    t[1] = __builtin_readcyclecounter() - t0;
    t0 = __builtin_readcyclecounter();
#pragma unroll 4
    for (int i = 0; i < N; ++i) { mfma1(i); __builtin_amdgcn_sched_barrier(0); valu8(); __builtin_amdgcn_sched_barrier(0); }
    asm volatile("s_nop 7\n\ts_nop 7\n\ts_nop 7" ::: "memory");
    t[2] = __builtin_readcyclecounter() - t0;
  }
  __syncthreads();
  if (wave == 0) {
    const uint64_t t0 = __builtin_readcyclecounter();
#pragma unroll 4
    for (int i = 0; i < N; ++i) { mfma1(i); __builtin_amdgcn_sched_barrier(0); }
    asm volatile("s_nop 7\n\ts_nop 7\n\ts_nop 7" ::: "memory");
    t[3] = __builtin_readcyclecounter() - t0;
  } else if (wave == 4) {
    const uint64_t t0 = __builtin_readcyclecounter();
#pragma unroll 4
    for (int i = 0; i < N; ++i) { valu8(); __builtin_amdgcn_sched_barrier(0); }
    t[4] = __builtin_readcyclecounter() - t0;
  }
  float keep = x[0] + x[1] + x[2] + x[3] + x[4] + x[5] + x[6] + x[7];
  for (int i = 0; i < 4; ++i) keep += acc[i][0];
  if ((threadIdx.x & 63) == 0) {
    if (wave == 0) {
      for (int i = 0; i < 4; ++i) out[i] = t[i] * 100 / N;        // hundredths of a cycle per iteration
      out[5] = (uint64_t)__builtin_bit_cast(uint32_t, keep);
    } else if (wave == 4) {
      out[4] = t[4] * 100 / N;
      out[6] = (uint64_t)__builtin_bit_cast(uint32_t, keep);
    }
  }
}

hipError_t launch_issue_probe(uint64_t* d_out, hipStream_t stream) {
  hipLaunchKernelGGL(issue_probe_kernel, dim3(1), dim3(320), 0, stream, d_out);
  return hipGetLastError();
}

hipError_t launch_copy(void* dst, const void* src, uint64_t bytes, int cus, hipStream_t stream) {
  hipLaunchKernelGGL(copy_kernel, dim3((unsigned)cus * 16), dim3(256), 0, stream, (uint4*)dst, (const uint4*)src, bytes / 16);
  return hipGetLastError();
}

bool kv_write_can_rotate(const PoolGeom& g) {
  return g.kind == SPD_KV_GQA && g.dk <= 128 && g.dv <= 128 && g.Hkv >= 2;
}

hipError_t launch_kv_write(const PoolGeom& g, char* pool_base, const TileDesc* d_tiles, int n_tiles, const void* k,
                           const void* v, hipStream_t stream, void* copy_dst, const void* copy_src, uint64_t copy_bytes,
                           const double* rope_w, int rot, int rot_off, bool interleaved) {
  const uint64_t n16 = copy_dst ? (copy_bytes + 15) / 16 : 0;
  const int copy_cols = n16 ? (int)std::min<uint64_t>(16, (n16 + 256ull * g.Hkv - 1) / (256ull * g.Hkv)) : 0;
  if (n_tiles <= 0 && copy_cols == 0) return hipSuccess;
  if (g.kind == SPD_KV_GQA && v != nullptr && g.dk <= 128 && g.dv <= 128 && g.Hkv >= 2) {
    constexpr int HG = 8;
    const int groups = (g.Hkv + HG - 1) / HG;
    // the metadata copy keeps its share of workgroups: copy_cols x Hkv of them before, the same number now
    const int cols = copy_cols ? (copy_cols * g.Hkv + groups - 1) / groups : 0;
    RopeFuse rp{rope_w, (bf16_t*)const_cast<void*>(k), rot, rot_off, interleaved ? 1 : 0};
    if (rope_w)
      hipLaunchKernelGGL((kv_write_heads_kernel<HG, true>), dim3(n_tiles + cols, groups), dim3(256), 0, stream, pool_base,
                         g.page_bytes, g.head_bytes, g.tile_bytes, g.tile_k_bytes, d_tiles, (const bf16_t*)k, (const bf16_t*)v,
                         g.Hkv, g.dk, g.dv, n_tiles, (uint4*)copy_dst, (const uint4*)copy_src, n16, rp);
    else
      hipLaunchKernelGGL((kv_write_heads_kernel<HG, false>), dim3(n_tiles + cols, groups), dim3(256), 0, stream, pool_base,
                         g.page_bytes, g.head_bytes, g.tile_bytes, g.tile_k_bytes, d_tiles, (const bf16_t*)k, (const bf16_t*)v,
                         g.Hkv, g.dk, g.dv, n_tiles, (uint4*)copy_dst, (const uint4*)copy_src, n16, rp);
    return hipGetLastError();
  }
  if (rope_w) return hipErrorInvalidValue;          // callers ask kv_write_can_rotate first
  hipLaunchKernelGGL(kv_write_kernel, dim3(n_tiles + copy_cols, g.Hkv), dim3(256), 0, stream, pool_base, g.page_bytes,
                     g.head_bytes, g.tile_bytes, g.tile_k_bytes, d_tiles, (const bf16_t*)k, (const bf16_t*)v, g.Hkv, g.dk,
                     g.dv, g.kind == SPD_KV_MLA_LATENT ? 1 : 0, n_tiles, (uint4*)copy_dst, (const uint4*)copy_src, n16);
  return hipGetLastError();
}

hipError_t launch_kv_gather(const PoolGeom& g, const char* pool_base, const TileDesc* d_tiles, int n_tiles, void* k_out,
                            void* v_out, hipStream_t stream) {
  if (n_tiles <= 0) return hipSuccess;
  hipLaunchKernelGGL(kv_gather_kernel, dim3(n_tiles, g.Hkv), dim3(256), 0, stream, pool_base, g.page_bytes,
                     g.head_bytes, g.tile_bytes, g.tile_k_bytes, d_tiles, (bf16_t*)k_out, (bf16_t*)v_out, g.Hkv, g.dk,
                     g.dv, g.kind == SPD_KV_MLA_LATENT ? 1 : 0);
  return hipGetLastError();
}

hipError_t launch_probe(int32_t* d_ids, int n_blocks, hipStream_t stream) {
  hipLaunchKernelGGL(probe_kernel, dim3(n_blocks), dim3(64), 0, stream, d_ids);
  return hipGetLastError();
}

}  // namespace spd
