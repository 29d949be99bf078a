// FP8 pages of the latent (MLA) KV cache: page write (quantising) and gather (dequantising).
//
// Paper, Evaluation "Model": DeepSeek-V3 is served with FP8 precision; the paper says no more.  The reading taken
// here for the cache of the latent path: a cached row c = [ckv (512) ; krope (64)] keeps its rope entries in bf16
// and its ckv entries as OCP FP8 E4M3 codes (largest finite value 448, no infinities) with one fp32 scale per block
// of 128 entries,
//     scale_b = amax_b / 448  (1 if the block is all zero),    code_i = E4M3(clamp(x_i / scale_b, -448, 448)),
// rounded to nearest even; the division and the scale in fp32.  A row takes 656 bytes instead of 1152:
//     [512 codes][4 scales, fp32][64 rope entries, bf16]
// and a page is page_tokens such rows in token order.  The decode kernel reads these rows and multiplies with
// decode(code) * scale rounded to bf16.
//
// Both kernels: one workgroup per 16-token tile, 16 lanes per token; a lane owns 32 consecutive ckv entries (a
// quarter of a scale block: the block's maximum is formed over 4 neighbouring lanes).
#include "internal.h"

namespace spd {

namespace {
typedef unsigned short bf16_t;
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));

constexpr int ROW = FP8_ROW_BYTES;   // 656
constexpr float E4M3_MAX = 448.f;

__device__ inline float bf_lo(uint32_t w) { return __builtin_bit_cast(float, w << 16); }
__device__ inline float bf_hi(uint32_t w) { return __builtin_bit_cast(float, w & 0xffff0000u); }
__device__ inline uint32_t pack_bf16(float a, float b) {
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(f32x2{a, b}, bf16x2));
}
__device__ inline float clamp448(float y) { return fminf(fmaxf(y, -E4M3_MAX), E4M3_MAX); }
}  // namespace

// grid (n_tiles + copy_cols), block 256.  latent: dense [rows, 576] bf16.
__global__ __launch_bounds__(256) void kv_write_latent_fp8_kernel(char* __restrict__ base, uint64_t page_bytes,
                                                                  uint32_t tile_bytes, const TileDesc* __restrict__ descs,
                                                                  const bf16_t* __restrict__ latent, int n_tiles,
                                                                  uint4* __restrict__ copy_dst, const uint4* __restrict__ copy_src,
                                                                  uint64_t copy_n16) {
  if ((int)blockIdx.x >= n_tiles) {
    const uint64_t blk = blockIdx.x - n_tiles;
    const uint64_t stride = (uint64_t)(gridDim.x - n_tiles) * blockDim.x;
    for (uint64_t i = blk * blockDim.x + threadIdx.x; i < copy_n16; i += stride) copy_dst[i] = copy_src[i];
    return;
  }
  const TileDesc d = descs[blockIdx.x];
  const int t = threadIdx.x >> 4, l = threadIdx.x & 15;
  if (t < d.t_begin || t >= d.t_end) return;        // whole groups of 16 lanes leave together: the shuffles below stay inside a group of 4
  const bf16_t* src = latent + (size_t)(d.src_row + t - d.t_begin) * 576;
  char* row = base + (uint64_t)d.page * page_bytes + (uint64_t)d.sub * tile_bytes + (size_t)t * ROW;
  // 32 entries of this lane: four 16-byte pieces
  uint32_t w[16];
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const uint4 p = *(const uint4*)(src + 32 * l + 8 * j);
    w[4 * j] = p.x; w[4 * j + 1] = p.y; w[4 * j + 2] = p.z; w[4 * j + 3] = p.w;
  }
  float amax = 0.f;
#pragma unroll
  for (int j = 0; j < 16; ++j) amax = fmaxf(amax, fmaxf(fabsf(bf_lo(w[j])), fabsf(bf_hi(w[j]))));
  amax = fmaxf(amax, __shfl_xor(amax, 1));
  amax = fmaxf(amax, __shfl_xor(amax, 2));
  const float scale = amax > 0.f ? amax / E4M3_MAX : 1.f;
  uint32_t codes[8];
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    // four entries per word: entries 4 j .. 4 j + 3 = the two halves of w[2 j] and w[2 j + 1]
    int pk = 0;
    pk = __builtin_amdgcn_cvt_pk_fp8_f32(clamp448(bf_lo(w[2 * j]) / scale), clamp448(bf_hi(w[2 * j]) / scale), pk, false);
    pk = __builtin_amdgcn_cvt_pk_fp8_f32(clamp448(bf_lo(w[2 * j + 1]) / scale), clamp448(bf_hi(w[2 * j + 1]) / scale), pk, true);
    codes[j] = (uint32_t)pk;
  }
  *(uint4*)(row + 32 * l) = uint4{codes[0], codes[1], codes[2], codes[3]};
  *(uint4*)(row + 32 * l + 16) = uint4{codes[4], codes[5], codes[6], codes[7]};
  if ((l & 3) == 0) *(float*)(row + 512 + 4 * (l >> 2)) = scale;
  if (l < 8) *(uint4*)(row + 528 + 16 * l) = *(const uint4*)(src + 512 + 8 * l);
}

// grid (n_tiles), block 256.  out: dense [rows, 576] bf16 = decode(code) * scale rounded to bf16, rope as stored.
__global__ __launch_bounds__(256) void kv_gather_latent_fp8_kernel(const char* __restrict__ base, uint64_t page_bytes,
                                                                   uint32_t tile_bytes, const TileDesc* __restrict__ descs,
                                                                   bf16_t* __restrict__ out) {
  const TileDesc d = descs[blockIdx.x];
  const int t = threadIdx.x >> 4, l = threadIdx.x & 15;
  if (t < d.t_begin || t >= d.t_end) return;
  const char* row = base + (uint64_t)d.page * page_bytes + (uint64_t)d.sub * tile_bytes + (size_t)t * ROW;
  bf16_t* dst = out + (size_t)(d.src_row + t - d.t_begin) * 576;
  const float scale = *(const float*)(row + 512 + 4 * (l >> 2));
#pragma unroll
  for (int half = 0; half < 2; ++half) {
    const uint4 c = *(const uint4*)(row + 32 * l + 16 * half);
    const uint32_t cw[4] = {c.x, c.y, c.z, c.w};
    uint32_t o[8];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const f32x2 a = __builtin_amdgcn_cvt_pk_f32_fp8((int)cw[j], false), b = __builtin_amdgcn_cvt_pk_f32_fp8((int)cw[j], true);
      o[2 * j] = pack_bf16(a[0] * scale, a[1] * scale);
      o[2 * j + 1] = pack_bf16(b[0] * scale, b[1] * scale);
    }
    *(uint4*)(dst + 32 * l + 16 * half) = uint4{o[0], o[1], o[2], o[3]};
    *(uint4*)(dst + 32 * l + 16 * half + 8) = uint4{o[4], o[5], o[6], o[7]};
  }
  if (l < 8) *(uint4*)(dst + 512 + 8 * l) = *(const uint4*)(row + 528 + 16 * l);
}

hipError_t launch_kv_write_fp8(const PoolGeom& g, char* pool_base, const TileDesc* d_tiles, int n_tiles, const void* latent,
                               hipStream_t stream, void* copy_dst, const void* copy_src, uint64_t copy_bytes) {
  const uint64_t n16 = copy_dst ? (copy_bytes + 15) / 16 : 0;
  const int copy_cols = n16 ? (int)std::min<uint64_t>(16, (n16 + 255) / 256) : 0;
  if (n_tiles <= 0 && copy_cols == 0) return hipSuccess;
  hipLaunchKernelGGL(kv_write_latent_fp8_kernel, dim3(n_tiles + copy_cols), dim3(256), 0, stream, pool_base, g.page_bytes,
                     g.tile_bytes, d_tiles, (const bf16_t*)latent, n_tiles, (uint4*)copy_dst, (const uint4*)copy_src, n16);
  return hipGetLastError();
}

hipError_t launch_kv_gather_fp8(const PoolGeom& g, const char* pool_base, const TileDesc* d_tiles, int n_tiles, void* out,
                                hipStream_t stream) {
  if (n_tiles <= 0) return hipSuccess;
  hipLaunchKernelGGL(kv_gather_latent_fp8_kernel, dim3(n_tiles), dim3(256), 0, stream, pool_base, g.page_bytes, g.tile_bytes,
                     d_tiles, (bf16_t*)out);
  return hipGetLastError();
}

}  // namespace spd
