// First step of the gated FFN: the gate and the up projection as ONE matrix product, with the
// activation applied to the accumulators.
//
// Paper, Evaluation "Implementation based on DistServe": the first two GEMMs of the gated FFN are
// fused into one.  With x [T, hidden] and the joint weight matrix w_gu [2 inter, hidden] (rows
// 64 b .. 64 b + 31 = gate rows 32 b .., rows 64 b + 32 .. 64 b + 63 = the up rows of the same outputs):
//     y = x . w_gu^T            out[t, 32 b + j] = silu(y[t, 64 b + j]) * y[t, 64 b + 32 + j]
// silu(z) = z / (1 + exp(-z)).  bf16 in, fp32 accumulation, one rounding to bf16 at the end.
//
// A dense contraction: v_mfma_f32_32x32x16_bf16.  One workgroup = 8 waves computes a tile of 256
// tokens x 256 joint columns (= 128 outputs); the waves form a 2 x 4 grid, each with 128 tokens x 64
// joint columns: one block of 32 gate columns and the 32 up columns that belong to them, so the
// activation needs nothing but the wave's own accumulators.  Both operands are contiguous along
// hidden; 32-wide slices of them stream from global memory straight into a ring of four LDS stages
// (global_load_lds_dwordx4, three slices ahead of the compute, one s_barrier per slice) and are read
// back with 16-byte reads in operand order.  Rows are 64 bytes in LDS; the four 16-byte chunks of a
// row are XOR-swizzled with bits 2..3 of the row number, which spreads 16 consecutive rows over all
// banks.
#include "internal.h"

namespace spd {

namespace {

typedef unsigned short bf16_t;
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));

constexpr int WAVES = 8;
constexpr int BM = 256, BNP = 256, BK = 32;     // tokens, joint columns, hidden entries per slice
constexpr int NSTAGE = 4, PD = NSTAGE - 1;
constexpr int A_BYTES = BM * BK * 2, B_BYTES = BNP * BK * 2, STAGE_BYTES = A_BYTES + B_BYTES;
constexpr int LPW = (A_BYTES + B_BYTES) / 1024 / WAVES;   // 1 KiB load instructions per wave per slice
static_assert(LPW == 4 && A_BYTES / 1024 == 2 * WAVES, "two A and two B load instructions per wave");

__device__ inline uint32_t cvt_bf16(float a) {
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(f32x2{a, a}, bf16x2)) & 0xffffu;
}
// 16 bytes per lane from global memory to LDS: lane i's data lands at lds_byte_addr + 16 * i.
// The compiler does not see this write; completion is tracked by hand with vmcnt.
__device__ inline void dma16s(const void* sbase, uint32_t voff, uint32_t lds_byte_addr) {
  asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(lds_byte_addr), "v"(voff), "s"(sbase) : "memory");
}
#define SPD_WAIT_VMCNT(N) __builtin_amdgcn_s_waitcnt(((N) & 15) | (7 << 4) | (15 << 8) | (((N) >> 4) << 14))

__global__ __launch_bounds__(512, 2) void ffn_gate_up_kernel(const bf16_t* __restrict__ x, const bf16_t* __restrict__ w,
                                                             bf16_t* __restrict__ out, int T, int K, int I, int tiles_m,
                                                             int tiles_n, int xcds) {
  __shared__ __attribute__((aligned(1024))) char smem[NSTAGE * STAGE_BYTES];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int n32 = lane & 31, hh = lane >> 5;
  const int wm = wave >> 2, wn = wave & 3;
  // Workgroup b runs on XCD b % xcds; every XCD takes a contiguous range of tiles, token tiles
  // fastest, so that the workgroups running together on an XCD share a slice of the weights.
  const int total = tiles_m * tiles_n;
  const int per = (total + xcds - 1) / xcds;
  const int slot = (int)blockIdx.x / xcds;
  const int tile_id = ((int)blockIdx.x % xcds) * per + slot;
  if (slot >= per || tile_id >= total) return;
  const int tm = tile_id % tiles_m, tn = tile_id / tiles_m;
  const int m0 = tm * BM, n0p = tn * BNP;
  const uint32_t smem_base = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char*)smem;
  const uint32_t pitch = (uint32_t)K * 2;

  // ---- slice loads.  Load instruction ii = wave + 8 j fills the 64 consecutive 16-byte slots
  // [64 ii, 64 ii + 64) of the stage: x rows first (row = slot / 4), then weight rows; slot s of a
  // row holds the row's chunk s ^ ((row >> 2) & 3).  Token rows past T re-read row T - 1.
  uint32_t ld_voff[LPW];
#pragma unroll
  for (int j = 0; j < LPW; ++j) {
    const int ii = wave + WAVES * j;
    const int s = (ii & 15) * 64 + lane, row = s >> 2, chunk = (s & 3) ^ ((row >> 2) & 3);
    const int grow = ii < 16 ? min(row, T - 1 - m0) : row;
    ld_voff[j] = (uint32_t)grow * pitch + (uint32_t)chunk * 16;
  }
  const char* a_base = (const char*)(x + (size_t)m0 * K);
  const char* b_base = (const char*)(w + (size_t)n0p * K);
  const int n_slices = K / BK;
  int pt = 0, ct = 0;
  auto produce_one = [&]() __attribute__((always_inline)) {
    if (pt >= n_slices) return;
    const uint32_t stage = __builtin_amdgcn_readfirstlane(smem_base + (uint32_t)(pt % NSTAGE) * STAGE_BYTES);
#pragma unroll
    for (int j = 0; j < LPW; ++j) {
      const int ii = wave + WAVES * j;
      dma16s((ii < 16 ? a_base : b_base) + (size_t)pt * (BK * 2), ld_voff[j], stage + (uint32_t)ii * 1024);
    }
    ++pt;
  };

  // ---- LDS operand addresses inside a stage: row r, k-step ks (16 hidden entries), lane half hh
  // reads chunk 2 ks + hh of the row
  const int sw = (n32 >> 2) & 3;
  int a_off[2], b_off[2];
#pragma unroll
  for (int ks = 0; ks < 2; ++ks) {
    a_off[ks] = (wm * 128 + n32) * 64 + (((2 * ks + hh) ^ sw) * 16);
    b_off[ks] = A_BYTES + (wn * 64 + n32) * 64 + (((2 * ks + hh) ^ sw) * 16);
  }

  // acc[mb][0] = gate, acc[mb][1] = up: element i of lane (n32, hh) is token 32 mb + 8 (i / 4) + 4 hh + i % 4,
  // column n32 of the wave's block
  f32x16 acc[4][2];
#pragma unroll
  for (int mb = 0; mb < 4; ++mb)
#pragma unroll
    for (int nb = 0; nb < 2; ++nb)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[mb][nb][e] = 0.f;

#pragma unroll
  for (int t = 0; t < PD; ++t) produce_one();

  for (; ct < n_slices;) {
    // this wave's loads of slice ct are done when at most (slices issued after it) * LPW remain
    const int later = pt - ct - 1;
    if (later >= 2) SPD_WAIT_VMCNT(2 * LPW);
    else if (later == 1) SPD_WAIT_VMCNT(LPW);
    else SPD_WAIT_VMCNT(0);
    // all waves: the slice has landed, and everyone is done with the one before, whose stage is refilled next
    asm volatile("s_barrier" ::: "memory");
    produce_one();
    const char* sbase = smem + (ct % NSTAGE) * STAGE_BYTES;
    ++ct;
    uint4 a[2][4], b[2][2];
#pragma unroll
    for (int ks = 0; ks < 2; ++ks) {
#pragma unroll
      for (int nb = 0; nb < 2; ++nb) b[ks][nb] = *(const uint4*)(sbase + b_off[ks] + nb * (32 * 64));
#pragma unroll
      for (int mb = 0; mb < 4; ++mb) a[ks][mb] = *(const uint4*)(sbase + a_off[ks] + mb * (32 * 64));
    }
#pragma unroll
    for (int ks = 0; ks < 2; ++ks)
#pragma unroll
      for (int mb = 0; mb < 4; ++mb)
#pragma unroll
        for (int nb = 0; nb < 2; ++nb)
          acc[mb][nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a[ks][mb]),
                                                                __builtin_bit_cast(bf16x8, b[ks][nb]), acc[mb][nb], 0, 0, 0);
  }

  // ---- activation and store: lanes 0..31 of a store hold 32 consecutive outputs of one token
  const int col = tn * (BNP / 2) + wn * 32 + n32;
#pragma unroll
  for (int mb = 0; mb < 4; ++mb)
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const int t = m0 + wm * 128 + mb * 32 + 8 * (i >> 2) + 4 * hh + (i & 3);
      const float g = acc[mb][0][i], u = acc[mb][1][i];
      const float s = g * __builtin_amdgcn_rcpf(1.f + __builtin_amdgcn_exp2f(-1.4426950408889634f * g));
      if (t < T) out[(size_t)t * I + col] = (bf16_t)cvt_bf16(s * u);
    }
}

// rows of the joint matrix from the two weight matrices: 16-byte pieces, one row of pieces per workgroup row
__global__ __launch_bounds__(256) void ffn_pack_kernel(const uint4* __restrict__ wg, const uint4* __restrict__ wu,
                                                       uint4* __restrict__ dst, int row_pieces, long n_rows) {
  for (long r = blockIdx.x; r < n_rows; r += gridDim.x) {
    const long blk = r >> 6;
    const int j = (int)(r & 63);
    const uint4* src = (j < 32 ? wg : wu) + (blk * 32 + (j & 31)) * (long)row_pieces;
    for (int c = threadIdx.x; c < row_pieces; c += blockDim.x) dst[r * row_pieces + c] = src[c];
  }
}

}  // namespace

int ffn_tile_tokens() { return BM; }

hipError_t launch_ffn_gate_up(const void* x, const void* w_gu, void* out, int T, int K, int I, int xcds, hipStream_t stream) {
  const int tiles_m = (T + BM - 1) / BM, tiles_n = 2 * I / BNP;
  const int total = tiles_m * tiles_n;
  if (total < xcds) xcds = 1;
  const int per = (total + xcds - 1) / xcds;
  hipLaunchKernelGGL(ffn_gate_up_kernel, dim3((unsigned)(per * xcds)), dim3(64 * WAVES), 0, stream, (const bf16_t*)x,
                     (const bf16_t*)w_gu, (bf16_t*)out, T, K, I, tiles_m, tiles_n, xcds);
  return hipGetLastError();
}

hipError_t launch_ffn_pack(const void* w_gate, const void* w_up, void* w_gu, int K, int I, hipStream_t stream) {
  const long n_rows = 2L * I;
  hipLaunchKernelGGL(ffn_pack_kernel, dim3((unsigned)std::min<long>(n_rows, 4096)), dim3(256), 0, stream, (const uint4*)w_gate,
                     (const uint4*)w_up, (uint4*)w_gu, K / 8, n_rows);
  return hipGetLastError();
}

}  // namespace spd
