// First step of the gated FFN: the gate and the up projection as ONE matrix product, with the
// activation applied to the accumulators.
//
// Paper, Evaluation "Implementation based on DistServe": the first two GEMMs of the gated FFN are
// fused into one.  With x [T, hidden] and the joint weight matrix w_gu [2 inter, hidden] (rows
// 64 b .. 64 b + 31 = gate rows 32 b .., rows 64 b + 32 .. 64 b + 63 = the up rows of the same outputs;
// stored tile by tile, 256 joint rows x 32 hidden entries, in the order the kernel's LDS stage has):
//     y = x . w_gu^T            out[t, 32 b + j] = silu(y[t, 64 b + j]) * y[t, 64 b + 32 + j]
// silu(z) = z / (1 + exp(-z)).  bf16 in, fp32 accumulation, one rounding to bf16 at the end.
//
// A dense contraction: v_mfma_f32_32x32x16_bf16.
//
// Prompt batches (ffn_gate_up_kernel): one workgroup = 8 waves computes a tile of 256 tokens x 256
// joint columns (= 128 outputs); the waves form a 2 x 4 grid, each with 128 tokens x 64 joint
// columns: one block of 32 gate columns and the 32 up columns that belong to them, so the
// activation needs nothing but the wave's own accumulators.  Both operands are contiguous along
// hidden; 32-wide slices of them stream from global memory straight into a ring of four LDS stages
// (global_load_lds_dwordx4, one s_barrier per slice) and are read back with 16-byte reads in operand
// order, one slice ahead of the MFMAs, into a second set of operand registers.  Rows are 64 bytes in
// LDS; the four 16-byte chunks of a row are XOR-swizzled with bits 2..3 of the row number, which
// spreads 16 consecutive rows over all banks.
//
// Decode batches (up to 256 tokens) are bound by reading the weights once: the same kernel with smaller
// tiles (128 x 128 with four waves, 64 x 128 with a ring of six stages, two workgroups per compute unit; 64 x 256
// with eight waves and a ring of seven stages where that still gives every unit a workgroup),
// so that every compute unit of the share has a workgroup and more weight bytes are in flight per unit.
#include "internal.h"

namespace spd {

namespace {

typedef unsigned short bf16_t;
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));

constexpr int BK = 32;                          // hidden entries per slice

__device__ inline uint32_t cvt_bf16(float a) {
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(f32x2{a, a}, bf16x2)) & 0xffffu;
}
// 16 bytes per lane from global memory to LDS: lane i's data lands at lds_byte_addr + 16 * i.
// The compiler does not see this write; completion is tracked by hand with vmcnt.
__device__ inline void dma16s(const void* sbase, uint32_t voff, uint32_t lds_byte_addr) {
  asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(lds_byte_addr), "v"(voff), "s"(sbase) : "memory");
}
#define SPD_WAIT_VMCNT(N) __builtin_amdgcn_s_waitcnt(((N) & 15) | (7 << 4) | (15 << 8) | (((N) >> 4) << 14))

// MB: 32-token blocks per wave; WNW: waves along the joint columns; NSTAGE: LDS ring.  The waves form a
// 2 x WNW grid, each with 32 MB tokens x 64 joint columns; the workgroup's tile is 64 MB tokens x 64 WNW
// joint columns.
// <4, 4, 4>: 256 x 256 for prompt batches.  For small batches the product is bound by reading the
// weights once, and what counts is how many weight bytes a CU keeps in flight: <2, 2, 4>: 128 x 128,
// four waves, two workgroups per CU, for up to 128 tokens; <1, 2, 6>: 64 x 128 with a ring of six
// 12 KiB stages, of which 8 KiB are weights, two workgroups per CU, for up to 64 tokens; <1, 4, 7>: 64 x 256,
// eight waves, a ring of seven 20 KiB stages of which 16 KiB are weights (x is a fifth of what a workgroup
// loads instead of a third), one workgroup per CU.
template <int MB, int WNW, int NSTAGE>
__global__ __launch_bounds__(128 * WNW, 2) void ffn_gate_up_kernel(const bf16_t* __restrict__ x, const bf16_t* __restrict__ w,
                                                                   bf16_t* __restrict__ out, int T, int K, int I, int tiles_m,
                                                                   int tiles_n, int xcds) {
  constexpr int WAVES = 2 * WNW, BM = 64 * MB, BNP = 64 * WNW, PD = NSTAGE - 1;
  constexpr int A_BYTES = BM * BK * 2, B_BYTES = BNP * BK * 2, STAGE_BYTES = A_BYTES + B_BYTES;
  // 1 KiB load instructions per wave per slice.  Where x has fewer pieces than there are waves (a 64-token tile under
  // eight waves), every wave loads one: piece wave % A_LOADS, so two waves write the same bytes to the same place.
  constexpr int A_LOADS = A_BYTES / 1024, B_LOADS = B_BYTES / 1024;
  constexpr bool A_SHARED = A_LOADS < WAVES;
  constexpr int LPW = A_SHARED ? 1 + B_LOADS / WAVES : (A_LOADS + B_LOADS) / WAVES;
  static_assert(B_LOADS % WAVES == 0 && (A_SHARED ? WAVES % A_LOADS == 0 : A_LOADS % WAVES == 0), "loads divide evenly over the waves");
  __shared__ __attribute__((aligned(1024))) char smem[NSTAGE * STAGE_BYTES];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int n32 = lane & 31, hh = lane >> 5;
  const int wm = wave / WNW, wn = wave % WNW;
  // Workgroup b runs on XCD b % xcds, and the workgroups of an XCD start in the order of b.  Every
  // XCD takes a contiguous range of weight tiles (columns) and all token tiles; inside it the tiles
  // are ordered so that the 16 or so workgroups running together form a block of about 4 x 4 tiles:
  // each slice of x and of the weights that misses the XCD's L2 then feeds four workgroups.
  int tm, tn;
  if (xcds > 1) {
    const int xcd = (int)blockIdx.x % xcds, slot = (int)blockIdx.x / xcds;
    const int base = tiles_n / xcds, rem = tiles_n % xcds;
    const int cnt = base + (xcd < rem ? 1 : 0), start = xcd * base + min(xcd, rem);
    if (slot >= cnt * tiles_m) return;
    const int full = cnt / 4;                   // column blocks of four weight tiles; the last one narrower
    int cb, q, wb;
    if (slot < full * 4 * tiles_m) {
      cb = slot / (4 * tiles_m);
      q = slot % (4 * tiles_m);
      wb = 4;
    } else {
      cb = full;
      q = slot - full * 4 * tiles_m;
      wb = cnt - 4 * full;
    }
    tm = q / wb;
    tn = start + 4 * cb + q % wb;
  } else {
    if ((int)blockIdx.x >= tiles_m * tiles_n) return;
    tm = (int)blockIdx.x % tiles_m;
    tn = (int)blockIdx.x / tiles_m;
  }
  const int m0 = tm * BM, n0p = tn * BNP;
  const uint32_t smem_base = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char*)smem;
  const uint32_t pitch = (uint32_t)K * 2;

  // ---- slice loads.  Load instruction ii = wave + WAVES j fills the 64 consecutive 16-byte slots
  // [64 ii, 64 ii + 64) of the stage: x rows first (row = slot / 4), then weight rows; slot s of a
  // row holds the row's chunk s ^ ((row >> 2) & 3).  Token rows past T re-read row T - 1.
  // piece number of this wave's load j: below A_LOADS a piece of x, from there on pieces of the weights
  auto piece_of = [&](int j) __attribute__((always_inline)) -> int {
    if constexpr (A_SHARED) return j == 0 ? wave % A_LOADS : A_LOADS + wave + WAVES * (j - 1);
    else return wave + WAVES * j;
  };
  uint32_t ld_voff[LPW];
#pragma unroll
  for (int j = 0; j < LPW; ++j) {
    const int ii = piece_of(j);
    if (ii < A_LOADS) {
      const int s = ii * 64 + lane, row = s >> 2, chunk = (s & 3) ^ ((row >> 2) & 3);
      ld_voff[j] = (uint32_t)min(row, T - 1 - m0) * pitch + (uint32_t)chunk * 16;
    } else {
      ld_voff[j] = (uint32_t)((ii - A_LOADS) * 64 + lane) * 16;   // the weights are stored in this very order
    }
  }
  const char* a_base = (const char*)(x + (size_t)m0 * K);
  // weight tile (joint rows 256 t .., slice ks) is 16 KiB at ((t * K / 32) + ks) * 16 KiB; a 128-row tile is half of one
  const char* b_base = (const char*)w + ((size_t)(n0p / 256) * (K / BK)) * 16384 + (size_t)(n0p % 256) * 64;
  const int n_slices = K / BK;
  int pt = 0, ct = 0;
  // load instruction j of slice pt; after the last one the slice counts as issued
  auto produce_piece = [&](int j) __attribute__((always_inline)) {
    if (pt >= n_slices) return;
    const uint32_t stage = __builtin_amdgcn_readfirstlane(smem_base + (uint32_t)(pt % NSTAGE) * STAGE_BYTES);
    const int ii = piece_of(j);
    dma16s(ii < A_LOADS ? a_base + (size_t)pt * (BK * 2) : b_base + (size_t)pt * 16384, ld_voff[j], stage + (uint32_t)ii * 1024);
    if (j == LPW - 1) ++pt;
  };
  auto produce_one = [&]() __attribute__((always_inline)) {
#pragma unroll
    for (int j = 0; j < LPW; ++j) produce_piece(j);
  };

  // ---- LDS operand addresses inside a stage: row r, k-step ks (16 hidden entries), lane half hh
  // reads chunk 2 ks + hh of the row
  const int sw = (n32 >> 2) & 3;
  int a_off[2], b_off[2];
#pragma unroll
  for (int ks = 0; ks < 2; ++ks) {
    a_off[ks] = (wm * (32 * MB) + n32) * 64 + (((2 * ks + hh) ^ sw) * 16);
    b_off[ks] = A_BYTES + (wn * 64 + n32) * 64 + (((2 * ks + hh) ^ sw) * 16);
  }

  // acc[mb][0] = gate, acc[mb][1] = up: element i of lane (n32, hh) is token 32 mb + 8 (i / 4) + 4 hh + i % 4,
  // column n32 of the wave's block
  f32x16 acc[MB][2];
#pragma unroll
  for (int mb = 0; mb < MB; ++mb)
#pragma unroll
    for (int nb = 0; nb < 2; ++nb)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[mb][nb][e] = 0.f;

#pragma unroll
  for (int t = 0; t < PD; ++t) produce_one();

  // The operands of slice t + 1 are read from LDS into a second set of registers while the matrix
  // cores work on slice t, so the barrier of a step guards the slice AFTER the one being multiplied.
  // Reads, tile loads and MFMAs alternate in program order: issued in a bunch behind the barrier, the
  // reads of all the waves keep the LDS pipe busy for most of a slice's matrix time, and no wave gets
  // to its MFMAs before its own reads are accepted.
  constexpr int N_READS = 2 * (MB + 2), N_MEM = N_READS + LPW, N_MFMA = 4 * MB;
  struct Ops { uint4 a[2][MB], b[2][2]; };
  auto read_op = [&](int slice, Ops& o, int n) __attribute__((always_inline)) {   // operand n in order of use
    const char* sbase = smem + (slice % NSTAGE) * STAGE_BYTES;
    const int ks = n / (MB + 2), r = n % (MB + 2);
    if (r < 2) o.b[ks][r] = *(const uint4*)(sbase + b_off[ks] + r * (32 * 64));
    else o.a[ks][r - 2] = *(const uint4*)(sbase + a_off[ks] + (r - 2) * (32 * 64));
  };
  auto load_ops = [&](int slice, Ops& o) __attribute__((always_inline)) {
#pragma unroll
    for (int n = 0; n < N_READS; ++n) read_op(slice, o, n);
  };
  // this wave's loads of slice s are done when at most (slices issued after it) * LPW remain
  auto wait_slice = [&](int s) __attribute__((always_inline)) {
    const int later = pt - s - 1;
    if (NSTAGE > 6 && later >= 5) SPD_WAIT_VMCNT(5 * LPW);
    else if (NSTAGE > 5 && later >= 4) SPD_WAIT_VMCNT(4 * LPW);
    else if (NSTAGE > 4 && later == 3) SPD_WAIT_VMCNT(3 * LPW);
    else if (later >= 2) SPD_WAIT_VMCNT(2 * LPW);
    else if (later == 1) SPD_WAIT_VMCNT(LPW);
    else SPD_WAIT_VMCNT(0);
  };
  // one step: slice t + 1 becomes readable for all waves (and everyone is done reading slice t - 1,
  // whose stage is refilled); slice t is multiplied, and the step's memory instructions (the operand
  // reads of slice t + 1, with the four loads of slice t + 3 evenly among them) go behind its MFMAs
  auto step = [&](int t, const Ops& cur, Ops& nxt) __attribute__((always_inline)) {
    const bool more = t + 1 < n_slices;
    if (more) wait_slice(t + 1);
    asm volatile("s_barrier" ::: "memory");
    int n_mem = 0, n_read = 0;
#pragma unroll
    for (int i = 0; i < N_MFMA; ++i) {
      const int ks = i / (2 * MB), mb = (i % (2 * MB)) / 2, nb = i % 2;
      acc[mb][nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, cur.a[ks][mb]),
                                                            __builtin_bit_cast(bf16x8, cur.b[ks][nb]), acc[mb][nb], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (; n_mem * N_MFMA < (i + 1) * N_MEM; ++n_mem) {
        if (n_mem % (N_MEM / LPW) == 1) {
          produce_piece(n_mem / (N_MEM / LPW));
        } else {
          if (more) read_op(t + 1, nxt, n_read);
          ++n_read;
        }
      }
      __builtin_amdgcn_sched_barrier(0);
    }
  };
  Ops o0, o1;
  wait_slice(0);
  asm volatile("s_barrier" ::: "memory");
  load_ops(0, o0);
  for (; ct < n_slices; ct += 2) {
    step(ct, o0, o1);
    if (ct + 1 < n_slices) step(ct + 1, o1, o0);
  }

  // ---- activation and store: lanes 0..31 of a store hold 32 consecutive outputs of one token
  const int col = tn * (BNP / 2) + wn * 32 + n32;
#pragma unroll
  for (int mb = 0; mb < MB; ++mb)
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const int t = m0 + wm * (32 * MB) + mb * 32 + 8 * (i >> 2) + 4 * hh + (i & 3);
      const float g = acc[mb][0][i], u = acc[mb][1][i];
      const float s = g * __builtin_amdgcn_rcpf(1.f + __builtin_amdgcn_exp2f(-1.4426950408889634f * g));
      if (t < T) out[(size_t)t * I + col] = (bf16_t)cvt_bf16(s * u);
    }
}

// The packed weights from the two weight matrices, one 16-byte piece per thread and step: piece
// number i of the output lies in tile i / 1024 = (tn, ks), row r = (i % 1024) / 4, slot s = i % 4, and
// holds the hidden entries 32 ks + 8 (s ^ ((r >> 2) & 3)) .. + 7 of joint row 256 tn + r.
__global__ __launch_bounds__(256) void ffn_pack_kernel(const uint4* __restrict__ wg, const uint4* __restrict__ wu,
                                                       uint4* __restrict__ dst, int n_ks, long n_pieces) {
  const long stride = (long)gridDim.x * blockDim.x;
  for (long i = (long)blockIdx.x * blockDim.x + threadIdx.x; i < n_pieces; i += stride) {
    const long tile = i >> 10;
    const int r = (int)(i & 1023) >> 2, sl = (int)(i & 3);
    const long tn = tile / n_ks;
    const int ks = (int)(tile % n_ks);
    const long R = tn * 256 + r;                // joint row: blocks of 32 gate rows + their 32 up rows
    const long n = (R >> 6) * 32 + (R & 31);
    const uint4* src = ((R & 63) < 32 ? wg : wu) + n * (long)(n_ks * 4) + ks * 4 + (sl ^ ((r >> 2) & 3));
    dst[i] = *src;
  }
}

}  // namespace

template <int MB, int WNW, int NSTAGE>
static hipError_t launch_tiles(const void* x, const void* w_gu, void* out, int T, int K, int I, int xcds, hipStream_t stream) {
  constexpr int BM = 64 * MB, BNP = 64 * WNW;
  const int tiles_m = (T + BM - 1) / BM, tiles_n = 2 * I / BNP;
  if (tiles_n < xcds) xcds = 1;
  const int per = xcds > 1 ? ((tiles_n + xcds - 1) / xcds) * tiles_m : tiles_m * tiles_n;
  hipLaunchKernelGGL((ffn_gate_up_kernel<MB, WNW, NSTAGE>), dim3((unsigned)(per * xcds)), dim3(128 * WNW), 0, stream, (const bf16_t*)x,
                     (const bf16_t*)w_gu, (bf16_t*)out, T, K, I, tiles_m, tiles_n, xcds);
  return hipGetLastError();
}

hipError_t launch_ffn_gate_up(const void* x, const void* w_gu, void* out, int T, int K, int I, int xcds, int cus,
                              hipStream_t stream) {
  // small batches are bound by reading the weights: the small tile where the large one would leave
  // half of the share's compute units without a workgroup
  const int large_tiles = ((T + 255) / 256) * (2 * I / 256);
  if (T <= 64) {
    // 64 x 256 tiles (one workgroup per CU, 96 KiB of weights in flight) where they give nearly every compute
    // unit of the share a workgroup; 64 x 128 tiles (two per CU, 80 KiB in flight) otherwise
    const int wide_tiles = 2 * I / 256;
    if (8 * wide_tiles >= 7 * cus) return launch_tiles<1, 4, 7>(x, w_gu, out, T, K, I, xcds, stream);
    return launch_tiles<1, 2, 6>(x, w_gu, out, T, K, I, xcds, stream);
  }
  if (T <= 128 || (T <= 256 && 2 * large_tiles <= cus)) return launch_tiles<2, 2, 4>(x, w_gu, out, T, K, I, xcds, stream);
  return launch_tiles<4, 4, 4>(x, w_gu, out, T, K, I, xcds, stream);
}

hipError_t launch_ffn_pack(const void* w_gate, const void* w_up, void* w_gu, int K, int I, hipStream_t stream) {
  const long n_pieces = 2L * I * K / 8;
  hipLaunchKernelGGL(ffn_pack_kernel, dim3((unsigned)std::min<long>((n_pieces + 255) / 256, 8192)), dim3(256), 0, stream,
                     (const uint4*)w_gate, (const uint4*)w_up, (uint4*)w_gu, K / 32, n_pieces);
  return hipGetLastError();
}

}  // namespace spd
