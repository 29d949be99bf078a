// Decode step, MLA latent cache (DeepSeek-V2-style multi-head latent attention, absorbed form).
//
// Paper, Evaluation "Model": DeepSeek-V2-Lite / V3 are served through the same two workers; the
// paper names the model only.  Per token the cache holds ONE latent row c_t = [ckv_t (512) ;
// krope_t (64)] shared by all heads.  For request b and head h with absorbed query q[b,h,:576]:
//     s[h,t]      = scale * q[b,h,:] . c_t
//     out[b,h,:]  = sum_{t<n} softmax_t(s[h,:]) * c_t[0:512]
// so the same bytes act as keys (contraction over the 576 dims) and as values (contraction over
// the tokens).  34.8 kflop per 1152-byte row: the fp32 vector units cannot keep up with HBM, the
// matrix cores must; the heads (<= 16) are the MFMA column dimension.
//
// One workgroup (4 waves) owns one (request, chunk of the context).  Steps of 16 tokens (18 KiB,
// contiguous in the page: latent pages keep the natural [token][dim] order) stream
// HBM -> LDS with global_load_lds_dwordx4 into a 4-stage ring, 3 steps ahead.  The ring takes
// 72 KiB, so two workgroups share a CU: 108 KiB are in flight per CU, and one workgroup's
// waits and start-up are covered by the other one's arithmetic.
// Out of LDS the rows are read twice, in the two operand orders:
//     S^T[token, head] = C[16 x 576] . Q^T[576 x 16]      ds_read_b128     + v_mfma_f32_16x16x32_bf16
//     O^T[dim, head]  += C^T[16 dims x 16 tokens] . P^T    ds_read_b64_tr_b16 + v_mfma_f32_16x16x16_bf16
// Every wave computes the (small) score product and the softmax statistics redundantly and owns
// 128 of the 512 output dims, so no cross-wave reduction is ever needed.  Split-K partials go to
// the same workspace / combine kernel as the GQA path.
//
// With two waves per SIMD little hides latency but the wave's own instruction stream, so both
// products are software-pipelined: LDS operand reads run a ring of 8 operands ahead of the MFMAs,
// the score product accumulates into three independent accumulators so that back-to-back MFMAs never
// wait for each other's result, and the second product of a step is issued in the next iteration,
// behind that step's first operand reads.  The loop reads no block table entry from memory and divides
// nothing: the chunk's page ids sit in one register (lane i = the chunk's i-th page).
#include "internal.h"

namespace spd {

typedef unsigned short bf16_t;
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef short s16x4 __attribute__((ext_vector_type(4)));

namespace mla {
constexpr int DL = 576;               // latent dims per token
constexpr int DV = 512;               // leading dims that act as values
constexpr int ROW_BYTES = DL * 2;     // 1152
constexpr int CH = DL / 8;            // 72 16-byte chunks per row
constexpr int STEP_T = 16;            // tokens per step
constexpr int STAGE_BYTES = STEP_T * ROW_BYTES;   // 18432
constexpr int NSTAGE = 4;
constexpr int PD = NSTAGE - 1;
constexpr int NI = STAGE_BYTES / 1024;            // 18 load instructions per step
constexpr int WAVES = 4;
constexpr int LPW = (NI + WAVES - 1) / WAVES;     // 5 for waves 0 and 1, 4 for waves 2 and 3
constexpr int KS = DL / 32;                       // 18 k-steps of the score product
constexpr int VB = DV / 16 / WAVES;               // 8 value blocks of 16 dims per wave
}  // namespace mla

__device__ inline uint32_t mla_pack_bf16(float a, float b) {
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(f32x2{a, b}, bf16x2));
}
__device__ inline void mla_dma16(const void* gptr, uint32_t lds_byte_addr) {
  asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, off" ::"s"(lds_byte_addr), "v"(gptr) : "memory");
}
// The same with the address split in a wave-uniform base and a 32-bit per-lane offset.
__device__ inline void mla_dma16s(const void* sbase, uint32_t voff, uint32_t lds_byte_addr) {
  // non-temporal: a decode step reads every latent row once, and the L2 is shared with the prefill partition
  asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, %2 nt" ::"s"(lds_byte_addr), "v"(voff), "s"(sbase) : "memory");
}
// max over the four 16-lane rows of a wave, on the vector ALU: the row swaps exchange odd rows of
// the first register with even rows of the second (rows of 16, then of 32 lanes)
__device__ inline float mla_max_over_rows(float x) {
  float y = x;
  asm volatile("s_nop 1\n\tv_permlane16_swap_b32 %0, %1\n\ts_nop 1" : "+v"(x), "+v"(y));
  x = fmaxf(x, y);
  y = x;
  asm volatile("s_nop 1\n\tv_permlane32_swap_b32 %0, %1\n\ts_nop 1" : "+v"(x), "+v"(y));
  return fmaxf(x, y);
}
// wait until at most N of the wave's vector memory loads are outstanding and all of its LDS reads have returned
// (the value operands read in the iteration before are used after the barrier, and the stage they came from is
// loaded into again right behind it)
#define SPD_MLA_WAIT_VMCNT(N) __builtin_amdgcn_s_waitcnt(((N) & 15) | (7 << 4) | (0 << 8) | (((N) >> 4) << 14))

// grid (n_items), block 256: work item = (request, chunk).  chunk_steps = 16-token steps per chunk.
// FP8: the pages hold 656-byte rows (512 E4M3 codes, 4 fp32 scales, 64 bf16 rope entries; kernels_kv_fp8.hip).  Such
// rows cannot go to LDS as they are: a step's rows travel through registers instead (16-byte pieces, two steps'
// worth in flight per lane), are multiplied out to bf16 (decode(code) * scale, rounded once) and stored into the
// stage in the very layout the bf16 path loads, so everything after the stage is shared.
template <bool FP8>
__global__ __launch_bounds__(256, 2) void decode_mla_kernel(
    const char* __restrict__ pool, uint64_t page_bytes, int steps_per_page, const bf16_t* __restrict__ q,
    bf16_t* __restrict__ out, const int32_t* __restrict__ ctx_lens, const int32_t* __restrict__ bt, int bt_stride,
    const int2* __restrict__ items, int H, float c /* scale * log2(e) */, int chunk_steps, int max_chunks, float* __restrict__ ws_o,
    float* __restrict__ ws_ml) {
  using namespace mla;
  __shared__ __attribute__((aligned(1024))) char smem[NSTAGE * STAGE_BYTES];
  const int2 item = items[blockIdx.x];
  const int b = item.x, chunk = item.y;
  const int n = ctx_lens[b];
  const int n_steps_all = (n + STEP_T - 1) / STEP_T;
  const int step0 = chunk * chunk_steps;
  if (step0 >= n_steps_all) return;
  const int n_steps = min(n_steps_all - step0, chunk_steps);
  const int n_chunks = (n_steps_all + chunk_steps - 1) / chunk_steps;
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int col = lane & 15, c4 = lane >> 4;       // col: head (B operand / accumulator column) or token (A operand row)
  const int32_t* bt_row = bt + (size_t)b * bt_stride;
  const uint32_t smem_base = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char*)smem;

  // absorbed-query fragments: B operand, column = head, dims 8 (4 s + c4) .. + 7 for k-step s
  bf16x8 qf[KS];
#pragma unroll
  for (int s = 0; s < KS; ++s) {
    uint4 raw = uint4{0, 0, 0, 0};
    if (col < H) raw = *(const uint4*)(q + ((size_t)b * H + col) * DL + 8 * (4 * s + c4));
    qf[s] = __builtin_bit_cast(bf16x8, raw);
  }

  // ---- loads: instruction ii = wave + 4 j fills LDS slots [64 ii, 64 ii + 64) of the stage;
  // slot s of row r holds the row's chunk s ^ (r & 7)
  uint32_t ld_off[LPW];
#pragma unroll
  for (int j = 0; j < LPW; ++j) {
    const int slot = (wave + WAVES * j) * 64 + lane, row = slot / CH, sl = slot % CH;
    ld_off[j] = (uint32_t)(row * ROW_BYTES + ((sl ^ (row & 7)) * 16));
  }
  const bool five = wave + WAVES * (LPW - 1) < NI;   // this wave issues LPW loads per step (else LPW - 1)
  // A step's loads: the wave-uniform source address and LDS stage first, then the instructions.
  // A load instruction occupies the CU's address unit for 16 cycles, and the wave that issues it
  // stalls meanwhile: in the loop they are handed out one at a time between MFMAs.
  auto load_src = [&](int st) -> const char* {
    const int gs = step0 + st;
    const int page = bt_row[gs / steps_per_page];
    return pool + (uint64_t)page * page_bytes + (size_t)(gs % steps_per_page) * STAGE_BYTES;
  };
  auto load_one = [&](const char* src, int st, int j) {
    if (j < LPW - 1 || five)
      mla_dma16s(src, ld_off[j], smem_base + (uint32_t)(st % NSTAGE) * STAGE_BYTES + (uint32_t)(wave + WAVES * j) * 1024);
  };
  auto issue_loads = [&](int st) {            // st: step index inside the chunk
    const char* src = load_src(st);
#pragma unroll
    for (int j = 0; j < LPW; ++j) load_one(src, st, j);
  };

  // ---- LDS operand addresses (byte offsets inside a stage)
  // score operand (k-step s): row = col, chunk 4 s + c4  ->  slot (4 s + c4) ^ (col & 7);
  // bit 2 of the swizzle flips the parity of s, hence two bases (even / odd s) + 128 * (s / 2)
  const int f = (col >> 2) & 1;
  const int k_base = col * ROW_BYTES + ((c4 ^ (col & 3)) * 16);
  const int k_even = k_base + 64 * f, k_odd = k_base + 64 * (1 - f);
  // value operand (16 dims of block blk): in each 16-lane group, lane r supplies row 4 c4 + r / 4
  // and dims 4 (r % 4) .. + 3; the transpose read hands lane i dim i of those 4 tokens
  const int v_row = 4 * c4 + (col >> 2);
  const int v_sw = v_row & 7;
  int v_base[4];                                   // by blk & 3; add 128 * (blk / 4)
#pragma unroll
  for (int b3 = 0; b3 < 4; ++b3) {
    const int ch_low = (2 * b3 + ((col & 3) >> 1)) ^ v_sw;         // low three bits of the chunk index
    v_base[b3] = v_row * ROW_BYTES + (16 * wave) * 16 + ch_low * 16 + (col & 1) * 8;
  }

  f32x4 O[VB];
#pragma unroll
  for (int i = 0; i < VB; ++i) O[i] = f32x4{0.f, 0.f, 0.f, 0.f};
  float m = -INFINITY, l = 0.f;

  // ---- FP8 rows: piece q = thread + 256 j (j < 3) of a step's 16 x 41 16-byte pieces; piece pc of a row is 16 codes
  // (pc < 32), the scales (pc = 32, fetched word by word with the codes they belong to) or 8 rope entries (pc > 32)
  constexpr int FP8_PIECES = FP8_ROW_BYTES / 16;             // 41
  constexpr int FP8_STEP_BYTES = STEP_T * FP8_ROW_BYTES;     // 10496
  struct Fp8Regs { uint4 d[3]; float sc[3]; };
  auto fp8_load = [&](const char* src, Fp8Regs& r) {
#pragma unroll
    for (int j = 0; j < 3; ++j) {
      // every thread issues the same six loads (a piece past the step's end repeats the last one, a piece without a
      // scale reads the row's last): with loads under branches the compiler cannot count what is in flight, and
      // waits for all of it wherever it needs any
      const int qd = min((int)threadIdx.x + 256 * j, STEP_T * FP8_PIECES - 1), row = qd / FP8_PIECES, pc = qd % FP8_PIECES;
      r.d[j] = *(const uint4*)(src + row * FP8_ROW_BYTES + pc * 16);
      r.sc[j] = *(const float*)(src + row * FP8_ROW_BYTES + 512 + 4 * min(pc >> 3, 3));
    }
  };
  auto fp8_store = [&](int st, const Fp8Regs& r) {
    char* stage = smem + (st % NSTAGE) * STAGE_BYTES;
#pragma unroll
    for (int j = 0; j < 3; ++j) {
      const int qd = (int)threadIdx.x + 256 * j, row = qd / FP8_PIECES, pc = qd % FP8_PIECES;
      if (qd >= STEP_T * FP8_PIECES || pc == 32) continue;
      char* lrow = stage + row * ROW_BYTES;
      if (pc > 32) {                                         // rope entries: chunk 64 + (pc - 33), as they are
        *(uint4*)(lrow + (((64 + pc - 33) ^ (row & 7)) * 16)) = r.d[j];
      } else {                                               // 16 codes -> chunks 2 pc and 2 pc + 1
        const uint32_t cw[4] = {r.d[j].x, r.d[j].y, r.d[j].z, r.d[j].w};
        uint32_t o[8];
#pragma unroll
        for (int k4 = 0; k4 < 4; ++k4) {
          const f32x2 a = __builtin_amdgcn_cvt_pk_f32_fp8((int)cw[k4], false), bb = __builtin_amdgcn_cvt_pk_f32_fp8((int)cw[k4], true);
          o[2 * k4] = mla_pack_bf16(a[0] * r.sc[j], a[1] * r.sc[j]);
          o[2 * k4 + 1] = mla_pack_bf16(bb[0] * r.sc[j], bb[1] * r.sc[j]);
        }
        *(uint4*)(lrow + (((2 * pc) ^ (row & 7)) * 16)) = uint4{o[0], o[1], o[2], o[3]};
        *(uint4*)(lrow + (((2 * pc + 1) ^ (row & 7)) * 16)) = uint4{o[4], o[5], o[6], o[7]};
      }
    }
  };
  auto fp8_src = [&](int st) -> const char* {
    const int gs = step0 + st;
    const int page = bt_row[gs / steps_per_page];
    return pool + (uint64_t)page * page_bytes + (size_t)(gs % steps_per_page) * FP8_STEP_BYTES;
  };
  // Two register sets that swap roles from step to step: iteration st stores step st + 1 out of one set and loads
  // step st + 3 into the same set, while step st + 2 is on its way into the other.  (Handing the values from set
  // to set instead made the compiler wait, at the end of every iteration, for the loads issued in it: 267 µs
  // against 228 at the DeepSeek-V2-Lite decode batch.  A third set, three steps in flight, changed nothing.)
  Fp8Regs set_a, set_b;
  if constexpr (FP8) {
    // steps 0 and 1 on their way, step 0 into its stage, step 2 behind it
    fp8_load(fp8_src(0), set_a);
    if (n_steps > 1) fp8_load(fp8_src(1), set_b);
    fp8_store(0, set_a);
    if (n_steps > 2) fp8_load(fp8_src(2), set_a);
  } else {
#pragma unroll
    for (int t = 0; t < PD; ++t)
      if (t < n_steps) issue_loads(t);
  }
  // The loop itself touches neither the block table in memory nor a division: lane i of `pages` holds the id of
  // the chunk's i-th page, the step to load next is tracked as (page, step inside the page).
  const int page_first = step0 / steps_per_page;
  const int n_pages_all = (n_steps_all + steps_per_page - 1) / steps_per_page;
  const int pages = bt_row[min(page_first + lane, n_pages_all - 1)];   // a chunk spans at most 64 pages (the host sees to it)
  int nl_page = (step0 + PD) / steps_per_page - page_first, nl_sub = (step0 + PD) % steps_per_page;
  // Draw the compiler's wait for the query loads (and the page ids) to this point, after the first steps are on
  // their way: left to itself it waits at their first use inside the loop, with a count that knows
  // nothing of the loads issued by hand, and every iteration would drain the prefetch queue.
#pragma unroll
  for (int s = 0; s < KS; ++s) asm volatile("" ::"v"(__builtin_bit_cast(uint4, qf[s]).x));
  asm volatile("" ::"v"(pages));

  constexpr int RING = 8;
  static_assert(RING == VB, "all value operands of a step are read ahead");
  // The second product of a step is issued at the start of the next iteration, between that step's first operand
  // reads and its first product, whose LDS latency it covers; the last one follows the loop.
  s16x4 vring[RING];
  uint2 pb = uint2{0u, 0u};
  auto step_body = [&](int st, Fp8Regs& set) __attribute__((always_inline)) {
    // this wave's loads of step st are done when at most (steps issued after it) * (its loads per step) remain
    const int later = min(PD - 1, n_steps - 1 - st);
    if constexpr (FP8) {
      SPD_MLA_WAIT_VMCNT(63);                      // the register-staged loads are the compiler's to wait for
    } else if (five) {
      if (later >= 2) SPD_MLA_WAIT_VMCNT(2 * LPW);
      else if (later == 1) SPD_MLA_WAIT_VMCNT(LPW);
      else SPD_MLA_WAIT_VMCNT(0);
    } else {
      if (later >= 2) SPD_MLA_WAIT_VMCNT(2 * (LPW - 1));
      else if (later == 1) SPD_MLA_WAIT_VMCNT(LPW - 1);
      else SPD_MLA_WAIT_VMCNT(0);
    }
    asm volatile("s_barrier" ::: "memory");        // step st has landed for all waves; stage of st - 1 is free
    const bool more = st + PD < n_steps;
    const int page_next = __builtin_amdgcn_readlane(pages, nl_page & 63);
    const char* src_next = pool + (uint64_t)page_next * page_bytes + (uint32_t)nl_sub * (FP8 ? FP8_STEP_BYTES : STAGE_BYTES);
    if (++nl_sub == steps_per_page) {
      nl_sub = 0;
      ++nl_page;
    }
    if constexpr (FP8) {
      // step st + 1 out of its registers into its stage (free since step st - 3), step st + 3 into the registers
      if (st + 1 < n_steps) fp8_store(st + 1, set);
      if (more) fp8_load(src_next, set);
    }

    const char* stage = smem + (st % NSTAGE) * STAGE_BYTES;
    const int tok0 = (step0 + st) * STEP_T;         // first token of the step
    auto read_s = [&](int sk) -> uint4 {
      return *(const uint4*)(stage + ((sk & 1) ? k_odd : k_even) + 128 * (sk >> 1));
    };
    auto read_v = [&](int blk) -> s16x4 {
      return __builtin_amdgcn_ds_read_tr16_b64_v4i16(
          (__attribute__((address_space(3))) s16x4*)(stage + v_base[blk & 3] + 128 * (blk >> 2)));
    };

    // ---- S^T = C . Q^T: k-step sk accumulates into accumulator sk % 3, so that back-to-back
    // MFMAs never wait for each other's result.  The loads of step st + PD go out between the
    // MFMAs, one every third.
    f32x4 acc[3];
#pragma unroll
    for (int i = 0; i < 3; ++i) acc[i] = f32x4{0.f, 0.f, 0.f, 0.f};
    uint4 ring[RING];
#pragma unroll
    for (int o = 0; o < RING; ++o) ring[o] = read_s(o);
    __builtin_amdgcn_sched_barrier(0);              // keep the issue order below (reads stay ahead of their use)
    if (st > 0) {                                   // O^T += C^T . P^T of the step before (never a context's last)
#pragma unroll
      for (int blk = 0; blk < VB; ++blk)
        O[blk] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(vring[blk], __builtin_bit_cast(s16x4, pb), O[blk], 0, 0, 0);
    }
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int sk = 0; sk < KS; ++sk) {
      acc[sk % 3] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, ring[sk % RING]), qf[sk], acc[sk % 3], 0, 0, 0);
      if (sk + RING < KS) ring[sk % RING] = read_s(sk + RING);
      if constexpr (!FP8)
        if (sk % 3 == 1 && sk / 3 < LPW && more) load_one(src_next, st + PD, sk / 3);
      __builtin_amdgcn_sched_barrier(0);
    }
    // value operands: in flight while the vector ALU does the softmax
#pragma unroll
    for (int o = 0; o < RING; ++o) vring[o] = read_v(o);
    __builtin_amdgcn_sched_barrier(0);
    f32x4 S = acc[0] + acc[1] + acc[2];
    // lane holds, for head col, tokens tok0 + 4 c4 + i
    if (tok0 + STEP_T > n) {
#pragma unroll
      for (int i = 0; i < 4; ++i)
        if (tok0 + 4 * c4 + i >= n) S[i] = -INFINITY;
    }
    float mx = fmaxf(fmaxf(S[0], S[1]), fmaxf(S[2], S[3]));
    mx = mla_max_over_rows(mx);
    const float m_new = fmaxf(m, mx);
    const float mc = m_new * c;
    float p[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) p[i] = __builtin_amdgcn_exp2f(S[i] * c - mc);
    const float psum = (p[0] + p[1]) + (p[2] + p[3]);
    pb = uint2{mla_pack_bf16(p[0], p[1]), mla_pack_bf16(p[2], p[3])};
    if (__builtin_amdgcn_ballot_w64(m_new > m) != 0) {        // rescale only when some running maximum moved
      const float alpha = __builtin_amdgcn_exp2f((m - m_new) * c);
      l *= alpha;
#pragma unroll
      for (int blk = 0; blk < VB; ++blk) O[blk] *= alpha;
      m = m_new;
    }
    l += psum;
  };
  if constexpr (FP8) {
    for (int st = 0; st < n_steps; st += 2) {      // step st + 1 sits in set_b when st is even
      step_body(st, set_b);
      if (st + 1 < n_steps) step_body(st + 1, set_a);
    }
  } else {
    for (int st = 0; st < n_steps; ++st) step_body(st, set_a);
  }
  // ---- the last step's second product.  Tokens of this lane's operand: tok_last + 4 c4 + {0..3}; slots past the
  // context hold arbitrary bytes and are cleared (their weights are zero, but 0 x NaN is not).
  {
    const int t0 = (step0 + n_steps - 1) * STEP_T + 4 * c4;
    const uint32_t m01 = (t0 + 0 < n ? 0x0000ffffu : 0u) | (t0 + 1 < n ? 0xffff0000u : 0u);
    const uint32_t m23 = (t0 + 2 < n ? 0x0000ffffu : 0u) | (t0 + 3 < n ? 0xffff0000u : 0u);
#pragma unroll
    for (int blk = 0; blk < VB; ++blk) {
      uint2 r = __builtin_bit_cast(uint2, vring[blk]);
      r.x &= m01;
      r.y &= m23;
      O[blk] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(__builtin_bit_cast(s16x4, r), __builtin_bit_cast(s16x4, pb), O[blk], 0, 0, 0);
    }
  }

  l += __shfl_xor(l, 16);
  l += __shfl_xor(l, 32);
  if (col < H) {
    const size_t head = (size_t)b * H + col;
    if (n_chunks == 1) {
      const float inv = 1.f / l;
      bf16_t* op = out + head * DV + 128 * wave + 4 * c4;
#pragma unroll
      for (int blk = 0; blk < VB; ++blk) {
        uint2 pk;
        pk.x = mla_pack_bf16(O[blk][0] * inv, O[blk][1] * inv);
        pk.y = mla_pack_bf16(O[blk][2] * inv, O[blk][3] * inv);
        *(uint2*)(op + 16 * blk) = pk;
      }
    } else {
      const size_t slot = head * max_chunks + chunk;
      float* wp = ws_o + slot * DV + 128 * wave + 4 * c4;
#pragma unroll
      for (int blk = 0; blk < VB; ++blk) *(f32x4*)(wp + 16 * blk) = O[blk];
      if (wave == 0 && c4 == 0) {
        ws_ml[slot * 2] = m * c;
        ws_ml[slot * 2 + 1] = l;
      }
    }
  }
}

// grid (H, B), block 128: merge the chunks of one (request, head); four output dims per thread, so that all
// workgroups of a batch are resident at once and the launch is one round of loads deep.
__global__ __launch_bounds__(128) void decode_mla_combine_kernel(bf16_t* __restrict__ out,
                                                                const int32_t* __restrict__ ctx_lens, int H,
                                                                int chunk_steps, int max_chunks,
                                                                const float* __restrict__ ws_o,
                                                                const float* __restrict__ ws_ml) {
  static_assert(mla::DV == 4 * 128, "one thread per four output dims");
  const int h = blockIdx.x, b = blockIdx.y, d = 4 * threadIdx.x;
  const int n_steps = (ctx_lens[b] + mla::STEP_T - 1) / mla::STEP_T;
  const int n_chunks = (n_steps + chunk_steps - 1) / chunk_steps;
  if (n_chunks <= 1) return;
  const size_t slot0 = ((size_t)b * H + h) * max_chunks;
  float m_tot = -INFINITY;
  for (int ck = 0; ck < n_chunks; ++ck) m_tot = fmaxf(m_tot, ws_ml[(slot0 + ck) * 2]);
  float l_tot = 0.f;
  f32x4 o = f32x4{0.f, 0.f, 0.f, 0.f};
  for (int ck = 0; ck < n_chunks; ++ck) {
    const float wgt = __builtin_amdgcn_exp2f(ws_ml[(slot0 + ck) * 2] - m_tot);
    l_tot += ws_ml[(slot0 + ck) * 2 + 1] * wgt;
    o += *(const f32x4*)(ws_o + (slot0 + ck) * mla::DV + d) * wgt;
  }
  uint2 pk;
  pk.x = mla_pack_bf16(o[0] / l_tot, o[1] / l_tot);
  pk.y = mla_pack_bf16(o[2] / l_tot, o[3] / l_tot);
  *(uint2*)(out + ((size_t)b * H + h) * mla::DV + d) = pk;
}

int decode_mla_step_tokens() { return mla::STEP_T; }

hipError_t launch_decode_mla(const PoolGeom& g, const char* pool_base, const void* q, void* out,
                             const int32_t* d_ctx_lens, const int32_t* d_block_tables, int bt_stride,
                             const void* d_items, int n_items, int B, int H, float scale, int chunk_steps,
                             int max_chunks, float* ws_o, float* ws_ml, hipStream_t stream, bool fp8) {
  const float c = scale * 1.4426950408889634f;
  // the kernel keeps a chunk's page ids in the 64 lanes of one register
  if (chunk_steps <= 0 || (chunk_steps + g.P / mla::STEP_T - 1) / (g.P / mla::STEP_T) + 1 > 64) return hipErrorInvalidValue;
  if (fp8)
    hipLaunchKernelGGL(decode_mla_kernel<true>, dim3((unsigned)n_items), dim3(256), 0, stream, pool_base, g.page_bytes,
                       g.P / mla::STEP_T, (const bf16_t*)q, (bf16_t*)out, d_ctx_lens, d_block_tables, bt_stride,
                       (const int2*)d_items, H, c, chunk_steps, max_chunks, ws_o, ws_ml);
  else
    hipLaunchKernelGGL(decode_mla_kernel<false>, dim3((unsigned)n_items), dim3(256), 0, stream, pool_base, g.page_bytes,
                       g.P / mla::STEP_T, (const bf16_t*)q, (bf16_t*)out, d_ctx_lens, d_block_tables, bt_stride,
                       (const int2*)d_items, H, c, chunk_steps, max_chunks, ws_o, ws_ml);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess || max_chunks <= 1) return e;
  hipLaunchKernelGGL(decode_mla_combine_kernel, dim3(H, B), dim3(128), 0, stream, (bf16_t*)out, d_ctx_lens, H,
                     chunk_steps, max_chunks, ws_o, ws_ml);
  return hipGetLastError();
}

}  // namespace spd
