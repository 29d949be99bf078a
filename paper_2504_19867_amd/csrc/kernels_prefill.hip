// Prefill step: causal attention over each request's prompt (varlen-packed batch).
//
// Paper, Background "LLM Processing Phases": the prefill phase processes the whole input
// context.  For request r, query head h (KV head g = h / (H / Hkv)), row i:
//     out[i,h,:] = sum_{j<=i} softmax_j(scale * q[i,h,:] . k[j,g,:]) * v[j,g,:]
// (The page write of K, V that belongs to the same step is kv_write_kernel.)
// With a cached prefix of p tokens (chunked prefill) the request's K, V hold p + len rows and
// query row i sits at position p + i: the sum runs over j <= p + i.
//
// A dense contraction, so it runs on the matrix cores.  One workgroup = 8 waves = one CU's worth
// of work; every wave owns 32 query rows of one head.  The 8 waves are HB query heads of ONE
// KV head (grouped-query attention: they all need the same K, V) times 8 / HB row sub-tiles,
// so each K/V tile fetched into LDS feeds 256 (row, head) pairs.
//
// Everything is kept TRANSPOSED so that a query is a lane (column), not a row:
//     S^T[key, query] = K_tile[64 x d] . Q^T[d x 32]          v_mfma_f32_32x32x16_bf16
//     O^T[dim, query] += V_tile^T[dv x 64] . P^T[64 x 32]
// With queries along lanes the softmax statistics (running max, running sum, rescale factor)
// are per-lane scalars, the row maximum needs one cross-lane exchange per tile (lane ^ 32), and
// the S^T accumulators are already in the B-operand order of the second product: P never
// leaves registers.  Q^T fragments live in registers for the whole workgroup.
//
// The kernel is persistent: one workgroup per compute unit of the prefill share walks a chain of
// work items (one item = one tile of query rows of one request for one group of heads), and the
// K/V tile loads run ahead of the compute across item boundaries, so that an item's first tiles,
// which a fresh workgroup would have to wait for, arrive while the item before is still computing.
//
// K and V tiles of 64 keys stream from global memory straight into a ring of LDS stages with
// global_load_lds_dwordx4 (no register staging, no LDS stores), ahead of the compute; one
// s_barrier per pair of tiles where the ring has four stages (one per tile with three).  K rows
// are read back with 16-byte reads in A-operand order; V stays in its natural [key][dim] order
// and the transposition that the second product needs is done by the LDS transpose read
// ds_read_b64_tr_b16.  Both tiles are XOR-swizzled at 16-byte granularity against bank conflicts.
//
// The softmax keeps a reference per query that is moved to the running maximum only when a row sum
// shows that it must be (an item's first tile, or scores that have outgrown it by 2^60).
#include "internal.h"
#include <type_traits>

namespace spd {

typedef unsigned short bf16_t;
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef short s16x4 __attribute__((ext_vector_type(4)));

constexpr int BN = 64;        // keys per LDS tile
constexpr int WAVES = 8;      // waves per workgroup

__device__ inline uint32_t cvt_pk_bf16(float a, float b) {
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(f32x2{a, b}, bf16x2));
}

// 16 bytes per lane from global memory to LDS: lane i's data lands at lds_byte_addr + 16 * i.
// The compiler does not see this write; completion is tracked by hand with vmcnt (below).
__device__ inline void dma16(const void* gptr, uint32_t lds_byte_addr) {
  asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, off" ::"s"(lds_byte_addr), "v"(gptr) : "memory");
}
// The same with the address split in a wave-uniform base and a 32-bit per-lane offset.
__device__ inline void dma16s(const void* sbase, uint32_t voff, uint32_t lds_byte_addr) {
  asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(lds_byte_addr), "v"(voff), "s"(sbase) : "memory");
}
// s_waitcnt vmcnt(N) only (expcnt and lgkmcnt fields left at their maxima)
#define SPD_WAIT_VMCNT(N) __builtin_amdgcn_s_waitcnt(((N) & 15) | (7 << 4) | (15 << 8) | (((N) >> 4) << 14))

// XOR swizzles (in units of 16-byte chunks) of a K row and a V row
template <int DQK> __device__ inline int k_swz(int row) { return DQK == 128 ? (row & 15) : ((row >> 1) & 7); }
template <int DV> __device__ inline int v_swz(int row) { return DV == 128 ? 4 * (row & 3) : 4 * ((row >> 1) & 1); }

template <int DQK, int DV, int HB>
__global__ __launch_bounds__(512, 2) void prefill_kernel(const bf16_t* __restrict__ q, const bf16_t* __restrict__ k,
                                                         const bf16_t* __restrict__ v, bf16_t* __restrict__ out,
                                                         const PrefillWork* __restrict__ work,
                                                         const int32_t* __restrict__ chain, int H, int Hkv,
                                                         float c /* scale * log2(e) */) {
  constexpr int QS = WAVES / HB;                // 32-row sub-tiles per workgroup
  constexpr int CHK = DQK / 8, CHV = DV / 8;    // 16-byte chunks per K / V row
  constexpr int K_BYTES = BN * DQK * 2, V_BYTES = BN * DV * 2, STAGE_BYTES = K_BYTES + V_BYTES;
  constexpr int NSTAGE = DQK > 128 ? 3 : 4;     // LDS ring
  constexpr int PD = NSTAGE - 1;                // tiles in flight ahead of the compute
  constexpr int NI = CHK + CHV;                 // 1 KiB load instructions per tile
  static_assert(NI % WAVES == 0, "tile loads must divide evenly over the waves");
  constexpr int LPW = NI / WAVES;               // load instructions per wave per tile
  constexpr int KS = DQK / 16, VB = DV / 32;
  constexpr int NS = 2 * KS;                    // MFMAs of S^T
  constexpr int RING = DQK > 128 ? 4 : 8;       // K operands in flight (fewer where registers are short)
  static_assert(NS >= RING, "operand ring longer than the first product");
  constexpr int OPITCH = 32 * 2 + 16;           // bytes per staged output row piece (32 dims, padded)
  constexpr int EPI_BYTES = WAVES * 32 * OPITCH;  // output staging, apart from the K/V stages
  __shared__ __attribute__((aligned(1024))) char smem[NSTAGE * STAGE_BYTES + EPI_BYTES];

  const int G = H / Hkv;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int n32 = lane & 31, hh = lane >> 5;
  const uint32_t k_pitch = (uint32_t)Hkv * DQK * 2, v_pitch = (uint32_t)Hkv * DV * 2;
  const uint32_t smem_base = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char*)smem;
  // this workgroup's chain of work items
  int it = __builtin_amdgcn_readfirstlane(chain[blockIdx.x]);
  const int it_end = __builtin_amdgcn_readfirstlane(chain[blockIdx.x + 1]);
  if (it >= it_end) return;

  // ---- tile loads.  Load instruction ii = wave + 8 j (j < LPW) fills the 64 consecutive 16-byte
  // slots [64 ii, 64 ii + 64) of the stage: K slots first (row = slot / CHK), then V slots.
  // Slot s of a row holds the row's chunk s ^ swz(row).
  // The per-lane part of the address does not depend on the tile (except past the prompt's end).
  auto slot_of = [&](int j, int& row, int& coff, uint32_t& pitch) {
    const int ii = wave + WAVES * j;
    if (ii < CHK) {
      const int slot = ii * 64 + lane, sl = slot % CHK;
      row = slot / CHK;
      coff = (sl ^ k_swz<DQK>(row)) * 16;
      pitch = k_pitch;
    } else {
      const int slot = (ii - CHK) * 64 + lane, sl = slot % CHV;
      row = slot / CHV;
      coff = (sl ^ v_swz<DV>(row)) * 16;
      pitch = v_pitch;
    }
  };
  uint32_t ld_voff[LPW];
#pragma unroll
  for (int j = 0; j < LPW; ++j) {
    int row, coff;
    uint32_t pitch;
    slot_of(j, row, coff, pitch);
    ld_voff[j] = (uint32_t)row * pitch + (uint32_t)coff;
  }
  // ---- the chain's work items, 64 at a time, one per lane: item i sits in lane i - dsc_base.  An item is then had
  // with six lane reads, where a load from memory at every item boundary (one by the producer, one by the
  // compute side, each waited for at once, and every such wait also drains the tile loads in flight) cost the
  // chain about as much as three tiles.  The producer is at most a few items ahead of the compute side, which
  // moves the window when it is half way through it.  (Not with 192 dims: the touch below needs the full wait that
  // only the paired tiles have.)
  constexpr bool ITEM_LANES = DQK <= 128;
  int dsc_base = it;
  int d_row0 = 0, d_len = 0, d_qtile = 0, d_head0 = 0, d_kvrow0 = 0, d_qoff = 0;
  auto load_items = [&](int base) __attribute__((always_inline)) {
    const PrefillWork pw = work[min(base + lane, it_end - 1)];
    d_row0 = pw.row0; d_len = pw.len; d_qtile = pw.q_tile; d_head0 = pw.head0; d_kvrow0 = pw.kv_row0; d_qoff = pw.q_off;
    dsc_base = base;
  };
  auto item_of = [&](int i) __attribute__((always_inline)) -> PrefillWork {
    if constexpr (!ITEM_LANES) return work[i];
    const int l = i - dsc_base;
    return PrefillWork{__builtin_amdgcn_readlane(d_row0, l), __builtin_amdgcn_readlane(d_len, l),
                       __builtin_amdgcn_readlane(d_qtile, l), __builtin_amdgcn_readlane(d_head0, l),
                       __builtin_amdgcn_readlane(d_kvrow0, l), __builtin_amdgcn_readlane(d_qoff, l)};
  };
  if constexpr (ITEM_LANES) load_items(it);
  // ---- producer: the tile loads run ahead of the compute (a pair of tiles, or PD tiles where the
  // ring has three stages), across the items of the chain.
  // pt counts the tiles issued so far (tile number pt goes to stage pt % NSTAGE).
  int p_it = it, p_kt = 0, p_n = 0, p_kv_len = 0, pt = 0;
  const char *p_kb = nullptr, *p_vb = nullptr;
  auto producer_item = [&]() {                  // producer state for item p_it
    const PrefillWork pw = item_of(p_it);
    const int pg = pw.head0 / G;
    p_kv_len = pw.q_off + pw.len;
    const int kv_end = min(p_kv_len, pw.q_off + pw.q_tile * (32 * QS) + 32 * QS);
    p_n = (kv_end + BN - 1) / BN;
    p_kb = (const char*)(k + ((size_t)pw.kv_row0 * Hkv + pg) * DQK);
    p_vb = (const char*)(v + ((size_t)pw.kv_row0 * Hkv + pg) * DV);
    p_kt = 0;
  };
  producer_item();
  auto produce_one = [&]() {
    if (p_it >= it_end) return;
    const int kv0 = p_kt * BN;
    const uint32_t stage = smem_base + (uint32_t)(pt % NSTAGE) * STAGE_BYTES;
    const char* kb = p_kb + (size_t)kv0 * k_pitch;
    const char* vb = p_vb + (size_t)kv0 * v_pitch;
    if (kv0 + BN <= p_kv_len) {
#pragma unroll
      for (int j = 0; j < LPW; ++j) {
        const int ii = wave + WAVES * j;
        dma16s(ii < CHK ? kb : vb, ld_voff[j], stage + (uint32_t)ii * 1024);
      }
    } else {                                    // rows past the prompt re-read its last row
      const int last = p_kv_len - 1 - kv0;
#pragma unroll
      for (int j = 0; j < LPW; ++j) {
        const int ii = wave + WAVES * j;
        int row, coff;
        uint32_t pitch;
        slot_of(j, row, coff, pitch);
        dma16s(ii < CHK ? kb : vb, (uint32_t)min(row, last) * pitch + (uint32_t)coff, stage + (uint32_t)ii * 1024);
      }
    }
    ++pt;
    if (++p_kt == p_n) {
      ++p_it;
      if (p_it < it_end) producer_item();
    }
  };

  // ---- LDS operand addresses (byte offsets inside a stage)
  // K operand (S^T block b, k-step ks): row 32 b + n32, chunk 2 ks + hh
  // (192 dims: the swizzle touches the low three bits of the chunk number only, so k-steps four apart differ by
  // 128 bytes and share a lane address; that frees eight registers)
  constexpr int KOFFS = DQK == 192 ? 4 : KS;
  int k_off[KOFFS];
#pragma unroll
  for (int ks = 0; ks < KOFFS; ++ks) k_off[ks] = n32 * (CHK * 16) + (((2 * ks + hh) ^ k_swz<DQK>(n32)) * 16);
  auto k_addr = [&](int ks) -> int { return k_off[ks % KOFFS] + (ks / KOFFS) * 128; };
  // V operand (16-key step kk, value block blk): two transpose reads.  In each group of 16 lanes
  // lane r supplies row (key) 4 hh + r / 4 and dims 4 (r % 4) .. + 3 of the group's 16 dims; the
  // hardware hands lane i of the group dim i of those 4 keys.
  const int r16 = lane & 15;
  const int v_row = 4 * hh + (r16 >> 2);                         // plus 16 kk + 8 half
  int v_off[VB];
#pragma unroll
  for (int blk = 0; blk < VB; ++blk) {
    const int dim = 32 * blk + 16 * ((lane >> 4) & 1) + 4 * (r16 & 3);
    v_off[blk] = K_BYTES + v_row * (CHV * 16) + (((dim >> 3) ^ v_swz<DV>(v_row)) * 16) + (dim & 7) * 2;
  }

  // The tile loop is unrolled over the ring's stages so that the stage offset is part of each LDS
  // read's 16-bit immediate; stages 2 and 3 lie beyond its reach and get a second set of lane addresses.
  constexpr bool UNROLL = NSTAGE == 4 && 2 * STAGE_BYTES <= 65536;
  constexpr bool PAIRS = UNROLL;                // a ring of four holds the pair in use and the pair in flight
  int k_off2[KS], v_off2[VB];
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) {
    k_off2[ks] = k_addr(ks) + 2 * STAGE_BYTES;
    asm volatile("" : "+v"(k_off2[ks]));        // a value of its own, not "k_off + constant" to be recomputed
  }
#pragma unroll
  for (int blk = 0; blk < VB; ++blk) {
    v_off2[blk] = v_off[blk] + 2 * STAGE_BYTES;
    asm volatile("" : "+v"(v_off2[blk]));
  }
  const uint32_t ones2 = 0x3f803f80u;           // (1.0, 1.0) in bf16

  int ct = 0;                                   // tiles consumed so far (tile number ct sits in stage ct % NSTAGE)
#pragma unroll
  for (int t = 0; t < (PAIRS ? 2 : PD); ++t) produce_one();

  // ---- state of the item being computed
  PrefillWork w;
  int h = 0, wave_q0 = 0, qi = 0, pos0 = 0, pos = 0, n_kv_tiles = 0, kt = 0;
  bool wave_active = false;
  bf16x8 qf[KS];                                // Q^T fragments (B operand: column = query, 8 consecutive dims per lane and k-step)
  f32x16 O[VB];
  float m = 0.f, l = 0.f;
  // The next item's query rows are touched ahead of time, one 128-byte line per lane, so that its fragment loads,
  // which nothing can overlap (every wave of the workgroup stands at the same item boundary), find them in the L2
  // instead of in HBM.  The touch goes out behind the first full wait of the item (a pair's barrier), so that it
  // has two tiles' time before the next one; the loaded word is never used, its register passes every full wait.
  uint32_t q_touch = 0;
  bool touch_next = false;
  auto touch_next_q = [&]() __attribute__((always_inline)) {
    const PrefillWork w2 = item_of(it + 1);
    constexpr int LINES = DQK / 64;               // 128-byte lines per query row
    int r2 = w2.q_tile * (32 * QS) + 32 * (wave / HB) + lane / LINES;
    r2 = r2 < w2.len ? r2 : w2.len - 1;
    const char* p2 = (const char*)(q + ((size_t)(w2.row0 + r2) * H + w2.head0 + wave % HB) * DQK) + (lane % LINES) * 128;
    asm volatile("global_load_dword %0, %1, off" : "=v"(q_touch) : "v"(p2) : "memory");
    touch_next = false;
  };
  auto item_begin = [&]() {
    if (ITEM_LANES && it - dsc_base >= 32) load_items(it);      // (the producer is past `it` and less than 32 items ahead)
    w = item_of(it);
    h = w.head0 + wave % HB;
    const int q_start = w.q_tile * (32 * QS);
    wave_q0 = q_start + 32 * (wave / HB);
    wave_active = wave_q0 < w.len;              // waves past the prompt's end only help loading
    qi = wave_q0 + n32;                         // this lane's query (row inside the request)
    const int qi_c = qi < w.len ? qi : w.len - 1;
    const int kv_len = w.q_off + w.len;         // cached prefix + this step's rows
    pos0 = w.q_off + wave_q0;                   // position of this wave's first query in the request
    pos = w.q_off + qi;                         // ... of this lane's query
    const bf16_t* qp = q + ((size_t)(w.row0 + qi_c) * H + h) * DQK + 8 * hh;
#pragma unroll
    for (int s = 0; s < KS; ++s) qf[s] = __builtin_bit_cast(bf16x8, *(const uint4*)(qp + 16 * s));
    const int kv_end = min(kv_len, w.q_off + q_start + 32 * QS);
    n_kv_tiles = (kv_end + BN - 1) / BN;
    kt = 0;
#pragma unroll
    for (int i = 0; i < VB; ++i)
#pragma unroll
      for (int e = 0; e < 16; ++e) O[i][e] = 0.f;
    m = -INFINITY;
    l = 0.f;
    // Draw the compiler's wait for the Q loads to this point.  Left to itself it waits at their first
    // use, inside the tile, with a count that knows nothing of the tile loads issued by hand.
#pragma unroll
    for (int s = 0; s < KS; ++s) asm volatile("" ::"v"(__builtin_bit_cast(uint4, qf[s]).x));
    touch_next = ITEM_LANES && it + 1 < it_end;
  };
  auto item_end = [&]() {
    l += __shfl_xor(l, 32);
    // Output: a lane holds one query row in 8-byte bits, 8 KiB apart from its neighbour's.  Each wave
    // turns its block round, 32 dims at a time, in its own piece of LDS and writes 64-byte row pieces.
    if (wave_active) {
      char* ost = smem + NSTAGE * STAGE_BYTES + wave * (32 * OPITCH);
      const float inv = 1.f / l;
      bf16_t* obase = out + ((size_t)(w.row0 + wave_q0) * H + h) * DV;
      const int rows = min(32, w.len - wave_q0);
#pragma unroll
      for (int blk = 0; blk < VB; ++blk) {
#pragma unroll
        for (int i4 = 0; i4 < 4; ++i4) {
          uint2 pk;
          pk.x = cvt_pk_bf16(O[blk][4 * i4] * inv, O[blk][4 * i4 + 1] * inv);
          pk.y = cvt_pk_bf16(O[blk][4 * i4 + 2] * inv, O[blk][4 * i4 + 3] * inv);
          *(uint2*)(ost + n32 * OPITCH + (8 * i4 + 4 * hh) * 2) = pk;
        }
#pragma unroll
        for (int itr = 0; itr < 2; ++itr) {       // 32 rows x 4 pieces of 16 bytes
          const int i = lane + 64 * itr;
          const int r = i >> 2, cc = i & 3;
          if (r < rows) *(uint4*)(obase + (size_t)r * H * DV + 32 * blk + cc * 8) = *(const uint4*)(ost + r * OPITCH + cc * 16);
        }
      }
    }
  };

  auto tile = [&](auto stc) {
    const int ST = stc;                         // ring stage of tile kt: a constant when the loop is unrolled
    const int kv0 = kt * BN;
    if constexpr (PAIRS) {
      // Tiles go in pairs: one wait and one barrier for two tiles, after which the waves run free
      // for two tiles' worth of work (the two waves of a SIMD drift apart, and one's matrix work
      // falls beside the other's softmax).  At the barrier the pair has landed and everyone is done
      // with the pair before, whose two stages are refilled, one now and one a tile later.
      if ((ST & 1) == 0) {
        SPD_WAIT_VMCNT(0);
        asm volatile("" : "+v"(q_touch));
        asm volatile("s_barrier" ::: "memory");
        produce_one();
        if (touch_next) touch_next_q();
      } else {
        produce_one();                          // the pair's second tile a tile later: eight loads at once queue up
      }
    } else {
      // this wave's loads of the tile are done when at most (tiles issued after it) * LPW remain
      const int later = pt - ct - 1;
      if (later >= 2) SPD_WAIT_VMCNT(2 * LPW);
      else if (later == 1) SPD_WAIT_VMCNT(LPW);
      else SPD_WAIT_VMCNT(0);
      // all waves: the tile has landed, and everyone is done with the one before, whose stage is refilled next
      asm volatile("s_barrier" ::: "memory");
      produce_one();
    }
    ++ct;
    if (!wave_active || kv0 > pos0 + 31) return;               // every key of the tile is in this wave's future

    const char* sbase = UNROLL ? smem + (ST & 1) * STAGE_BYTES : smem + ST * STAGE_BYTES;
    auto read_k = [&](int i) -> uint4 {
      return *(const uint4*)(sbase + (UNROLL && ST >= 2 ? k_off2[i / 2] : k_addr(i / 2)) + (i % 2) * (32 * CHK * 16));
    };
    auto read_v = [&](int i, int half) -> s16x4 {
      const int kk = i / VB, blk = i % VB;
      return __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(
          sbase + (UNROLL && ST >= 2 ? v_off2[blk] : v_off[blk]) + (16 * kk + 8 * half) * (CHV * 16)));
    };

    // ---- S^T = K . Q^T.  Operand i: block b = i % 2 (32 keys), k-step ks = i / 2; LDS reads run
    // RING operands ahead of the MFMAs that consume them.
    __builtin_amdgcn_s_setprio(0);
    f32x16 S[2];
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
      for (int e = 0; e < 16; ++e) S[b][e] = 0.f;
    uint4 ring[RING];
#pragma unroll
    for (int i = 0; i < RING; ++i) ring[i] = read_k(i);
    __builtin_amdgcn_sched_barrier(0);          // keep the issue order below: the scheduler would
#pragma unroll                                  // otherwise sink every read next to its use
    for (int i = 0; i < NS; ++i) {
      S[i % 2] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, ring[i % RING]), qf[i / 2], S[i % 2], 0, 0, 0);
      if (i + RING < NS) ring[i % RING] = read_k(i + RING);
      __builtin_amdgcn_sched_barrier(0);
    }
    // first V operands: in flight while the vector units do the softmax.  Operand j = 16-key step j / VB, value
    // block j % VB; a queue of VQ operands, read VAH ahead of the MFMA that takes them (a whole step ahead, two
    // steps' worth of registers; with 192 dims two operands ahead in a queue of three: registers are short there)
    constexpr int VAH = DQK > 128 ? 2 : VB, VQ = DQK > 128 ? VAH + 1 : 2 * VB;
    s16x4 vq[VQ][2];
#pragma unroll
    for (int j = 0; j < VAH; ++j) {
      vq[j][0] = read_v(j, 0);
      vq[j][1] = read_v(j, 1);
    }

    // lane holds, for the query at position pos, keys kv0 + 32b + 8*(i/4) + 4*hh + i%4
    if (kv0 + BN - 1 > pos0) {               // tile crosses this wave's diagonal (or the prompt's end)
#pragma unroll
      for (int b = 0; b < 2; ++b)
#pragma unroll
        for (int i = 0; i < 16; ++i)
          if (kv0 + 32 * b + 8 * (i >> 2) + 4 * hh + (i & 3) > pos) S[b][i] = -INFINITY;
    }
    // p = exp2(S c - m c) against a reference m per query that need not be the running maximum: any
    // reference gives the same softmax as long as nothing overflows, and bf16 and fp32 keep their
    // relative precision over the whole exponent range.  So the tile's maximum is not computed at
    // all unless the row sum says that the reference is out of range (an item's first tile, where
    // m = -inf makes every p infinite or NaN, or a tile whose scores exceed the reference by 2^60):
    // then the reference moves to the true maximum, the accumulators are rescaled, and p is redone.
    // A wave's priority rises as it gets on with its tile: first product 0, softmax 3, second product 1.  The wave
    // that is further along is served first, so the two waves of a SIMD fall out of step instead of contending
    // phase by phase, and the softmax's vector instructions go out between the other wave's MFMAs (each of which
    // takes only a few issue cycles of the SIMD) instead of queueing behind them.
    __builtin_amdgcn_s_setprio(3);
    uint32_t pb[2][8];
    auto softmax_p = [&](float mc) -> float {
      float ls[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int b = 0; b < 2; ++b)
#pragma unroll
        for (int i = 0; i < 16; i += 2) {
          const float p0 = __builtin_amdgcn_exp2f(S[b][i] * c - mc);
          const float p1 = __builtin_amdgcn_exp2f(S[b][i + 1] * c - mc);
          pb[b][i >> 1] = cvt_pk_bf16(p0, p1);
          // the row sum runs over the rounded values, the ones the second product multiplies: two per
          // instruction (the compiler places the wait states that a dot product's result needs)
          ls[(i >> 1) & 3] = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, pb[b][i >> 1]),
                                                             __builtin_bit_cast(bf16x2, ones2), ls[(i >> 1) & 3], false);
        }
      return (ls[0] + ls[1]) + (ls[2] + ls[3]);
    };
    // (an item's first tile has no reference yet: the pass against it would be thrown away, so it is not made)
    float psum = INFINITY;
    if (kt != 0) psum = softmax_p(m * c);
    if (__builtin_amdgcn_ballot_w64(!(psum < 0x1p60f)) != 0) {
      float mx = S[0][0];
#pragma unroll
      for (int i = 1; i < 16; ++i) mx = fmaxf(mx, S[0][i]);
#pragma unroll
      for (int i = 0; i < 16; ++i) mx = fmaxf(mx, S[1][i]);
      {
        // the other half of the wave holds the other 32 keys of the same query: exchange on the
        // vector ALU (swap of the upper half of one register with the lower half of another;
        // written as machine code: the compiler's builtin for it loses the second result)
        float mx2 = mx;
        asm volatile("s_nop 1\n\tv_permlane32_swap_b32 %0, %1\n\ts_nop 1" : "+v"(mx), "+v"(mx2));
        mx = fmaxf(mx, mx2);
      }
      const float m_new = fmaxf(m, mx);
      const float alpha = __builtin_amdgcn_exp2f((m - m_new) * c);
      l *= alpha;
#pragma unroll
      for (int blk = 0; blk < VB; ++blk)
#pragma unroll
        for (int e = 0; e < 16; ++e) O[blk][e] *= alpha;
      m = m_new;
      psum = softmax_p(m * c);
    }
    l += psum;
    __builtin_amdgcn_s_setprio(1);

    // ---- O^T += V^T . P^T : 16-key step kk multiplies with S^T block kk/2, registers 8*(kk%2) .. +7;
    // operand j + VAH is read while operand j multiplies
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int kk = 0; kk < BN / 16; ++kk) {
      const uint4 praw = uint4{pb[kk >> 1][4 * (kk & 1)], pb[kk >> 1][4 * (kk & 1) + 1], pb[kk >> 1][4 * (kk & 1) + 2],
                               pb[kk >> 1][4 * (kk & 1) + 3]};
#pragma unroll
      for (int blk = 0; blk < VB; ++blk) {
        const int j = kk * VB + blk;
        const uint2 lo = __builtin_bit_cast(uint2, vq[j % VQ][0]), hi = __builtin_bit_cast(uint2, vq[j % VQ][1]);
        const uint4 a = uint4{lo.x, lo.y, hi.x, hi.y};
        O[blk] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, praw),
                                                         O[blk], 0, 0, 0);
        if (j + VAH < (BN / 16) * VB) {
          vq[(j + VAH) % VQ][0] = read_v(j + VAH, 0);
          vq[(j + VAH) % VQ][1] = read_v(j + VAH, 1);
        }
        __builtin_amdgcn_sched_barrier(0);
      }
    }
  };


  // one tile of the chain; false when the chain is finished
  auto step = [&](auto stc) -> bool {
    tile(stc);
    if (++kt == n_kv_tiles) {
      item_end();
      if (++it >= it_end) return false;
      item_begin();
    }
    return true;
  };
  item_begin();
  if constexpr (UNROLL) {
    // the ring's stages in turn, each with its LDS offsets as immediates; items follow one another
    // without a break in the ring
    for (;;) {
      if (!step(std::integral_constant<int, 0>{})) break;
      if (!step(std::integral_constant<int, 1>{})) break;
      if (!step(std::integral_constant<int, 2>{})) break;
      if (!step(std::integral_constant<int, 3>{})) break;
    }
  } else {
    while (step(ct % NSTAGE)) {
    }
  }
}

bool prefill_shape_supported(int dqk, int dv) {
  return (dqk == 64 && dv == 64) || (dqk == 128 && dv == 128) || (dqk == 192 && dv == 128);
}

// Query heads of one KV head that share a workgroup: the largest of 8, 4, 2, 1 dividing the group size.
int prefill_heads_per_block(int group) {
  for (int hb = WAVES; hb > 1; hb >>= 1)
    if (group % hb == 0) return hb;
  return 1;
}
int prefill_block_m(int group) { return 32 * (WAVES / prefill_heads_per_block(group)); }

template <int DQK, int DV>
static void launch_hb(int hb, dim3 grid, hipStream_t stream, const bf16_t* q, const bf16_t* k, const bf16_t* v,
                      bf16_t* out, const PrefillWork* work, const int32_t* chain, int H, int Hkv, float c) {
  const dim3 block(64 * WAVES);
  if (hb == 8) hipLaunchKernelGGL((prefill_kernel<DQK, DV, 8>), grid, block, 0, stream, q, k, v, out, work, chain, H, Hkv, c);
  else if (hb == 4) hipLaunchKernelGGL((prefill_kernel<DQK, DV, 4>), grid, block, 0, stream, q, k, v, out, work, chain, H, Hkv, c);
  else if (hb == 2) hipLaunchKernelGGL((prefill_kernel<DQK, DV, 2>), grid, block, 0, stream, q, k, v, out, work, chain, H, Hkv, c);
  else hipLaunchKernelGGL((prefill_kernel<DQK, DV, 1>), grid, block, 0, stream, q, k, v, out, work, chain, H, Hkv, c);
}

hipError_t launch_prefill(const void* q, const void* k, const void* v, void* out, const PrefillWork* d_work,
                          const int32_t* d_chain, int n_blocks, int H, int Hkv, int dqk, int dv, float scale, hipStream_t stream) {
  const float c = scale * 1.4426950408889634f;
  const int hb = prefill_heads_per_block(H / Hkv);
  const dim3 grid((unsigned)n_blocks);
  const bf16_t *qq = (const bf16_t*)q, *kk = (const bf16_t*)k, *vv = (const bf16_t*)v;
  if (dqk == 64 && dv == 64) launch_hb<64, 64>(hb, grid, stream, qq, kk, vv, (bf16_t*)out, d_work, d_chain, H, Hkv, c);
  else if (dqk == 128 && dv == 128) launch_hb<128, 128>(hb, grid, stream, qq, kk, vv, (bf16_t*)out, d_work, d_chain, H, Hkv, c);
  else if (dqk == 192 && dv == 128) launch_hb<192, 128>(hb, grid, stream, qq, kk, vv, (bf16_t*)out, d_work, d_chain, H, Hkv, c);
  else return hipErrorInvalidValue;
  return hipGetLastError();
}

}  // namespace spd
