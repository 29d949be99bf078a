// Prefill step: causal attention over each request's prompt (varlen-packed batch).
//
// Paper, Background "LLM Processing Phases": the prefill phase processes the whole input
// context.  For request r, query head h (KV head g = h / (H / Hkv)), row i:
//     out[i,h,:] = sum_{j<=i} softmax_j(scale * q[i,h,:] . k[j,g,:]) * v[j,g,:]
// (The page write of K, V that belongs to the same step is kv_write_kernel.)
//
// A dense contraction, so it runs on the matrix cores.  One workgroup = 4 waves = one tile of
// 128 query rows of one head; each wave owns 32 rows.  Everything is kept TRANSPOSED so that a
// query is a lane (column), not a row:
//     S^T[key, query] = K_tile[64 x d] . Q^T[d x 32]     v_mfma_f32_32x32x16_bf16
//     O^T[dim, query] += V_tile^T[dv x 64] . P^T[64 x 32]
// With queries along lanes the softmax statistics (running max, running sum, rescale factor)
// are per-lane scalars, the row maximum needs one cross-lane exchange per tile (lane ^ 32), and
// the S^T accumulators are already in the B-operand order of the second product - P never
// leaves registers.  Q^T fragments live in registers for the whole workgroup; K and V tiles
// of 64 keys are staged through LDS (K row-padded, V transposed in registers on the way in and
// stored with an XOR swizzle) so that every operand read is a conflict-free 16-byte read.
#include "internal.h"

namespace spd {

typedef unsigned short bf16_t;
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));

constexpr int BM = 128;   // query rows per workgroup
constexpr int BN = 64;    // keys per LDS tile

__device__ inline uint32_t cvt_pk_bf16(float a, float b) {
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(f32x2{a, b}, bf16x2));
}

// Position of key offset o (0..15) inside its 16-key group of the transposed V tile: the order
// in which the S^T accumulator registers of one lane enumerate keys (bits 2 and 3 swapped).
__device__ inline int vt_unit_swizzle(int d) { return (d & 7) ^ ((d >> 3) & 7); }

template <int DQK, int DV>
__global__ __launch_bounds__(256, 2) void prefill_kernel(const bf16_t* __restrict__ q, const bf16_t* __restrict__ k,
                                                         const bf16_t* __restrict__ v, bf16_t* __restrict__ out,
                                                         const PrefillWork* __restrict__ work, int H, int Hkv,
                                                         float c /* scale * log2(e) */) {
  constexpr int KROW = DQK + 8;                 // padded K row (elements): consecutive rows shift by 4 banks
  constexpr int KCH = DQK / 8;                  // 16-byte chunks per K row
  constexpr int K_LD = (BN * KCH) / 256;        // 16-byte global loads per thread for the K tile
  constexpr int VCH = DV / 8;
  constexpr int V_ITEMS = (BN / 4) * VCH;       // (key quad, 8-dim chunk) items of the V tile
  constexpr int V_LD = (V_ITEMS + 255) / 256;
  static_assert((BN * KCH) % 256 == 0, "K tile does not divide over 256 threads");
  __shared__ __attribute__((aligned(16))) bf16_t Ks[BN * KROW];
  __shared__ __attribute__((aligned(16))) bf16_t Vt[DV * BN];

  const PrefillWork w = work[blockIdx.x / H];
  const int h = blockIdx.x % H;
  const int g = h / (H / Hkv);
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int n32 = lane & 31, hh = lane >> 5;
  const int q_start = w.q_tile * BM;
  const int wave_q0 = q_start + 32 * wave;
  const int qi = wave_q0 + n32;                                  // this lane's query (row inside the request)
  const int qi_c = qi < w.len ? qi : w.len - 1;

  // Q^T fragments (B operand: column = query, 8 consecutive dims per lane and k-step)
  bf16x8 qf[DQK / 16];
  {
    const bf16_t* qp = q + ((size_t)(w.row0 + qi_c) * H + h) * DQK + 8 * hh;
#pragma unroll
    for (int s = 0; s < DQK / 16; ++s) qf[s] = __builtin_bit_cast(bf16x8, *(const uint4*)(qp + 16 * s));
  }

  f32x16 O[DV / 32];
#pragma unroll
  for (int i = 0; i < DV / 32; ++i)
#pragma unroll
    for (int e = 0; e < 16; ++e) O[i][e] = 0.f;
  float m = -INFINITY, l = 0.f;

  const int kv_end = min(w.len, q_start + BM);
  const int n_kv_tiles = (kv_end + BN - 1) / BN;
  const bf16_t* kbase = k + ((size_t)w.row0 * Hkv + g) * DQK;
  const bf16_t* vbase = v + ((size_t)w.row0 * Hkv + g) * DV;

  uint4 kreg[K_LD], vreg[V_LD][4];
  auto load_tile = [&](int kt) {
    const int kv0 = kt * BN;
#pragma unroll
    for (int p = 0; p < K_LD; ++p) {
      const int idx = p * 256 + tid, row = idx / KCH, ch = idx % KCH;
      const int key = min(kv0 + row, w.len - 1);
      kreg[p] = *(const uint4*)(kbase + (size_t)key * Hkv * DQK + 8 * ch);
    }
#pragma unroll
    for (int p = 0; p < V_LD; ++p) {
      const int idx = p * 256 + tid, kq = idx / VCH, dc = idx % VCH;
      if (V_ITEMS % 256 != 0 && idx >= V_ITEMS) break;
#pragma unroll
      for (int t = 0; t < 4; ++t) {
        const int key = min(kv0 + 4 * kq + t, w.len - 1);
        vreg[p][t] = *(const uint4*)(vbase + (size_t)key * Hkv * DV + 8 * dc);
      }
    }
  };
  auto store_tile = [&]() {
#pragma unroll
    for (int p = 0; p < K_LD; ++p) {
      const int idx = p * 256 + tid, row = idx / KCH, ch = idx % KCH;
      *(uint4*)(Ks + row * KROW + 8 * ch) = kreg[p];
    }
#pragma unroll
    for (int p = 0; p < V_LD; ++p) {
      const int idx = p * 256 + tid, kq = idx / VCH, dc = idx % VCH;
      if (V_ITEMS % 256 != 0 && idx >= V_ITEMS) break;
      // keys 4kq..4kq+3 sit at 4 consecutive positions of row d: 16*(kq/4) + 8*(kq&1) + 4*((kq>>1)&1)
      const int pos4 = 16 * (kq >> 2) + 8 * (kq & 1) + 4 * ((kq >> 1) & 1);
      const uint32_t* r0 = (const uint32_t*)&vreg[p][0];
      const uint32_t* r1 = (const uint32_t*)&vreg[p][1];
      const uint32_t* r2 = (const uint32_t*)&vreg[p][2];
      const uint32_t* r3 = (const uint32_t*)&vreg[p][3];
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const int d = 8 * dc + e;
        uint2 o;
        if (e & 1) {
          o.x = (r0[e >> 1] >> 16) | (r1[e >> 1] & 0xffff0000u);
          o.y = (r2[e >> 1] >> 16) | (r3[e >> 1] & 0xffff0000u);
        } else {
          o.x = (r0[e >> 1] & 0xffffu) | (r1[e >> 1] << 16);
          o.y = (r2[e >> 1] & 0xffffu) | (r3[e >> 1] << 16);
        }
        const int unit = (pos4 >> 3) ^ vt_unit_swizzle(d);
        *(uint2*)(Vt + d * BN + unit * 8 + (pos4 & 7)) = o;
      }
    }
  };

  load_tile(0);
  for (int kt = 0; kt < n_kv_tiles; ++kt) {
    const int kv0 = kt * BN;
    __syncthreads();                 // everyone is done reading the previous tile
    store_tile();
    __syncthreads();
    if (kt + 1 < n_kv_tiles) load_tile(kt + 1);
    if (kv0 > wave_q0 + 31) continue;          // every key of the tile is in this wave's future

    // ---- S^T = K . Q^T : two 32-key blocks
    f32x16 S[2];
#pragma unroll
    for (int b = 0; b < 2; ++b) {
#pragma unroll
      for (int e = 0; e < 16; ++e) S[b][e] = 0.f;
      const bf16_t* kp = Ks + (32 * b + n32) * KROW + 8 * hh;
#pragma unroll
      for (int s = 0; s < DQK / 16; ++s) {
        const bf16x8 a = __builtin_bit_cast(bf16x8, *(const uint4*)(kp + 16 * s));
        S[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[s], S[b], 0, 0, 0);
      }
    }
    // lane holds, for query qi, keys kv0 + 32b + 8*(i/4) + 4*hh + i%4
    if (kv0 + BN - 1 > wave_q0) {              // tile crosses this wave's diagonal (or the prompt's end)
#pragma unroll
      for (int b = 0; b < 2; ++b)
#pragma unroll
        for (int i = 0; i < 16; ++i)
          if (kv0 + 32 * b + 8 * (i >> 2) + 4 * hh + (i & 3) > qi) S[b][i] = -INFINITY;
    }
    float mx = S[0][0];
#pragma unroll
    for (int i = 1; i < 16; ++i) mx = fmaxf(mx, S[0][i]);
#pragma unroll
    for (int i = 0; i < 16; ++i) mx = fmaxf(mx, S[1][i]);
    mx = fmaxf(mx, __shfl_xor(mx, 32));
    const float m_new = fmaxf(m, mx);
    const float alpha = __builtin_amdgcn_exp2f((m - m_new) * c);
    const float mc = m_new * c;
    float psum = 0.f;
    uint32_t pb[2][8];
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
      for (int i = 0; i < 16; i += 2) {
        const float p0 = __builtin_amdgcn_exp2f(S[b][i] * c - mc);
        const float p1 = __builtin_amdgcn_exp2f(S[b][i + 1] * c - mc);
        psum += p0 + p1;
        pb[b][i >> 1] = cvt_pk_bf16(p0, p1);
      }
    l = l * alpha + psum;
    m = m_new;
#pragma unroll
    for (int blk = 0; blk < DV / 32; ++blk)
#pragma unroll
      for (int e = 0; e < 16; ++e) O[blk][e] *= alpha;

    // ---- O^T += V^T . P^T : four 16-key steps; step kk uses S^T block kk/2, registers 8*(kk%2)..+7
#pragma unroll
    for (int kk = 0; kk < BN / 16; ++kk) {
      const uint4 praw = uint4{pb[kk >> 1][4 * (kk & 1)], pb[kk >> 1][4 * (kk & 1) + 1], pb[kk >> 1][4 * (kk & 1) + 2],
                               pb[kk >> 1][4 * (kk & 1) + 3]};
      const bf16x8 pfrag = __builtin_bit_cast(bf16x8, praw);
#pragma unroll
      for (int blk = 0; blk < DV / 32; ++blk) {
        const int d = 32 * blk + n32;
        const int unit = (2 * kk + hh) ^ vt_unit_swizzle(d);
        const bf16x8 a = __builtin_bit_cast(bf16x8, *(const uint4*)(Vt + d * BN + unit * 8));
        O[blk] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, pfrag, O[blk], 0, 0, 0);
      }
    }
  }

  l += __shfl_xor(l, 32);
  if (qi < w.len) {
    const float inv = 1.f / l;
    bf16_t* op = out + ((size_t)(w.row0 + qi) * H + h) * DV + 4 * hh;
#pragma unroll
    for (int blk = 0; blk < DV / 32; ++blk)
#pragma unroll
      for (int i4 = 0; i4 < 4; ++i4) {
        uint2 pk;
        pk.x = cvt_pk_bf16(O[blk][4 * i4] * inv, O[blk][4 * i4 + 1] * inv);
        pk.y = cvt_pk_bf16(O[blk][4 * i4 + 2] * inv, O[blk][4 * i4 + 3] * inv);
        *(uint2*)(op + 32 * blk + 8 * i4) = pk;
      }
  }
}

bool prefill_shape_supported(int dqk, int dv) {
  return (dqk == 64 && dv == 64) || (dqk == 128 && dv == 128) || (dqk == 192 && dv == 128);
}
int prefill_block_m() { return BM; }

hipError_t launch_prefill(const void* q, const void* k, const void* v, void* out, const PrefillWork* d_work, int n_work,
                          int H, int Hkv, int dqk, int dv, float scale, hipStream_t stream) {
  const float c = scale * 1.4426950408889634f;
  const dim3 grid((unsigned)n_work * (unsigned)H), block(256);
#define SPD_LAUNCH(DQ, DVV)                                                                                         \
  hipLaunchKernelGGL((prefill_kernel<DQ, DVV>), grid, block, 0, stream, (const bf16_t*)q, (const bf16_t*)k,          \
                     (const bf16_t*)v, (bf16_t*)out, d_work, H, Hkv, c)
  if (dqk == 64 && dv == 64) SPD_LAUNCH(64, 64);
  else if (dqk == 128 && dv == 128) SPD_LAUNCH(128, 128);
  else if (dqk == 192 && dv == 128) SPD_LAUNCH(192, 128);
  else return hipErrorInvalidValue;
#undef SPD_LAUNCH
  return hipGetLastError();
}

}  // namespace spd
