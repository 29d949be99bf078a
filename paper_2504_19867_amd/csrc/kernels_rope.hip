// Rotary position embedding, in place, on the query and key rows of a step.
//
// Paper, Evaluation, "Implementation based on DistServe": the implementation carries a RoPE kernel,
// modified for the Llama-3.1 models; it runs on the phase's partition before the attention step.
// A head vector at token position p is rotated pairwise, pair i by the angle p * w_i:
//     x'_a = x_a cos - x_b sin,   x'_b = x_b cos + x_a sin
// with (a, b) = (off + i, off + i + R/2) in the half layout, (off + 2i, off + 2i + 1) in the
// interleaved one (R rotating entries starting at entry off of every head).  The frequencies w_i come
// from the host in fp64, Llama-3.1 scaling already applied.
//
// Bound by HBM: every row is read and written once.  A thread owns 8 pairs of one token (two 16-byte
// pieces of a head) and walks over a chunk of heads, so the 8 angles are computed once per thread:
// angle in fp64 (p * w reaches 1e5 rad, fp32 would lose the low bits that matter), reduced to
// [-pi, pi], then the fp32 library sine / cosine.
#include "internal.h"

namespace spd {

typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));

__device__ inline float bf_lo(uint32_t w) { return __builtin_bit_cast(float, w << 16); }
__device__ inline float bf_hi(uint32_t w) { return __builtin_bit_cast(float, w & 0xffff0000u); }
__device__ inline uint32_t pack_bf16(float a, float b) {
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(f32x2{a, b}, bf16x2));
}

struct RopeArgs {
  unsigned short* x[2];   // q, k (k may be null)
  int heads[2];
  int dim, rot, off;      // entries per head, rotating entries, first rotating entry
  int n_tokens;
  int groups;             // rot / 16: threads per (token, head chunk)
  int chunk;              // heads per thread
  int chunks[2];          // head chunks of q, of k
  const int32_t* pos;     // [n_tokens]
  const double* w;        // [rot / 2]
};

template <bool INTERLEAVED>
__global__ __launch_bounds__(256) void rope_kernel(RopeArgs a) {
  const long long tid = (long long)blockIdx.x * 256 + threadIdx.x;
  const int per_token = (a.chunks[0] + a.chunks[1]) * a.groups;
  const long long t = tid / per_token;
  if (t >= a.n_tokens) return;
  int rem = (int)(tid - t * per_token);
  const int g = rem % a.groups;
  int c = rem / a.groups;
  const int which = c < a.chunks[0] ? 0 : 1;
  if (which) c -= a.chunks[0];
  const int h0 = c * a.chunk, h1 = min(h0 + a.chunk, a.heads[which]);

  // the 8 pairs of this thread: pair index 8 g + j
  float cs[8], sn[8];
  const double p = (double)a.pos[t];
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    const double turns = p * a.w[8 * g + j] * 0.15915494309189535;   // angle / 2 pi
    const float r = (float)((turns - __builtin_rint(turns)) * 6.283185307179586);   // in [-pi, pi]
    sincosf(r, &sn[j], &cs[j]);
  }
  // entry offsets of the two 16-byte pieces inside a head
  const int ea = INTERLEAVED ? a.off + 16 * g : a.off + 8 * g;
  const int eb = INTERLEAVED ? a.off + 16 * g + 8 : a.off + a.rot / 2 + 8 * g;
  unsigned short* row = a.x[which] + ((size_t)t * a.heads[which] + h0) * a.dim;
  for (int h = h0; h < h1; ++h, row += a.dim) {
    uint4 A = *(const uint4*)(row + ea), B = *(const uint4*)(row + eb);
    uint32_t aw[4] = {A.x, A.y, A.z, A.w}, bw[4] = {B.x, B.y, B.z, B.w};
    if (INTERLEAVED) {
      // word j of A holds pair j (low half = a, high half = b); word j of B holds pair 4 + j
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const float xa = bf_lo(aw[j]), xb = bf_hi(aw[j]);
        aw[j] = pack_bf16(xa * cs[j] - xb * sn[j], xb * cs[j] + xa * sn[j]);
        const float ya = bf_lo(bw[j]), yb = bf_hi(bw[j]);
        bw[j] = pack_bf16(ya * cs[4 + j] - yb * sn[4 + j], yb * cs[4 + j] + ya * sn[4 + j]);
      }
    } else {
      // entry e of A pairs with entry e of B
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const float a0 = bf_lo(aw[j]), a1 = bf_hi(aw[j]), b0 = bf_lo(bw[j]), b1 = bf_hi(bw[j]);
        aw[j] = pack_bf16(a0 * cs[2 * j] - b0 * sn[2 * j], a1 * cs[2 * j + 1] - b1 * sn[2 * j + 1]);
        bw[j] = pack_bf16(b0 * cs[2 * j] + a0 * sn[2 * j], b1 * cs[2 * j + 1] + a1 * sn[2 * j + 1]);
      }
    }
    *(uint4*)(row + ea) = uint4{aw[0], aw[1], aw[2], aw[3]};
    *(uint4*)(row + eb) = uint4{bw[0], bw[1], bw[2], bw[3]};
  }
}

hipError_t launch_rope(void* q, int n_q_heads, void* k, int n_kv_heads, int dim, int rot, int off, bool interleaved,
                       int n_tokens, const int32_t* d_pos, const double* d_w, hipStream_t stream) {
  RopeArgs a;
  a.x[0] = (unsigned short*)q;
  a.x[1] = (unsigned short*)k;
  a.heads[0] = n_q_heads;
  a.heads[1] = k ? n_kv_heads : 0;
  a.dim = dim; a.rot = rot; a.off = off; a.n_tokens = n_tokens;
  a.groups = rot / 16;
  // enough threads to fill the chip even for a decode batch, at most 8 heads per thread
  const int total_heads = a.heads[0] + a.heads[1];
  int chunk = 8;
  while (chunk > 1 && (long long)n_tokens * a.groups * ((total_heads + chunk - 1) / chunk) < 4 * 256 * 256) chunk >>= 1;
  a.chunk = chunk;
  a.chunks[0] = (a.heads[0] + chunk - 1) / chunk;
  a.chunks[1] = (a.heads[1] + chunk - 1) / chunk;
  a.pos = d_pos; a.w = d_w;
  const long long threads = (long long)n_tokens * (a.chunks[0] + a.chunks[1]) * a.groups;
  if (threads == 0) return hipSuccess;
  const dim3 grid((unsigned)((threads + 255) / 256));
  if (interleaved) hipLaunchKernelGGL(rope_kernel<true>, grid, dim3(256), 0, stream, a);
  else hipLaunchKernelGGL(rope_kernel<false>, grid, dim3(256), 0, stream, a);
  return hipGetLastError();
}

}  // namespace spd

// ------------------------------------------------------------------------------------------------
// Decode step with RoPE: one launch rotates the new token's query (into a workspace copy, the caller's
// tensor is left alone) and key, and appends the rotated key and the value to the request's page
// (paper, Evaluation "Implementation based on DistServe": the RoPE kernel; Background: the decode
// phase appends the new key / value to the cache).  One workgroup per request; the token's position
// is ctx_len - 1.  Sixteen-byte pieces of 8 entries: a piece inside the rotating range reads its
// partner piece as well and produces its own 8 rotated entries.
namespace spd {

struct RopeAppendArgs {
  const unsigned short* q;
  unsigned short* q_out;
  const unsigned short* k;
  const unsigned short* v;
  int Hq, Hkv, dq, dk, dv;
  int rot, off, interleaved;
  const double* w;
  const int32_t* ctx_lens;
  const TileDesc* descs;
  char* base;
  uint64_t page_bytes;
  uint32_t head_bytes, tile_bytes, tile_k_bytes;
  int natural;
};

// the 8 entries starting at entry e0 of a head vector `row`, rotated
__device__ inline uint4 rope_piece(const unsigned short* row, int e0, int off, int rot, bool interleaved, const float* cs,
                                   const float* sn) {
  const uint4 own = *(const uint4*)(row + e0);
  if (e0 < off || e0 >= off + rot) return own;
  uint32_t ow[4] = {own.x, own.y, own.z, own.w};
  if (interleaved) {
    const int p0 = (e0 - off) >> 1;               // first pair of the piece
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const float xa = bf_lo(ow[j]), xb = bf_hi(ow[j]);
      ow[j] = pack_bf16(xa * cs[p0 + j] - xb * sn[p0 + j], xb * cs[p0 + j] + xa * sn[p0 + j]);
    }
  } else {
    const int half = rot >> 1;
    const bool first = e0 < off + half;           // this piece holds the a side of its 8 pairs
    const int p0 = first ? e0 - off : e0 - off - half;
    const uint4 oth = *(const uint4*)(row + (first ? e0 + half : e0 - half));
    const uint32_t tw[4] = {oth.x, oth.y, oth.z, oth.w};
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const float m0 = bf_lo(ow[j]), m1 = bf_hi(ow[j]), o0 = bf_lo(tw[j]), o1 = bf_hi(tw[j]);
      const float c0 = cs[p0 + 2 * j], s0 = sn[p0 + 2 * j], c1 = cs[p0 + 2 * j + 1], s1 = sn[p0 + 2 * j + 1];
      // a side: x_a cos - x_b sin;  b side: x_b cos + x_a sin
      ow[j] = first ? pack_bf16(m0 * c0 - o0 * s0, m1 * c1 - o1 * s1) : pack_bf16(m0 * c0 + o0 * s0, m1 * c1 + o1 * s1);
    }
  }
  return uint4{ow[0], ow[1], ow[2], ow[3]};
}

__global__ __launch_bounds__(256) void rope_append_kernel(RopeAppendArgs a) {
  __shared__ float cs[128], sn[128];              // rotary_dim <= 256
  const int r = blockIdx.x;
  const int npairs = a.rot >> 1;
  const double p = (double)(a.ctx_lens[r] - 1);
  for (int i = threadIdx.x; i < npairs; i += blockDim.x) {
    const double turns = p * a.w[i] * 0.15915494309189535;
    const float ang = (float)((turns - __builtin_rint(turns)) * 6.283185307179586);
    sincosf(ang, &sn[i], &cs[i]);
  }
  __syncthreads();
  // query: rotated copy
  const int qp = a.dq >> 3;
  for (int i = threadIdx.x; i < a.Hq * qp; i += blockDim.x) {
    const int h = i / qp, c = i % qp;
    const unsigned short* row = a.q + ((size_t)r * a.Hq + h) * a.dq;
    *(uint4*)(a.q_out + ((size_t)r * a.Hq + h) * a.dq + 8 * c) = rope_piece(row, 8 * c, a.off, a.rot, a.interleaved != 0, cs, sn);
  }
  if (a.k == nullptr) return;
  // key: rotated, straight into the page; value: as it is
  const TileDesc d = a.descs[r];
  const int t = d.t_begin;
  const int kp = a.dk >> 3;
  for (int i = threadIdx.x; i < a.Hkv * kp; i += blockDim.x) {
    const int g = i / kp, c = i % kp;
    const unsigned short* row = a.k + ((size_t)r * a.Hkv + g) * a.dk;
    char* tile = a.base + (uint64_t)d.page * a.page_bytes + (uint64_t)g * a.head_bytes + (uint64_t)d.sub * a.tile_bytes;
    const size_t off = a.natural ? (size_t)t * a.dk * 2 + (size_t)c * 16 : ((size_t)(c * 16 + t) << 4);
    *(uint4*)(tile + off) = rope_piece(row, 8 * c, a.off, a.rot, a.interleaved != 0, cs, sn);
  }
  if (a.v == nullptr) return;
  for (int i = threadIdx.x; i < a.Hkv * a.dv; i += blockDim.x) {
    const int g = i / a.dv, dd = i % a.dv;
    char* tile = a.base + (uint64_t)d.page * a.page_bytes + (uint64_t)g * a.head_bytes + (uint64_t)d.sub * a.tile_bytes;
    ((unsigned short*)(tile + a.tile_k_bytes))[v_elem_offset(t, dd)] = a.v[((size_t)r * a.Hkv + g) * a.dv + dd];
  }
}

hipError_t launch_rope_append(const PoolGeom& g, char* pool_base, const TileDesc* d_descs, const int32_t* d_ctx_lens, int B,
                              const void* q, void* q_out, int Hq, int dq, const void* k_new, const void* v_new, int rot,
                              int off, bool interleaved, const double* d_w, hipStream_t stream) {
  if (B <= 0) return hipSuccess;
  RopeAppendArgs a;
  a.q = (const unsigned short*)q; a.q_out = (unsigned short*)q_out;
  a.k = (const unsigned short*)k_new; a.v = (const unsigned short*)v_new;
  a.Hq = Hq; a.Hkv = g.Hkv; a.dq = dq; a.dk = g.dk; a.dv = g.dv;
  a.rot = rot; a.off = off; a.interleaved = interleaved ? 1 : 0;
  a.w = d_w; a.ctx_lens = d_ctx_lens; a.descs = d_descs;
  a.base = pool_base; a.page_bytes = g.page_bytes; a.head_bytes = g.head_bytes; a.tile_bytes = g.tile_bytes;
  a.tile_k_bytes = g.tile_k_bytes; a.natural = g.kind == SPD_KV_MLA_LATENT ? 1 : 0;
  hipLaunchKernelGGL(rope_append_kernel, dim3((unsigned)B), dim3(256), 0, stream, a);
  return hipGetLastError();
}

}  // namespace spd
