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
