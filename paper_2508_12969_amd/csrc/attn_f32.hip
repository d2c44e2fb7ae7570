// Plain fp32 sparse attention: one workgroup per (batch, head, query tile), one thread per
// query token, keys streamed through LDS a few at a time.  It follows Appendix D's block loop
// literally (running max, running sum, rescaled accumulator, one key at a time) and exists for
// fp32 problems and as an on-device cross-check of the MFMA kernel; it is not tuned.
#include "kernels.h"

namespace ca {
namespace {

constexpr int kKeysPerStage = 16;
constexpr float kLog2e = 1.4426950408889634f;

template <int D>
__global__ __launch_bounds__(128) void attn_f32_kernel(AttnArgs a) {
  __shared__ float ks[kKeysPerStage][D];
  __shared__ float vs[kKeysPerStage][D];

  const int64_t rows = (int64_t)a.num_heads * a.n;
  const int64_t item = blockIdx.x % rows;
  const int64_t b = blockIdx.x / rows;
  const int64_t row = a.order ? a.order[item] : item;
  const int64_t head = row / a.n, q_tile = row % a.n;
  const int64_t plane = (b * a.num_heads + head) * a.n * a.B * D;
  const float* Q = static_cast<const float*>(a.q) + plane;
  const float* K = static_cast<const float*>(a.k) + plane;
  const float* V = static_cast<const float*>(a.v) + plane;
  float* O = static_cast<float*>(a.out) + plane;

  const int tid = threadIdx.x;
  const bool has_query = tid < a.B;
  const SlotMask qmask = a.class_mask[a.tile_class[q_tile]];
  const bool q_real = has_query && ((qmask.w[tid >> 5] >> (tid & 31)) & 1u);

  float q[D], o[D];
#pragma unroll
  for (int c = 0; c < D; ++c) {
    q[c] = has_query ? Q[(q_tile * a.B + tid) * D + c] : 0.f;
    o[c] = 0.f;
  }
  float m = -1e30f, l = 0.f;
  const float c2 = a.scale * kLog2e;  // scores are kept in log2 units

  const int64_t begin = a.row_ptr ? a.row_ptr[row] : 0;
  const int64_t count = a.row_ptr ? a.row_ptr[row + 1] - begin : a.n;
  for (int64_t j = 0; j < count; ++j) {
    const int32_t word = a.col_meta[begin + j];  // tile id | padding class << 24 | half-empty flag << 31
    const int64_t kv_tile = word & 0xffffff;
    const SlotMask kmask = a.class_mask[(word >> 24) & 0x7f];
    for (int k0 = 0; k0 < a.B; k0 += kKeysPerStage) {
      const int stage = min(kKeysPerStage, a.B - k0);
      __syncthreads();
      for (int e = tid; e < stage * D; e += blockDim.x) {
        const int kk = e / D, c = e % D;
        ks[kk][c] = K[(kv_tile * a.B + k0 + kk) * D + c];
        vs[kk][c] = V[(kv_tile * a.B + k0 + kk) * D + c];
      }
      __syncthreads();
      for (int kk = 0; kk < stage; ++kk) {
        const int slot = k0 + kk;
        if (!((kmask.w[slot >> 5] >> (slot & 31)) & 1u)) continue;  // padding key: never attended
        float s = 0.f;
#pragma unroll
        for (int c = 0; c < D; ++c) s = fmaf(q[c], ks[kk][c], s);
        s *= c2;
        const float m_new = fmaxf(m, s);
        const float alpha = exp2f(m - m_new);
        const float p = exp2f(s - m_new);
        l = l * alpha + p;
#pragma unroll
        for (int c = 0; c < D; ++c) o[c] = fmaf(p, vs[kk][c], o[c] * alpha);
        m = m_new;
      }
    }
  }
  if (has_query) {
    const float inv = (q_real && l > 0.f) ? 1.f / l : 0.f;
#pragma unroll
    for (int c = 0; c < D; ++c) O[(q_tile * a.B + tid) * D + c] = o[c] * inv;
  }
}

}  // namespace

hipError_t launch_attn_f32(const AttnArgs& a, hipStream_t stream) {
  const int64_t items = (int64_t)a.batch * a.num_heads * a.n;
  if (items == 0) return hipSuccess;
  if (items > 0x7fffffff) return hipErrorInvalidValue;
  const dim3 grid((unsigned)items), block(128);
  switch (a.D) {
    case 32: hipLaunchKernelGGL(attn_f32_kernel<32>, grid, block, 0, stream, a); break;
    case 64: hipLaunchKernelGGL(attn_f32_kernel<64>, grid, block, 0, stream, a); break;
    case 128: hipLaunchKernelGGL(attn_f32_kernel<128>, grid, block, 0, stream, a); break;
    default: return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

}  // namespace ca
