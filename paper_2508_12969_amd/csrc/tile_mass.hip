// Attention mass per tile pair on bf16 MFMA (Sec. 4.2 of the paper: masks are searched by the
// recall they keep, i.e. by how much of the full attention's probability mass falls on the kept
// tile pairs).  For every (batch, head, query tile a) the kernel produces, for all key tiles b,
//     mass[a, b] = sum_{i in a} sum_{j in b} softmax_row_i(scale * Q K^T)[j]
// over real tokens only (padding queries add nothing, padding keys are never attended).
//
// Same decomposition as the attention kernel in attn_bf16.hip: one workgroup per row, a wave owns
// 32 queries, transposed product S^T = K Q^T so that a lane owns one query, K tiles copied into
// swizzled LDS, two buffers.  There is no V.  The row is walked twice over all n key tiles:
//   walk 1  running exponent reference and row sum l_i (lazy reference as in the attention kernel);
//   walk 2  the scores again, p = exp2(scale' * (s - m_i)) / l_i, summed over the lane's registers,
//           the wave and the workgroup's waves (fixed order, so the result is run-to-run
//           identical), one float per key tile.
// The second product is the price of not storing the N x N scores; the whole call costs as many
// FLOPs as one dense attention pass.
#include "attn_bf16_common.h"

namespace ca {
namespace {

template <int B, int D>
__global__ __attribute__((amdgpu_flat_work_group_size(B * 2, B * 2), amdgpu_waves_per_eu(2, 2)))
void tile_mass_kernel(MassArgs a) {
  using S = Shape<B, D>;
  __shared__ __attribute__((aligned(1024))) char lds_k[2 * S::kTileBytes];
  __shared__ float lds_part[2][S::kWaves];

  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int qi = lane & 31;  // query column owned by this lane inside the wave's 32 queries
  const int g = lane >> 5;   // lane group: which half of every 8-key pair this lane holds

  const int64_t rows = (int64_t)a.num_heads * a.n;
  const int64_t row = blockIdx.x % rows;
  const int64_t batch = blockIdx.x / rows;
  const int64_t head = row / a.n, q_tile = row - head * a.n;
  const int64_t plane = (batch * a.num_heads + head) * a.n * (int64_t)S::kTileBytes;
  const char* Kp = static_cast<const char*>(a.k) + plane;
  float* out = a.mass + ((batch * a.num_heads + head) * a.n + q_tile) * a.n;
  const auto tile_class = CONST_PTR(int32_t, a.tile_class);
  const auto class_mask = CONST_PTR(uint32_t, a.class_mask);  // 4 words per class
  const int n = (int)a.n;

  const float c2 = a.scale * kLog2e;
  const float lazy_raw = kLazyLog2 / c2;
  const uint32_t q_valid = class_mask[tile_class[q_tile] * 4 + wave];
  const bool q_real = (q_valid >> qi) & 1u;

  // Q fragment: B operand of S^T, lane (qi, g) holds d = 16*step + 8*g .. +7 of its query.
  bf16x8 qf[S::kQkSteps];
  {
    const int64_t q_row = q_tile * B + wave * 32 + qi;
    const char* Qp = static_cast<const char*>(a.q) + plane + q_row * S::kRowBytes + g * 16;
#pragma unroll
    for (int s = 0; s < S::kQkSteps; ++s) qf[s] = *reinterpret_cast<const bf16x8*>(Qp + s * 32);
    // wait for these loads here: inside the loops the vector-memory counter belongs to the tile copies
#pragma unroll
    for (int s = 0; s < S::kQkSteps; ++s) asm volatile("" : "+v"(qf[s]));
  }

  // exponent reference of this lane's query (raw units); neg_m = -m_run in all 16 registers is the
  // C operand of the first contraction step, so scores leave the MFMA as (score - reference)
  float m_run = 0.f, l_run = 0.f;
  floatx16 neg_m;
#pragma unroll
  for (int r = 0; r < 16; ++r) neg_m[r] = 0.f;

  const int k_lane_row_off = qi * S::kRowBytes;
  const int k_lane_swz = k_swizzle<D>(qi);
  const TileLoader<S, false> k_loader(wave, lane);
  const uint32_t lds_k_addr = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char*)lds_k;

  // scores of key tile j (already in LDS buffer j%2) against this wave's queries, padding keys -inf
  auto scores = [&](int j, floatx16 (&acc_s)[S::kKeyBlocks]) {
    const char* kbuf = lds_k + (j & 1) * S::kTileBytes;
#pragma unroll
    for (int s = 0; s < S::kQkSteps; ++s) {
#pragma unroll
      for (int kb = 0; kb < S::kKeyBlocks; ++kb) {
        const int off = kb * 32 * S::kRowBytes + k_lane_row_off + (((2 * s + g) ^ k_lane_swz) << 4);
        const bf16x8 kf = *reinterpret_cast<const bf16x8*>(kbuf + off);
        acc_s[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[s], s == 0 ? neg_m : acc_s[kb], 0, 0, 0);
      }
    }
    const int cls = __builtin_amdgcn_readfirstlane(tile_class[j]);
    if (cls != 0) {  // wave-uniform: only tiles on a padded face of the grid have invalid slots
#pragma unroll
      for (int kb = 0; kb < S::kKeyBlocks; ++kb) {
        const uint32_t bits = __builtin_amdgcn_readfirstlane(class_mask[cls * 4 + kb]);
        if (bits != 0xffffffffu) {
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const int bit = 8 * (r / 4) + (r % 4);  // lanes 0-31 hold key 8*(r/4) + r%4 of the block, lanes 32-63 that + 4
            const uint32_t lo = 0u - ((bits >> bit) & 1u), hi = 0u - ((bits >> (bit + 4)) & 1u);
            const uint64_t keep = (uint64_t)lo | ((uint64_t)hi << 32);
            asm("v_cndmask_b32 %0, %1, %0, %2" : "+v"(acc_s[kb][r]) : "v"(kMinusInf), "s"(keep));
          }
        }
      }
    }
  };
  // top of a step: K(j) landed and visible, buffer (j+1)%2 free; start the next copy
  auto step_begin = [&](int j) {
    WAIT_VMCNT(0);
    WAIT_LGKMCNT0();  // this wave's partial sum of the previous tile is in LDS
    BARRIER();
    if (j + 1 < n) k_loader.issue(Kp + (int64_t)(j + 1) * S::kTileBytes, lds_k_addr + ((j + 1) & 1) * S::kTileBytes, wave);
  };

  // ---- walk 1: exponent reference and row sum ------------------------------------------------
  k_loader.issue(Kp, lds_k_addr, wave);
  for (int j = 0; j < n; ++j) {
    step_begin(j);
    floatx16 acc_s[S::kKeyBlocks];
    scores(j, acc_s);
    float mx = acc_s[0][0];
#pragma unroll
    for (int kb = 0; kb < S::kKeyBlocks; ++kb)
#pragma unroll
      for (int r = 0; r < 16; ++r) mx = fmaxf(mx, acc_s[kb][r]);
    mx = max_with_partner(mx);
    const uint64_t over = __builtin_amdgcn_ballot_w64(mx > lazy_raw);
    if (j == 0 || __builtin_amdgcn_readfirstlane((uint32_t)over | (uint32_t)(over >> 32)) != 0) {
      float delta = (j == 0 || mx > lazy_raw) ? mx : 0.f;
      if (delta == kMinusInf) delta = 0.f;
      const float alpha = j == 0 ? 1.0f : __builtin_amdgcn_exp2f(-delta * c2);
      m_run += delta;
      l_run *= alpha;
#pragma unroll
      for (int kb = 0; kb < S::kKeyBlocks; ++kb)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc_s[kb][r] -= delta;
#pragma unroll
      for (int r = 0; r < 16; ++r) neg_m[r] = -m_run;
    }
#pragma unroll
    for (int kb = 0; kb < S::kKeyBlocks; ++kb)
#pragma unroll
      for (int r = 0; r < 16; ++r) l_run += __builtin_amdgcn_exp2f(acc_s[kb][r] * c2);
  }
  const float l_tot = sum_with_partner(l_run);
  const float inv = (q_real && l_tot > 0.f) ? 1.0f / l_tot : 0.f;

  // ---- walk 2: probabilities summed per key tile -----------------------------------------------
  BARRIER();  // every wave has left walk 1 before buffer 0 is refilled
  k_loader.issue(Kp, lds_k_addr, wave);
  for (int j = 0; j < n; ++j) {
    step_begin(j);
    if (j > 0 && threadIdx.x == 0) {  // the partial sums of tile j-1 were published before the barrier
      float m = 0.f;
#pragma unroll
      for (int w = 0; w < S::kWaves; ++w) m += lds_part[(j - 1) & 1][w];
      out[j - 1] = m;
    }
    floatx16 acc_s[S::kKeyBlocks];
    scores(j, acc_s);
    float part = 0.f;
#pragma unroll
    for (int kb = 0; kb < S::kKeyBlocks; ++kb)
#pragma unroll
      for (int r = 0; r < 16; ++r) part += __builtin_amdgcn_exp2f(acc_s[kb][r] * c2);
    part *= inv;
#pragma unroll
    for (int sh = 32; sh >= 1; sh >>= 1) part += __shfl_xor(part, sh, 64);
    if (lane == 0) lds_part[j & 1][wave] = part;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    float m = 0.f;
#pragma unroll
    for (int w = 0; w < S::kWaves; ++w) m += lds_part[(n - 1) & 1][w];
    out[n - 1] = m;
  }
}

template <int B, int D>
hipError_t launch(const MassArgs& a, hipStream_t stream) {
  const int64_t items = (int64_t)a.batch * a.num_heads * a.n;
  hipLaunchKernelGGL((tile_mass_kernel<B, D>), dim3((unsigned)items), dim3(B * 2), 0, stream, a);
  return hipGetLastError();
}

}  // namespace

hipError_t launch_tile_mass(const MassArgs& a, hipStream_t stream) {
  const int64_t items = (int64_t)a.batch * a.num_heads * a.n;
  if (items == 0) return hipSuccess;
  if (items > 0x7fffffff) return hipErrorInvalidValue;
  if (a.B == 128 && a.D == 128) return launch<128, 128>(a, stream);
  if (a.B == 128 && a.D == 64) return launch<128, 64>(a, stream);
  if (a.B == 64 && a.D == 128) return launch<64, 128>(a, stream);
  if (a.B == 64 && a.D == 64) return launch<64, 64>(a, stream);
  return hipErrorInvalidValue;
}

}  // namespace ca
