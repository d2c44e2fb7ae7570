// Attention mass per tile pair on bf16 MFMA (Sec. 4.2 of the paper: masks are searched by the
// recall they keep, i.e. by how much of the full attention's probability mass falls on the kept
// tile pairs).  For every (batch, head, query tile a) the kernel produces, for all key tiles b,
//     mass[a, b] = sum_{i in a} sum_{j in b} softmax_row_i(scale * Q K^T)[j]
// over real tokens only (padding queries add nothing, padding keys are never attended).
//
// Same decomposition as the attention kernel in attn_bf16.hip: one workgroup per row, a wave owns
// 32 queries, transposed product S^T = K Q^T so that a lane owns one query (QueryWave in
// attn_bf16_common.h), K tiles copied into swizzled LDS, two buffers.  There is no V.
//
// One product per tile pair.  The normaliser l_i of a query is known only after its last key tile,
// so the walk over the n key tiles keeps what it cannot finish: per query i and key tile b the
// unnormalised sum  e[b][i] = sum_{j in b} exp2(scale' * (s_ij - m)), together with the exponent
// reference m it was taken against (it moves when a sum outgrows it, rarely), two floats, written to a workspace in device memory (2 * n * B floats per
// workgroup; 1 KiB per step against a 32 KB tile copy).  After the walk the workgroup reads its
// block back, brings every sum to the query's final reference and reduces over the queries,
//     mass[a, b] = sum_i e[b][i] * exp2(scale' * (m[b][i] - m_i)) / l_i,
// in a fixed order, so the result is run-to-run identical.  (The alternative without a workspace
// walks every row twice and multiplies twice; it measured twice the time per product.)
#include <algorithm>

#include "attn_bf16_common.h"

namespace ca {
namespace {

constexpr float kSumLimit = 0x1p40f;  // a tile's row sum beyond this moves the query's exponent reference

template <int B, int D>
__global__ __attribute__((amdgpu_flat_work_group_size(B * 2, B * 2), amdgpu_waves_per_eu(2, 2)))
void tile_mass_kernel(MassArgs a) {
  using S = Shape<B, D>;
  __shared__ __attribute__((aligned(1024))) char lds_k[2 * S::kTileBytes];
  __shared__ __attribute__((aligned(16))) float lds_inv[B];  // 1 / l_i
  __shared__ __attribute__((aligned(16))) float lds_ref[B];  // m_i
  __shared__ int lds_ticket;

  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int64_t rows = (int64_t)a.num_heads * a.n;
  const int total = (int)a.row_count;  // rows of this launch: items row_base .. row_base + row_count - 1
  // this workgroup's block of the workspace: [n][B] pairs (sum, reference), reused row after row
  float2* part = reinterpret_cast<float2*>(a.partial) + (int64_t)blockIdx.x * a.n * B;
  // one packed word per key tile 0..n-1: tile id | padding class << 24 | bit 31: upper key blocks empty
  const auto meta = CONST_PTR(int32_t, a.dense_meta);
  const auto class_mask = CONST_PTR(uint32_t, a.class_mask);  // 4 words per class
  const int n = (int)a.n;
  const TileLoader<S, false> k_loader(wave, lane);
  const uint32_t lds_k_addr = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char*)lds_k;
  const LdsTile k_tile = (LdsTile)lds_k;

  // The grid is at most as many workgroups as the card holds at a time; each takes (batch, head,
  // query tile) rows of the launch by ticket until none is left, so an XCD that runs faster takes
  // more rows.  Every workgroup draws once more than it has rows; whoever draws the last ticket of
  // all zeroes the counter for the next launch.
  for (;;) {
  if (threadIdx.x == 0) {
    const int t = atomicAdd(a.counter, 1);
    if (t == total + (int)gridDim.x - 1) __hip_atomic_store(a.counter, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    lds_ticket = t;
  }
  __syncthreads();
  if (lds_ticket >= total) return;  // all threads of the workgroup alike
  const int64_t item = a.row_base + lds_ticket;  // (batch, head, query tile), row-major
  const int64_t row = item % rows;
  const int64_t batch = item / rows;
  const int64_t head = row / a.n, q_tile = row - head * a.n;
  const int64_t plane = (batch * a.num_heads + head) * a.n * (int64_t)S::kTileBytes;
  const char* Kp = static_cast<const char*>(a.k) + plane;
  float* out = a.mass + item * a.n;

  // A wave without a real query (see query_slot) takes part in the tile copies and barriers only.
  QueryWave<S> w(lane, a.scale);
  const QuerySlot qs = query_slot<B>(a, q_tile, wave * 32, w.qi);
  const bool wave_active = qs.wave_active;
  w.load_q(static_cast<const char*>(a.q) + plane + (q_tile * B + qs.slot) * S::kRowBytes);
  const int mine = wave * 32 + w.qi;  // this lane's query in the workspace block and in lds_inv
  const bool writer = w.g == 0;       // both lanes of a pair hold the query's sum; the lower one stores it

  // the packed words are fetched two steps ahead of their use (the table is readable two words past its end)
  int32_t word = meta[0], word1 = meta[1];
  k_loader.issue(Kp, lds_k_addr, wave);
  float2 prev = {0.f, 0.f};  // the previous tile's sum and its reference, stored at the head of the next step
  float l_row = 0.f;   // the query's running sum over all key tiles (both lanes of a pair hold it)

  for (int j = 0; j < n; ++j) {
    const int32_t word2 = meta[j + 2];
    // K(j) landed and visible, buffer (j+1)%2 free, the previous step's store has been written
    WAIT_VMCNT(0);
    BARRIER();
    if (j + 1 < n) k_loader.issue(Kp + (int64_t)(j + 1) * S::kTileBytes, lds_k_addr + ((j + 1) & 1) * S::kTileBytes, wave);
    if (j > 0 && writer) part[(int64_t)(j - 1) * B + mine] = prev;  // a whole step to complete

    float e = 0.f;
    if (wave_active) {
      floatx16 acc_s[S::kKeyBlocks];
      w.qk_tile(k_tile + (j & 1) * S::kTileBytes, acc_s, word >= 0);
      w.mask_padding_keys(acc_s, (word >> 24) & 0x7f, class_mask);

      // The exponent reference is the first tile's row maximum.  Afterwards no maximum is taken: the
      // sums are formed against the reference as it stands and only a tile whose row sum leaves
      // [0, kSumLimit] for some query (it overflows, or is about to) is redone for those queries
      // with its row maximum as their new reference.  Numerator and denominator of a query always
      // share one reference after the final pass, so the masses are those of the exact softmax.
      auto row_sum = [&]() {
        float e4[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int kb = 0; kb < S::kKeyBlocks; ++kb)
#pragma unroll
          for (int r = 0; r < 16; ++r) e4[r & 3] += __builtin_amdgcn_exp2f(acc_s[kb][r] * w.c2);
        return sum_with_partner((e4[0] + e4[1]) + (e4[2] + e4[3]));
      };
      bool move = true;  // this lane's query takes a new reference (every query on the first tile)
      if (j > 0) {
        e = row_sum();
        move = !(e <= kSumLimit);  // also true for inf and NaN
      }
      const uint64_t movers = __builtin_amdgcn_ballot_w64(move);
      if (__builtin_amdgcn_readfirstlane((uint32_t)movers | (uint32_t)(movers >> 32)) != 0) {
        float mx = acc_s[0][0];
#pragma unroll
        for (int kb = 0; kb < S::kKeyBlocks; ++kb)
#pragma unroll
          for (int r = 0; r < 16; ++r) mx = fmaxf(mx, acc_s[kb][r]);
        mx = max_with_partner(mx);
        float delta = move ? mx : 0.f;
        if (delta == kMinusInf) delta = 0.f;  // a row that has seen no real key yet keeps its reference
        w.m_run += delta;
        l_row *= __builtin_amdgcn_exp2f(-delta * w.c2);
#pragma unroll
        for (int kb = 0; kb < S::kKeyBlocks; ++kb)
#pragma unroll
          for (int r = 0; r < 16; ++r) acc_s[kb][r] -= delta;
#pragma unroll
        for (int r = 0; r < 16; ++r) w.neg_m[r] = -w.m_run;
        e = row_sum();
      }
      l_row += e;
    }
    prev.x = e;
    prev.y = w.m_run;
    word = word1;
    word1 = word2;
  }

  // ---- mass[a, b] = sum_i e[b][i] * exp2(scale' * (m[b][i] - m_i)) / l_i --------------------------
  if (writer) {
    part[(int64_t)(n - 1) * B + mine] = prev;
    lds_inv[mine] = (qs.real && l_row > 0.f) ? 1.0f / l_row : 0.f;  // a padding query adds nothing
    lds_ref[mine] = w.m_run;
  }
  __threadfence();  // the stored pairs are read back by other waves of this workgroup
  __syncthreads();
  constexpr int kLanesPerTile = B / 4;  // a key tile's B pairs, four per lane
  constexpr int kTilesPerPass = S::kThreads / kLanesPerTile;
  const int sub = threadIdx.x / kLanesPerTile, l4 = threadIdx.x % kLanesPerTile;
  const float4 inv = *reinterpret_cast<const float4*>(&lds_inv[4 * l4]);
  const float4 ref = *reinterpret_cast<const float4*>(&lds_ref[4 * l4]);
  const float c2 = w.c2;
  // kBatch key tiles per lane at a time, all loads requested before the first is used
  constexpr int kBatch = 4;
  for (int b0 = sub; b0 < n; b0 += kBatch * kTilesPerPass) {
    float4 p01[kBatch], p23[kBatch];  // (e0, m0, e1, m1), (e2, m2, e3, m3)
#pragma unroll
    for (int u = 0; u < kBatch; ++u) {
      const int b = min(b0 + u * kTilesPerPass, n - 1);  // past the end: a valid tile, not stored
      const float4* p = reinterpret_cast<const float4*>(part + (int64_t)b * B + 4 * l4);
      p01[u] = p[0];
      p23[u] = p[1];
    }
#pragma unroll
    for (int u = 0; u < kBatch; ++u) {
      const int b = b0 + u * kTilesPerPass;
      const float t0 = p01[u].x * __builtin_amdgcn_exp2f((p01[u].y - ref.x) * c2) * inv.x;
      const float t1 = p01[u].z * __builtin_amdgcn_exp2f((p01[u].w - ref.y) * c2) * inv.y;
      const float t2 = p23[u].x * __builtin_amdgcn_exp2f((p23[u].y - ref.z) * c2) * inv.z;
      const float t3 = p23[u].z * __builtin_amdgcn_exp2f((p23[u].w - ref.w) * c2) * inv.w;
      float s = (t0 + t1) + (t2 + t3);
#pragma unroll
      for (int sh = kLanesPerTile / 2; sh >= 1; sh >>= 1) s += __shfl_xor(s, sh, 64);
      if (l4 == 0 && b < n) out[b] = s;
    }
  }
  __syncthreads();  // the row is done: its ticket and its LDS tables may be overwritten
  }
}

template <int B, int D>
hipError_t launch(MassArgs a, hipStream_t stream) {
  // Launches on one stream run one after another, so each has the workspace and the counter to itself.
  const int64_t items = (int64_t)a.batch * a.num_heads * a.n;
  for (int64_t base = 0; base < items; base += a.rows_per_launch) {
    a.row_base = base;
    a.row_count = std::min(items - base, a.rows_per_launch);
    const int64_t grid = std::min(a.row_count, a.partial_rows);
    hipLaunchKernelGGL((tile_mass_kernel<B, D>), dim3((unsigned)grid), dim3(B * 2), 0, stream, a);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  return hipSuccess;
}

}  // namespace

hipError_t launch_tile_mass(const MassArgs& a, hipStream_t stream) {
  const int64_t items = (int64_t)a.batch * a.num_heads * a.n;
  if (items == 0) return hipSuccess;
  if (!a.partial || !a.counter || a.partial_rows < 1 || a.rows_per_launch < 1) return hipErrorInvalidValue;
  if (std::min(items, a.rows_per_launch) + a.partial_rows > 0x7fffffff) return hipErrorInvalidValue;
  if (a.B == 128 && a.D == 128) return launch<128, 128>(a, stream);
  if (a.B == 128 && a.D == 64) return launch<128, 64>(a, stream);
  if (a.B == 64 && a.D == 128) return launch<64, 128>(a, stream);
  if (a.B == 64 && a.D == 64) return launch<64, 64>(a, stream);
  return hipErrorInvalidValue;
}

}  // namespace ca
