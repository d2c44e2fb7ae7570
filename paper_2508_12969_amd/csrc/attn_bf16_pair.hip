// The paired kernel for 64-token tiles with head dim 128: every workgroup serves two query tiles
// (attn_bf16_pair_body.h).
#include "attn_bf16_pair_body.h"

namespace ca {
namespace {

template <bool kNat>
__global__ __attribute__((amdgpu_flat_work_group_size(256, 256), amdgpu_waves_per_eu(2, 2)))
void attn_bf16_pair_kernel(AttnArgs a) {
  using S = PairShape<64>;
  __shared__ __attribute__((aligned(1024))) char lds_k[S::kTileBytes];
  __shared__ __attribute__((aligned(1024))) char lds_v[S::kTileBytes];
  __shared__ int pool_ticket;
  const int64_t linear = launch_entry(a, &pool_ticket);
  if (linear < 0) return;  // a surplus pool workgroup (all of its threads)
  attn_pair_body<64, kNat>(a, linear % a.num_pairs, linear / a.num_pairs, lds_k, lds_v);
}

}  // namespace

hipError_t launch_attn_bf16_pair(const AttnArgs& a, hipStream_t stream) {
  const int64_t items = (int64_t)a.batch * a.num_pairs;
  if (items == 0) return hipSuccess;
  if (a.B != 64 || a.D != 128 || !a.pair_rows || !a.pair_desc) return hipErrorInvalidValue;
  if (a.static_items + a.pool_wgs > 0x7fffffff || a.static_items + a.pool_items != items) return hipErrorInvalidValue;
  if (a.natural && a.tw % PairShape<64>::kRowsPerLoad != 0) return hipErrorInvalidValue;  // a KiB block must stay inside one run
  const dim3 grid((unsigned)(a.static_items + a.pool_wgs)), block(256);
  if (a.natural) hipLaunchKernelGGL((attn_bf16_pair_kernel<true>), grid, block, 0, stream, a);
  else hipLaunchKernelGGL((attn_bf16_pair_kernel<false>), grid, block, 0, stream, a);
  return hipGetLastError();
}

}  // namespace ca
