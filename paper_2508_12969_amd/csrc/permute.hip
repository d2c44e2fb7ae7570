// Tile-order flattening of the token sequence and its inverse (Sec. 3.1 / Appendix D of the
// paper): every run of B consecutive tokens of the permuted sequence is one tt x th x tw tile.
//
// HBM-bound copy.  One workgroup moves one tile of one (batch, head) plane.  Inside a tile the
// tw tokens that share (frame, row) are contiguous in both orders, so the unit of work is such a
// run: a wave derives the run's two offsets with scalar arithmetic and its lanes move 16-byte
// chunks, which keeps every access a full-width contiguous burst.  Padding slots are written as
// zero on the way in and skipped on the way out.
#include "kernels.h"

namespace ca {
namespace {

typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

constexpr int kThreads = 256;
constexpr int kWaves = kThreads / 64;

__global__ __launch_bounds__(kThreads) void permute_kernel(PermuteArgs a) {
  const int64_t tile = blockIdx.x;
  const int64_t plane = blockIdx.y;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int lane = threadIdx.x & 63;
  const int64_t rb = a.row_bytes;

  const char* nat = static_cast<const char*>(a.inverse ? (const void*)a.dst : a.src) + plane * a.N_real * rb;
  const char* til = static_cast<const char*>(a.inverse ? a.src : (const void*)a.dst) + plane * a.N_pad * rb;

  const int runs = a.tt * a.th;                      // runs of tw tokens in a tile
  const int run_chunks = (int)((a.tw * rb) >> 4);    // 16-byte chunks per run
  int kt = 0, kh = 0, kw = 0;
  const bool text = tile >= a.n_vid;
  if (!text) {
    kw = (int)(tile % a.nW);
    const int64_t r = tile / a.nW;
    kh = (int)(r % a.nH);
    kt = (int)(r / a.nH);
  }
  for (int run = wave; run < runs; run += kWaves) {
    int64_t nat_off;   // byte offset of the run's first token in natural order
    int valid_chunks;  // chunks of the run that hold real tokens
    if (text) {
      nat_off = (a.N_video + (tile - a.n_vid) * a.B + (int64_t)run * a.tw) * rb;
      valid_chunks = run_chunks;
    } else {
      const int dt = run / a.th, dy = run - dt * a.th;
      const int t = kt * a.tt + dt, y = kh * a.th + dy, x0 = kw * a.tw;
      const int xs = (t < a.T && y < a.H) ? min(a.tw, a.W - x0) : 0;
      nat_off = (((int64_t)t * a.H + y) * a.W + x0) * rb;
      valid_chunks = (int)((xs * rb) >> 4);
    }
    const int64_t til_off = (tile * a.B + (int64_t)run * a.tw) * rb;
    if (!a.inverse) {
      for (int c = lane; c < run_chunks; c += 64) {
        u32x4 val = {0u, 0u, 0u, 0u};
        if (c < valid_chunks) val = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(nat + nat_off) + c);
        __builtin_nontemporal_store(val, reinterpret_cast<u32x4*>(const_cast<char*>(til) + til_off) + c);
      }
    } else {
      for (int c = lane; c < valid_chunks; c += 64) {
        const u32x4 val = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(til + til_off) + c);
        __builtin_nontemporal_store(val, reinterpret_cast<u32x4*>(const_cast<char*>(nat) + nat_off) + c);
      }
    }
  }
}

}  // namespace

hipError_t launch_permute(const PermuteArgs& a, hipStream_t stream) {
  const int64_t n_tiles = a.N_pad / a.B;
  if (n_tiles == 0 || a.planes == 0) return hipSuccess;
  if (a.planes > 65535) return hipErrorInvalidValue;
  dim3 grid((unsigned)n_tiles, (unsigned)a.planes, 1);
  hipLaunchKernelGGL(permute_kernel, grid, dim3(kThreads), 0, stream, a);
  return hipGetLastError();
}

}  // namespace ca
