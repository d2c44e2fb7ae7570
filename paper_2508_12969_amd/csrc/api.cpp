// C-ABI entry points: argument checking, layout life cycle, device upload, kernel dispatch.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <atomic>
#include <cmath>
#include <cstring>
#include <mutex>
#include <new>
#include <vector>

#include "kernels.h"
#include "layout.h"

using ca::set_error;

namespace {

// Device memory of compact_attn_forward_static: the layout tables of the sparse forward live here
// instead of in allocated memory.  Every GPU the library runs on holds its own copy of the array
// until the process ends.  In host code the name below is only a handle for hipGetSymbolAddress;
// the address kernels and copies use is the per-device pointer kept in g_scratch.
constexpr size_t kScratchBytes = (size_t)8 << 20;
static __device__ __align__(256) unsigned char scratch[kScratchBytes];

constexpr int kMaxDevices = 64;
struct ScratchState {
  unsigned char* ptr = nullptr;  // device address of `scratch` on this device
  uint64_t owner = 0;            // serial of the layout whose tables the last call enqueued there
};
ScratchState g_scratch[kMaxDevices];
std::mutex g_scratch_mutex;
std::atomic<uint64_t> g_next_serial{1};

int fail(int status, const char* what) {
  set_error("%s", what);
  return status;
}

int hip_fail(hipError_t e, const char* where) {
  set_error("%s: %s", where, hipGetErrorString(e));
  return CA_ERR_HIP;
}

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }

int elem_size(int32_t dtype) { return dtype == CA_BF16 ? 2 : 4; }

template <class T>
int upload_vec(const T* host, size_t count, T** dev) {
  *dev = nullptr;
  const size_t bytes = (count ? count : 1) * sizeof(T);
  hipError_t e = hipMalloc(reinterpret_cast<void**>(dev), bytes);
  if (e != hipSuccess) {
    set_error("hipMalloc of %zu bytes for a layout table failed: %s", bytes, hipGetErrorString(e));
    (void)hipGetLastError();
    return CA_ERR_ALLOC;
  }
  if (count) {
    e = hipMemcpy(*dev, host, count * sizeof(T), hipMemcpyHostToDevice);
    if (e != hipSuccess) return hip_fail(e, "hipMemcpy of a layout table");
  }
  return CA_OK;
}

void free_device_tables(ca::DeviceTables& d) {
  if (d.row_ptr) (void)hipFree(d.row_ptr);
  if (d.col_meta) (void)hipFree(d.col_meta);
  if (d.dense_meta) (void)hipFree(d.dense_meta);
  if (d.order) (void)hipFree(d.order);
  if (d.pair_rows) (void)hipFree(d.pair_rows);
  if (d.pair_desc) (void)hipFree(d.pair_desc);
  if (d.launch_rows) (void)hipFree(d.launch_rows);
  if (d.pair_walk_ptr) (void)hipFree(d.pair_walk_ptr);
  if (d.pair_walk) (void)hipFree(d.pair_walk);
  if (d.dense_pair_walk) (void)hipFree(d.dense_pair_walk);
  if (d.tile_class) (void)hipFree(d.tile_class);
  if (d.class_mask) (void)hipFree(d.class_mask);
  if (d.class_perm) (void)hipFree(d.class_perm);
  if (d.tile_origin) (void)hipFree(d.tile_origin);
  if (d.mass_partial) (void)hipFree(d.mass_partial);
  if (d.pool_counters) (void)hipFree(d.pool_counters);
  d = ca::DeviceTables{};
}

// Makes sure the layout's tables are on the current device.  The first call for a layout allocates
// device memory and copies synchronously, which a stream under capture must not see: there the call
// fails and names compact_attn_layout_upload instead.
int ensure_uploaded(ca_layout* L, hipStream_t stream) {
  std::lock_guard<std::mutex> lock(L->upload_mutex);
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return hip_fail(e, "hipGetDevice");
  if (L->uploaded) {
    if (dev != L->device) {
      set_error("layout tables live on device %d but the current device is %d", L->device, dev);
      return CA_ERR_INVALID_ARG;
    }
    return CA_OK;
  }
  if (stream) {
    hipStreamCaptureStatus cap = hipStreamCaptureStatusNone;
    e = hipStreamIsCapturing(stream, &cap);
    if (e != hipSuccess) return hip_fail(e, "hipStreamIsCapturing");
    if (cap != hipStreamCaptureStatusNone) {
      set_error("the layout's tables are not on the device yet and the stream is being captured: call "
                "compact_attn_layout_upload before the capture");
      return CA_ERR_INVALID_ARG;
    }
  }
  ca::PackedTables t;
  int st = ca::pack_device_tables(*L, false, t);
  if (st != CA_OK) return st;
  ca::DeviceTables d;
  st = upload_vec(L->row_ptr.data(), L->row_ptr.size(), &d.row_ptr);
  if (st == CA_OK) st = upload_vec(t.col_meta.data(), t.col_meta.size(), &d.col_meta);
  if (st == CA_OK) st = upload_vec(t.dense_meta.data(), t.dense_meta.size(), &d.dense_meta);
  if (st == CA_OK) st = upload_vec(L->order.data(), L->order.size(), &d.order);
  if (st == CA_OK) st = upload_vec(L->pair_rows.data(), L->pair_rows.size(), &d.pair_rows);
  d.num_pairs = (int64_t)L->pair_rows.size() / 2;
  if (st == CA_OK && d.num_pairs) st = upload_vec(L->pair_desc.data(), L->pair_desc.size(), &d.pair_desc);
  if (st == CA_OK && L->packed_faces) {
    st = upload_vec(L->launch_rows.data(), L->launch_rows.size(), &d.launch_rows);
    d.num_launch_rows = (int64_t)L->launch_rows.size();
  }
  if (st == CA_OK && d.num_pairs) st = upload_vec(L->pair_walk_ptr.data(), L->pair_walk_ptr.size(), &d.pair_walk_ptr);
  if (st == CA_OK && d.num_pairs) st = upload_vec(t.pair_walk.data(), t.pair_walk.size(), &d.pair_walk);
  if (st == CA_OK && d.num_pairs) st = upload_vec(t.dense_pair_walk.data(), t.dense_pair_walk.size(), &d.dense_pair_walk);
  if (st == CA_OK) st = upload_vec(L->tile_class.data(), L->tile_class.size(), &d.tile_class);
  if (st == CA_OK) st = upload_vec(L->class_mask.data(), L->class_mask.size(), &d.class_mask);
  if (st == CA_OK) st = upload_vec(t.class_perm.data(), t.class_perm.size(), &d.class_perm);
  if (st == CA_OK && !t.tile_origin.empty()) st = upload_vec(t.tile_origin.data(), t.tile_origin.size(), &d.tile_origin);
  if (st == CA_OK) {
    const int32_t zeros[ca::kPoolSlots] = {};
    st = upload_vec(zeros, (size_t)ca::kPoolSlots, &d.pool_counters);
    d.pool_slots = ca::kPoolSlots;
  }
  if (st != CA_OK) {
    free_device_tables(d);
    return st;
  }
  L->dev = d;
  L->device = dev;
  L->uploaded = true;
  return CA_OK;
}

// The tile-mass kernel is launched with as many workgroups as the device holds at a time (two waves
// per SIMD), each of which takes rows by ticket and keeps two floats per (query, key tile) of the row
// it is working on.  The workspace for that and the ticket counter are allocated at the first call
// for the layout (not under capture, like the tables) and freed with it.
int ensure_mass_workspace(ca_layout* L, hipStream_t stream) {
  std::lock_guard<std::mutex> lock(L->upload_mutex);
  if (L->dev.mass_partial) return CA_OK;
  if (stream) {
    hipStreamCaptureStatus cap = hipStreamCaptureStatusNone;
    const hipError_t e = hipStreamIsCapturing(stream, &cap);
    if (e != hipSuccess) return hip_fail(e, "hipStreamIsCapturing");
    if (cap != hipStreamCaptureStatusNone) {
      set_error("the tile-mass workspace is not allocated yet and the stream is being captured: call "
                "compact_attn_tile_mass once before the capture");
      return CA_ERR_INVALID_ARG;
    }
  }
  int dev = -1, cus = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e == hipSuccess) e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
  if (e != hipSuccess) return hip_fail(e, "hipDeviceGetAttribute");
  if (cus < 1) cus = 1;
  const int64_t rows_total = (int64_t)L->prob.batch * L->prob.num_heads * L->n;
  const int64_t resident = (int64_t)cus * (8 / (L->B / 32));  // eight waves per CU, B / 32 waves per workgroup
  const int64_t rows = std::max<int64_t>(1, std::min(rows_total, resident));
  const size_t bytes = (size_t)rows * (size_t)L->N_pad * 2 * sizeof(float);
  void* p = nullptr;
  e = hipMalloc(&p, bytes + 256);  // the ticket counter follows the workspace
  if (e != hipSuccess) {
    (void)hipGetLastError();
    set_error("hipMalloc of the tile-mass workspace (%zu bytes): %s", bytes, hipGetErrorString(e));
    return CA_ERR_ALLOC;
  }
  e = hipMemset(static_cast<char*>(p) + bytes, 0, 256);
  if (e != hipSuccess) {
    (void)hipFree(p);
    return hip_fail(e, "hipMemset of the tile-mass ticket counter");
  }
  L->dev.mass_partial = static_cast<float*>(p);
  L->dev.mass_partial_rows = rows;
  L->dev.mass_counter = reinterpret_cast<int32_t*>(static_cast<char*>(p) + bytes);
  return CA_OK;
}

// Do the byte ranges [a, a + na) and [b, b + nb) share a byte?
bool ranges_overlap(const void* a, int64_t na, const void* b, int64_t nb) {
  const uintptr_t a0 = reinterpret_cast<uintptr_t>(a), b0 = reinterpret_cast<uintptr_t>(b);
  return a0 < b0 + (uintptr_t)nb && b0 < a0 + (uintptr_t)na;
}

int check_attn_support(const ca_layout* L) {
  const ca_problem& p = L->prob;
  if (p.dtype == CA_BF16) {
    const bool ok = (L->B == 64 || L->B == 128) && (p.head_dim == 64 || p.head_dim == 128);
    if (!ok) {
      set_error("bf16 attention supports tile sizes 64/128 and head_dim 64/128; got B=%lld D=%d", (long long)L->B,
                p.head_dim);
      return CA_ERR_UNSUPPORTED;
    }
  } else {
    const bool ok = L->B <= 128 && (p.head_dim == 32 || p.head_dim == 64 || p.head_dim == 128);
    if (!ok) {
      set_error("f32 attention supports tile sizes <= 128 and head_dim 32/64/128; got B=%lld D=%d", (long long)L->B,
                p.head_dim);
      return CA_ERR_UNSUPPORTED;
    }
  }
  return CA_OK;
}

// Argument checks shared by the attention entry points.  `natural` selects the natural-order tensor length.
int check_attention_args(const void* q, const void* k, const void* v, const ca_layout* L, const void* out, bool natural) {
  if (!q || !k || !v || !L || !out) return fail(CA_ERR_INVALID_ARG, "null argument");
  if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(out))
    return fail(CA_ERR_INVALID_ARG, "q, k, v and out must be 16-byte aligned");
  int st = check_attn_support(L);
  if (st != CA_OK) return st;
  const ca_problem& p = L->prob;
  const int64_t bytes = (int64_t)p.batch * p.num_heads * (natural ? L->N_real : L->N_pad) * p.head_dim * elem_size(p.dtype);
  if (ranges_overlap(out, bytes, q, bytes) || ranges_overlap(out, bytes, k, bytes) || ranges_overlap(out, bytes, v, bytes))
    return fail(CA_ERR_INVALID_ARG, "out must not overlap q, k or v");
  if (natural) {
    if (p.dtype != CA_BF16) return fail(CA_ERR_UNSUPPORTED, "natural-order attention is built for bf16 problems only");
    const int rows_per_block = 1024 / (p.head_dim * 2);
    if (p.tw % rows_per_block != 0) {
      set_error("natural-order attention needs a tile width that is a multiple of %d tokens at head_dim %d; got tw=%d",
                rows_per_block, p.head_dim, p.tw);
      return CA_ERR_UNSUPPORTED;
    }
    if (L->N_real >= ((int64_t)1 << 31)) return fail(CA_ERR_UNSUPPORTED, "natural-order attention needs fewer than 2^31 tokens");
  }
  return CA_OK;
}

// Fills the kernel arguments from the problem and a set of device tables, and launches.
int launch_attention(const void* q, const void* k, const void* v, const ca_layout* L, const ca::DeviceTables& t, void* out,
                     void* stream, bool dense, bool natural) {
  ca::AttnArgs a{};
  a.q = q;
  a.k = k;
  a.v = v;
  a.out = out;
  a.row_ptr = dense ? nullptr : t.row_ptr;
  a.col_meta = dense ? t.dense_meta : t.col_meta;
  a.pair_rows = t.pair_rows;
  a.num_pairs = t.num_pairs;
  a.pair_desc = t.pair_desc;
  a.pair_walk_ptr = dense ? nullptr : t.pair_walk_ptr;
  a.pair_walk = dense ? t.dense_pair_walk : t.pair_walk;
  a.tile_class = t.tile_class;
  a.class_mask = t.class_mask;
  a.class_perm = t.class_perm;
  a.batch = L->prob.batch;
  a.num_heads = L->prob.num_heads;
  a.n = L->n;
  a.B = (int32_t)L->B;
  a.D = L->prob.head_dim;
  a.scale = L->scale;
  a.natural = natural ? 1 : 0;
  a.tile_origin = t.tile_origin;
  a.H = L->prob.H;
  a.W = L->prob.W;
  a.th = L->prob.th;
  a.tw = L->prob.tw;
  a.n_vid = L->n_vid;
  a.N_real = L->N_real;
  const bool bf16 = L->prob.dtype == CA_BF16;
  // Which kernel serves which rows.  64-token tiles with head dim 128: the paired kernel, all rows.
  // 128-token tiles with head dim 128 on a padded grid: one launch of the one-tile-per-workgroup
  // kernel whose order (launch_rows) also holds the workgroups of packed query tiles.  Everything
  // else: that kernel on `order`.
  const bool all_paired = bf16 && a.B == 64 && a.D == 128;
  const bool some_paired = bf16 && a.B == 128 && a.D == 128 && t.num_pairs > 0 && t.launch_rows;
  a.order = some_paired ? t.launch_rows : (dense ? nullptr : t.order);
  a.entries = some_paired ? t.num_launch_rows : (int64_t)a.num_heads * a.n;
  a.packed = some_paired ? 1 : 0;
  if (a.B == 128)
    for (size_t c = 0; c < L->class_mask.size() && c < 64; ++c)
      if ((L->class_mask[c].w[2] | L->class_mask[c].w[3]) == 0) a.upper_empty_classes |= (uint64_t)1 << c;
  // the statically dealt part of a launch and its dynamically drawn tail (bf16 kernels; the split is
  // that of one batch entry's launch order, the batch entries before the last are static as a whole)
  auto set_split = [&](int64_t entries, const ca::LaunchSplit& sp) {
    a.static_items = entries * a.batch;
    a.pool_items = a.pool_wgs = 0;
    a.pool_counter = nullptr;
    if (bf16 && t.pool_counters && t.pool_slots > 0 && sp.pool_entries > 0) {
      a.static_items = entries * (a.batch - 1) + sp.static_entries;
      a.pool_items = sp.pool_entries;
      a.pool_wgs = (int32_t)std::min<int64_t>(((int64_t)sp.pool_entries * 2 + 7) / 8 * 8, (int64_t)1 << 30);
      a.pool_counter = t.pool_counters + L->launch_seq.fetch_add(1, std::memory_order_relaxed) % (uint32_t)t.pool_slots;
    }
  };
  hipError_t e = hipSuccess;
  if (!all_paired && a.entries > 0) {
    set_split(a.entries, dense ? L->split_rows_dense : L->split_rows);
    e = bf16 ? ca::launch_attn_bf16(a, (hipStream_t)stream) : ca::launch_attn_f32(a, (hipStream_t)stream);
  }
  if (e == hipSuccess && all_paired) {
    set_split(t.num_pairs, dense ? L->split_pairs_dense : L->split_pairs);
    e = ca::launch_attn_bf16_pair(a, (hipStream_t)stream);
  }
  if (e != hipSuccess) return hip_fail(e, dense ? "dense attention launch" : "sparse attention launch");
  return CA_OK;
}

int run_attention(const void* q, const void* k, const void* v, ca_layout* L, void* out, void* stream, bool dense,
                  bool natural = false) {
  ca::clear_error();
  int st = check_attention_args(q, k, v, L, out, natural);
  if (st != CA_OK) return st;
  st = ensure_uploaded(L, (hipStream_t)stream);
  if (st != CA_OK) return st;
  return launch_attention(q, k, v, L, L->dev, out, stream, dense, natural);
}

// Packs the sparse forward's tables into L->static_image (once per layout).  Caller holds g_scratch_mutex.
int build_static_image(ca_layout* L) {
  if (!L->static_image.empty()) return CA_OK;
  ca::PackedTables t;
  int st = ca::pack_device_tables(*L, true, t);
  if (st != CA_OK) return st;
  auto aligned = [](size_t x) { return (x + 255) & ~(size_t)255; };
  struct Part {
    const void* src;
    size_t bytes;
    size_t* off;
  };
  ca_layout::StaticOffsets& o = L->static_off;
  const bool paired = !L->pair_rows.empty();
  const Part parts[] = {
      {L->row_ptr.data(), L->row_ptr.size() * sizeof(int64_t), &o.row_ptr},
      {t.col_meta.data(), t.col_meta.size() * sizeof(int32_t), &o.col_meta},
      {L->order.data(), L->order.size() * sizeof(int32_t), &o.order},
      {L->pair_rows.data(), paired ? L->pair_rows.size() * sizeof(int32_t) : 0, &o.pair_rows},
      {L->pair_walk_ptr.data(), paired ? L->pair_walk_ptr.size() * sizeof(int64_t) : 0, &o.pair_walk_ptr},
      {t.pair_walk.data(), paired ? t.pair_walk.size() * sizeof(int32_t) : 0, &o.pair_walk},
      {L->tile_class.data(), L->tile_class.size() * sizeof(int32_t), &o.tile_class},
      {L->class_mask.data(), L->class_mask.size() * sizeof(ca::SlotMask), &o.class_mask},
      {t.class_perm.data(), t.class_perm.size(), &o.class_perm},
      {nullptr, 2 * 256, &o.pool_counter},  // two ticket counters, 256 bytes apart; they stay zero: the kernels put them back after every launch
      {L->pair_desc.data(), paired ? L->pair_desc.size() * sizeof(int32_t) : 0, &o.pair_desc},
      {L->launch_rows.data(), L->packed_faces ? L->launch_rows.size() * sizeof(int32_t) : 0, &o.launch_rows},
  };
  size_t total = 0;
  for (const Part& p : parts) {
    *p.off = total;
    total += aligned(p.bytes);
  }
  if (total == 0) total = 256;
  try {
    L->static_image.assign(total, 0);
  } catch (const std::bad_alloc&) {
    set_error("out of host memory while packing the device tables");
    return CA_ERR_ALLOC;
  }
  for (const Part& p : parts)
    if (p.bytes && p.src) std::memcpy(L->static_image.data() + *p.off, p.src, p.bytes);
  return CA_OK;
}

// Checks a problem description and allocates a layout with its geometry filled in (no tables yet).
int new_layout(const ca_problem& p, ca_layout** out) {
  if (p.T <= 0 || p.H <= 0 || p.W <= 0) return fail(CA_ERR_INVALID_ARG, "T, H, W must be positive");
  if (p.tt <= 0 || p.th <= 0 || p.tw <= 0) return fail(CA_ERR_INVALID_ARG, "tile dims must be positive");
  if (p.batch <= 0 || p.num_heads <= 0 || p.head_dim <= 0)
    return fail(CA_ERR_INVALID_ARG, "batch, num_heads, head_dim must be positive");
  if (p.dtype != CA_F32 && p.dtype != CA_BF16) return fail(CA_ERR_INVALID_ARG, "unknown dtype");
  if (!(p.scale == p.scale) || std::isinf(p.scale)) return fail(CA_ERR_INVALID_ARG, "scale is not finite");
  const int64_t B = (int64_t)p.tt * p.th * p.tw;
  if (B > (1 << 20)) return fail(CA_ERR_INVALID_ARG, "tile too large");
  if (p.n_text < 0 || p.n_text % B != 0) return fail(CA_ERR_INVALID_ARG, "n_text must be a non-negative multiple of tt*th*tw");
  if (((int64_t)p.head_dim * elem_size(p.dtype)) % 16 != 0)
    return fail(CA_ERR_INVALID_ARG, "head_dim * element size must be a multiple of 16 bytes");
  const int64_t nT = ceil_div(p.T, p.tt), nH = ceil_div(p.H, p.th), nW = ceil_div(p.W, p.tw);
  const int64_t n = nT * nH * nW + p.n_text / B;
  if (n * B >= (int64_t)1 << 31 || (int64_t)p.num_heads * n >= (int64_t)1 << 31)
    return fail(CA_ERR_INVALID_ARG, "problem too large for 32-bit tile/row ids");

  ca_layout* L = new (std::nothrow) ca_layout();
  if (!L) return fail(CA_ERR_ALLOC, "out of host memory");
  L->serial = g_next_serial.fetch_add(1);
  L->prob = p;
  L->nT = (int32_t)nT;
  L->nH = (int32_t)nH;
  L->nW = (int32_t)nW;
  L->B = B;
  L->n_vid = nT * nH * nW;
  L->n_txt = p.n_text / B;
  L->n = n;
  L->N_real = (int64_t)p.T * p.H * p.W + p.n_text;
  L->N_pad = n * B;
  L->scale = p.scale > 0.f ? p.scale : 1.0f / std::sqrt((float)p.head_dim);
  *out = L;
  return CA_OK;
}

}  // namespace

extern "C" {

int compact_attn_build_layout(const ca_problem* problem, const ca_head* heads, ca_layout** out) {
  ca::clear_error();
  if (out) *out = nullptr;
  if (!problem || !heads || !out) return fail(CA_ERR_INVALID_ARG, "null argument");
  ca_layout* L = nullptr;
  int st = new_layout(*problem, &L);
  if (st != CA_OK) return st;
  st = ca::build_host_tables(*L, heads);
  if (st != CA_OK) {
    delete L;
    return st;
  }
  *out = L;
  return CA_OK;
}

int compact_attn_layout_from_csr(const ca_problem* problem, const int64_t* const* row_ptr, const int32_t* const* col_idx,
                                 ca_layout** out) {
  ca::clear_error();
  if (out) *out = nullptr;
  if (!problem || !row_ptr || !col_idx || !out) return fail(CA_ERR_INVALID_ARG, "null argument");
  ca_layout* L = nullptr;
  int st = new_layout(*problem, &L);
  if (st != CA_OK) return st;
  st = ca::import_host_tables(*L, row_ptr, col_idx);
  if (st != CA_OK) {
    delete L;
    return st;
  }
  *out = L;
  return CA_OK;
}

int compact_attn_layout_union(const ca_layout* a, const ca_layout* b, ca_layout** out) {
  ca::clear_error();
  if (out) *out = nullptr;
  if (!a || !b || !out) return fail(CA_ERR_INVALID_ARG, "null argument");
  const ca_problem &pa = a->prob, &pb = b->prob;
  const bool same = pa.T == pb.T && pa.H == pb.H && pa.W == pb.W && pa.tt == pb.tt && pa.th == pb.th && pa.tw == pb.tw &&
                    pa.n_text == pb.n_text && pa.batch == pb.batch && pa.num_heads == pb.num_heads &&
                    pa.head_dim == pb.head_dim && pa.dtype == pb.dtype && a->scale == b->scale;
  if (!same) return fail(CA_ERR_INVALID_ARG, "layouts to merge must describe the same problem");
  ca_layout* L = nullptr;
  int st = new_layout(pa, &L);
  if (st != CA_OK) return st;
  L->scale = a->scale;
  st = ca::union_host_tables(*L, *a, *b);
  if (st != CA_OK) {
    delete L;
    return st;
  }
  *out = L;
  return CA_OK;
}

int compact_attn_layout_similarity(const ca_layout* a, int32_t head_a, const ca_layout* b, int32_t head_b, double* sim) {
  ca::clear_error();
  if (!a || !b || !sim) return fail(CA_ERR_INVALID_ARG, "null argument");
  if (a->n != b->n) return fail(CA_ERR_INVALID_ARG, "layouts must have the same number of tiles");
  if (head_a < 0 || head_a >= a->prob.num_heads || head_b < 0 || head_b >= b->prob.num_heads)
    return fail(CA_ERR_INVALID_ARG, "head out of range");
  *sim = ca::head_similarity(*a, head_a, *b, head_b);
  return CA_OK;
}

int compact_attn_layout_info(const ca_layout* L, int64_t* n_tiles, int64_t* tokens_per_tile, int64_t* n_tokens_real,
                             int64_t* n_tokens_padded, int64_t* nnz_total) {
  ca::clear_error();
  if (!L) return fail(CA_ERR_INVALID_ARG, "null layout");
  if (n_tiles) *n_tiles = L->n;
  if (tokens_per_tile) *tokens_per_tile = L->B;
  if (n_tokens_real) *n_tokens_real = L->N_real;
  if (n_tokens_padded) *n_tokens_padded = L->N_pad;
  if (nnz_total) *nnz_total = (int64_t)L->col_idx.size();
  return CA_OK;
}

int compact_attn_layout_csr(const ca_layout* L, int32_t head, const int64_t** row_ptr, const int32_t** col_idx) {
  ca::clear_error();
  if (!L || !row_ptr || !col_idx) return fail(CA_ERR_INVALID_ARG, "null argument");
  if (head < 0 || head >= L->prob.num_heads) return fail(CA_ERR_INVALID_ARG, "head out of range");
  *row_ptr = L->head_row_ptr[head].data();
  *col_idx = L->col_idx.data() + L->row_ptr[(int64_t)head * L->n];
  return CA_OK;
}

int compact_attn_layout_order(const ca_layout* L, const int32_t** order) {
  ca::clear_error();
  if (!L || !order) return fail(CA_ERR_INVALID_ARG, "null argument");
  *order = L->order.data();
  return CA_OK;
}

int compact_attn_layout_pairs(const ca_layout* L, const int32_t** pairs, int64_t* num_pairs, const int64_t** walk_ptr,
                              const int32_t** walk) {
  ca::clear_error();
  if (!L || !pairs || !num_pairs) return fail(CA_ERR_INVALID_ARG, "null argument");
  *pairs = L->pair_rows.data();
  *num_pairs = (int64_t)L->pair_rows.size() / 2;
  if (walk_ptr) *walk_ptr = L->pair_walk_ptr.data();
  if (walk) *walk = L->pair_walk.data();
  return CA_OK;
}

int compact_attn_layout_packing(const ca_layout* L, const int32_t** desc, const int32_t** launch_rows, int64_t* num_launch_rows) {
  ca::clear_error();
  if (!L || !desc || !launch_rows || !num_launch_rows) return fail(CA_ERR_INVALID_ARG, "null argument");
  *desc = L->pair_desc.data();
  const std::vector<int32_t>& rows = L->packed_faces ? L->launch_rows : L->order;
  const bool all_paired = !L->pair_rows.empty() && !L->packed_faces;
  *launch_rows = all_paired ? nullptr : rows.data();
  *num_launch_rows = all_paired ? 0 : (int64_t)rows.size();
  return CA_OK;
}

int compact_attn_layout_upload(ca_layout* L) {
  ca::clear_error();
  if (!L) return fail(CA_ERR_INVALID_ARG, "null layout");
  return ensure_uploaded(L, nullptr);
}

void compact_attn_free_layout(ca_layout* L) {
  if (!L) return;
  if (L->uploaded) free_device_tables(L->dev);
  delete L;
}

int compact_attn_permute(const void* src, void* dst, ca_layout* L, int32_t inverse, void* stream) {
  ca::clear_error();
  if (!src || !dst || !L) return fail(CA_ERR_INVALID_ARG, "null argument");
  if (!aligned16(src) || !aligned16(dst)) return fail(CA_ERR_INVALID_ARG, "src and dst must be 16-byte aligned");
  if (inverse != 0 && inverse != 1) return fail(CA_ERR_INVALID_ARG, "inverse must be 0 or 1");
  const ca_problem& p = L->prob;
  {
    const int64_t per_token = (int64_t)p.batch * p.num_heads * p.head_dim * elem_size(p.dtype);
    const int64_t natural_bytes = per_token * L->N_real, tiled_bytes = per_token * L->N_pad;
    if (ranges_overlap(src, inverse ? tiled_bytes : natural_bytes, dst, inverse ? natural_bytes : tiled_bytes))
      return fail(CA_ERR_INVALID_ARG, "src and dst must not overlap");
  }
  ca::PermuteArgs a{};
  a.src = src;
  a.dst = dst;
  a.T = p.T; a.H = p.H; a.W = p.W;
  a.tt = p.tt; a.th = p.th; a.tw = p.tw;
  a.nH = L->nH; a.nW = L->nW;
  a.n_vid = L->n_vid;
  a.B = L->B;
  a.N_real = L->N_real;
  a.N_pad = L->N_pad;
  a.N_video = (int64_t)p.T * p.H * p.W;
  a.planes = (int64_t)p.batch * p.num_heads;
  a.row_bytes = p.head_dim * elem_size(p.dtype);
  a.inverse = inverse;
  const hipError_t e = ca::launch_permute(a, (hipStream_t)stream);
  if (e != hipSuccess) return hip_fail(e, "permute launch");
  return CA_OK;
}

int compact_attn_forward(const void* q, const void* k, const void* v, ca_layout* L, void* out, void* stream) {
  return run_attention(q, k, v, L, out, stream, false);
}

int compact_attn_forward_static(const void* q, const void* k, const void* v, ca_layout* L, void* out, void* stream) {
  ca::clear_error();
  int st = check_attention_args(q, k, v, L, out, false);
  if (st != CA_OK) return st;
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return hip_fail(e, "hipGetDevice");
  if (dev < 0 || dev >= kMaxDevices) return fail(CA_ERR_UNSUPPORTED, "device index beyond the static table slots");
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  ScratchState& sc = g_scratch[dev];
  if (!sc.ptr) {
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess || !p) return hip_fail(e, "hipGetSymbolAddress of the static table array");
    sc.ptr = static_cast<unsigned char*>(p);
  }
  st = build_static_image(L);
  if (st != CA_OK) return st;
  if (L->static_image.size() > kScratchBytes) {
    set_error("the layout's tables take %zu bytes, the static device array holds %zu: use compact_attn_forward",
              L->static_image.size(), kScratchBytes);
    return CA_ERR_UNSUPPORTED;
  }
  if (sc.owner != L->serial) {
    // the array holds another layout's tables (or nothing yet): replace them, in stream order
    if (stream) {
      hipStreamCaptureStatus cap = hipStreamCaptureStatusNone;
      e = hipStreamIsCapturing((hipStream_t)stream, &cap);
      if (e != hipSuccess) return hip_fail(e, "hipStreamIsCapturing");
      if (cap != hipStreamCaptureStatusNone) {
        set_error("the static device array does not hold this layout's tables and the stream is being captured: "
                  "make one call with this layout before the capture");
        return CA_ERR_INVALID_ARG;
      }
    }
    e = hipMemcpyAsync(sc.ptr, L->static_image.data(), L->static_image.size(), hipMemcpyHostToDevice, (hipStream_t)stream);
    if (e != hipSuccess) {
      sc.owner = 0;
      return hip_fail(e, "copy of the layout tables into the static device array");
    }
    sc.owner = L->serial;
  }
  const ca_layout::StaticOffsets& o = L->static_off;
  ca::DeviceTables t;
  t.row_ptr = reinterpret_cast<int64_t*>(sc.ptr + o.row_ptr);
  t.col_meta = reinterpret_cast<int32_t*>(sc.ptr + o.col_meta);
  t.order = reinterpret_cast<int32_t*>(sc.ptr + o.order);
  t.num_pairs = (int64_t)L->pair_rows.size() / 2;
  if (t.num_pairs) {
    t.pair_rows = reinterpret_cast<int32_t*>(sc.ptr + o.pair_rows);
    t.pair_walk_ptr = reinterpret_cast<int64_t*>(sc.ptr + o.pair_walk_ptr);
    t.pair_walk = reinterpret_cast<int32_t*>(sc.ptr + o.pair_walk);
  }
  t.tile_class = reinterpret_cast<int32_t*>(sc.ptr + o.tile_class);
  t.class_mask = reinterpret_cast<ca::SlotMask*>(sc.ptr + o.class_mask);
  t.class_perm = sc.ptr + o.class_perm;
  t.pool_counters = reinterpret_cast<int32_t*>(sc.ptr + o.pool_counter);
  t.pool_slots = 1;
  if (t.num_pairs) t.pair_desc = reinterpret_cast<int32_t*>(sc.ptr + o.pair_desc);
  if (L->packed_faces) {
    t.launch_rows = reinterpret_cast<int32_t*>(sc.ptr + o.launch_rows);
    t.num_launch_rows = (int64_t)L->launch_rows.size();
  }
  st = launch_attention(q, k, v, L, t, out, stream, false, false);
  if (st != CA_OK) sc.owner = 0;
  return st;
}

int compact_attn_forward_natural(const void* q, const void* k, const void* v, ca_layout* L, void* out, void* stream) {
  return run_attention(q, k, v, L, out, stream, false, true);
}

int compact_attn_dense(const void* q, const void* k, const void* v, ca_layout* L, void* out, void* stream) {
  return run_attention(q, k, v, L, out, stream, true);
}

int compact_attn_tile_mass(const void* q, const void* k, ca_layout* L, float* mass, void* stream) {
  ca::clear_error();
  if (!q || !k || !L || !mass) return fail(CA_ERR_INVALID_ARG, "null argument");
  if (!aligned16(q) || !aligned16(k)) return fail(CA_ERR_INVALID_ARG, "q and k must be 16-byte aligned");
  const ca_problem& p = L->prob;
  if (p.dtype != CA_BF16 || !((L->B == 64 || L->B == 128) && (p.head_dim == 64 || p.head_dim == 128))) {
    set_error("tile mass supports bf16 with tile sizes 64/128 and head_dim 64/128; got dtype=%d B=%lld D=%d", p.dtype,
              (long long)L->B, p.head_dim);
    return CA_ERR_UNSUPPORTED;
  }
  const int64_t in_bytes = (int64_t)p.batch * p.num_heads * L->N_pad * p.head_dim * 2;
  const int64_t mass_bytes = (int64_t)p.batch * p.num_heads * L->n * L->n * 4;
  if ((reinterpret_cast<uintptr_t>(mass) & 3u) != 0) return fail(CA_ERR_INVALID_ARG, "mass must be 4-byte aligned");
  if (ranges_overlap(mass, mass_bytes, q, in_bytes) || ranges_overlap(mass, mass_bytes, k, in_bytes))
    return fail(CA_ERR_INVALID_ARG, "mass must not overlap q or k");
  int st = ensure_uploaded(L, (hipStream_t)stream);
  if (st == CA_OK) st = ensure_mass_workspace(L, (hipStream_t)stream);
  if (st != CA_OK) return st;
  ca::MassArgs a{};
  a.q = q;
  a.k = k;
  a.mass = mass;
  a.partial = L->dev.mass_partial;
  a.partial_rows = L->dev.mass_partial_rows;
  a.counter = L->dev.mass_counter;
  // 128-token tiles: one launch, every workgroup goes from row to row.  64-token tiles: one launch per
  // set of resident workgroups, so that all of them start a row together and walk the key tiles in
  // step: their steps are short, and once the workgroups of an XCD have drifted apart the tile copies
  // miss its L2 (measured at the 75K-token layout: 94.7 ms in one launch against 84.6 ms).
  a.rows_per_launch = L->B >= 128 ? (int64_t)p.batch * p.num_heads * L->n : L->dev.mass_partial_rows;
  a.dense_meta = L->dev.dense_meta;
  a.tile_class = L->dev.tile_class;
  a.class_mask = L->dev.class_mask;
  a.class_perm = L->dev.class_perm;
  a.batch = p.batch;
  a.num_heads = p.num_heads;
  a.n = L->n;
  a.B = (int32_t)L->B;
  a.D = p.head_dim;
  a.scale = L->scale;
  const hipError_t e = ca::launch_tile_mass(a, (hipStream_t)stream);
  if (e != hipSuccess) return hip_fail(e, "tile mass launch");
  return CA_OK;
}

int compact_attn_search_head(const ca_layout* L, const float* mass, const int32_t* group_max_dt, int32_t num_groups,
                             double tau, double lambda, int32_t pattern, ca_group* groups, double* recall,
                             double* kept_fraction) {
  ca::clear_error();
  if (!L || !mass || !group_max_dt || !groups) return fail(CA_ERR_INVALID_ARG, "null argument");
  if (num_groups < 1 || num_groups > CA_MAX_GROUPS) return fail(CA_ERR_INVALID_ARG, "num_groups must be in 1..CA_MAX_GROUPS");
  for (int32_t g = 0; g < num_groups; ++g)
    if (group_max_dt[g] < 0 || (g > 0 && group_max_dt[g] <= group_max_dt[g - 1]))
      return fail(CA_ERR_INVALID_ARG, "group_max_dt must be non-negative and strictly increasing");
  if (!(tau >= 0.0 && tau <= 1.0) || !(lambda >= 0.0)) return fail(CA_ERR_INVALID_ARG, "tau must lie in [0, 1] and lambda be >= 0");
  if (pattern != CA_PATTERN_CUBIC && pattern != CA_PATTERN_FRAME_GROUPS && pattern != CA_PATTERN_DUAL)
    return fail(CA_ERR_INVALID_ARG, "pattern must be a ca_pattern value");
  try {
    return ca::search_head_windows(*L, mass, group_max_dt, num_groups, tau, lambda, pattern, groups, recall, kept_fraction);
  } catch (const std::bad_alloc&) {
    return fail(CA_ERR_ALLOC, "out of host memory in the window search");
  }
}

const char* compact_attn_last_error(void) { return ca::last_error(); }

}  // extern "C"
