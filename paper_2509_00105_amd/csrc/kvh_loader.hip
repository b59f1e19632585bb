// Load path: stored blobs in pinned host memory -> device staging slots -> decode, with the copy of
// group g + 1 overlapping the decode of group g (the paper charges a stored entry size / Bandwidth
// of loading delay plus its decompression overhead; Design section, utility and estimator).
//
// Consecutive blobs are packed into groups that fill one staging slot.  A group is moved by ONE
// launch of a small copy kernel that reads the pinned host memory over the bus (the blobs of a
// group need not be contiguous on the host) and also writes the group's decode descriptors at the
// head of the slot, then decoded by ONE batched decode launch.  Per-blob runtime copies were
// measured to leave 30-60 us of idle bus between two copies on this platform; with groups the
// fixed costs are paid once per slot.  Two streams (copy, caller's compute) and two events per slot
// order the ring; one more event orders a run's copies after what the caller's stream already holds.
#include <mutex>
#include <new>

#include "kvh_common.hpp"

namespace kvh {
namespace {

constexpr int kMaxSlots = 64;
constexpr int kMaxGroup = 32;                                   // blobs per group
constexpr size_t kDescBytes = (size_t)kMaxGroup * sizeof(kvh_kept_item);  // descriptor area at the head of a slot
#ifndef KVH_LD_BLOCKS
#define KVH_LD_BLOCKS 4   // copy blocks per blob (the bus, not the CUs, bounds the copy: few blocks leave the rest to the decode)
#endif
#ifndef KVH_LD_UNROLL
#define KVH_LD_UNROLL 4   // 16-byte loads in flight per thread
#endif
constexpr int kCopyThreads = 256;
constexpr int kCopyBlocksPerBlob = KVH_LD_BLOCKS;
constexpr int kCopyUnroll = KVH_LD_UNROLL;

typedef uint32_t uintx4 __attribute__((ext_vector_type(4)));

struct CopyGroup {
  int n;
  const uint8_t* src[kMaxGroup];  // pinned host memory, device-visible
  uint64_t off[kMaxGroup];        // byte offset of the blob inside the slot
  uint64_t n16[kMaxGroup];        // blob size in 16-byte words
  kvh_kept_item item[kMaxGroup];  // decode descriptor (blob = slot + off)
};

// grid = (kCopyBlocksPerBlob, blobs of the group)
__global__ __launch_bounds__(kCopyThreads) void load_group_kernel(CopyGroup g, uint8_t* slot) {
  const int j = blockIdx.y;
  const uintx4* src = reinterpret_cast<const uintx4*>(g.src[j]);
  uintx4* dst = reinterpret_cast<uintx4*>(slot + g.off[j]);
  const uint64_t n16 = g.n16[j];
  if (blockIdx.x == 0 && threadIdx.x < sizeof(kvh_kept_item) / 4) {
    const uint32_t* d = reinterpret_cast<const uint32_t*>(&g.item[j]);
    reinterpret_cast<uint32_t*>(slot)[j * (sizeof(kvh_kept_item) / 4) + threadIdx.x] = d[threadIdx.x];
  }
  const uint64_t stride = (uint64_t)gridDim.x * kCopyThreads;
  for (uint64_t i = (uint64_t)blockIdx.x * kCopyThreads + threadIdx.x; i < n16; i += stride * kCopyUnroll) {
    uintx4 r[kCopyUnroll];
#pragma unroll
    for (int u = 0; u < kCopyUnroll; ++u)
      if (i + u * stride < n16) r[u] = __builtin_nontemporal_load(src + i + u * stride);
#pragma unroll
    for (int u = 0; u < kCopyUnroll; ++u)
      if (i + u * stride < n16) dst[i + u * stride] = r[u];
  }
}


// Everything kvh_loader_run and kvh_load_static check before they enqueue anything.  `capacity` = bytes a slot
// offers to blobs.
int validate_load(const kvh_load_item* items, int n_items, kvh_dtype dt, int l, int c, const kvh_kv_view* dst,
                  int block_tokens, size_t capacity) {
  if (items == nullptr || n_items < 1 || (dt != KVH_F16 && dt != KVH_BF16) || block_tokens < 1) return KVH_E_ARG;
  if (dst == nullptr || dst->k == nullptr || dst->v == nullptr || dst->layer_stride < 0 || dst->token_stride < c)
    return KVH_E_ARG;
  if (((reinterpret_cast<uintptr_t>(dst->k) | reinterpret_cast<uintptr_t>(dst->v)) & 15u) != 0 ||
      dst->layer_stride % 8 != 0 || dst->token_stride % 8 != 0)
    return KVH_E_ALIGN;
  for (int i = 0; i < n_items; ++i) {
    const kvh_load_item& it = items[i];
    if (it.blob_host == nullptr || it.dst_token0 < 0) return KVH_E_ARG;
    if ((reinterpret_cast<uintptr_t>(it.blob_host) & 15u) != 0) return KVH_E_ALIGN;
    if (level_bits(it.level) < 0) return KVH_E_LEVEL;
    const size_t need = kvh_blob_size(l, it.n_tokens, c, it.level);
    if (need == 0) return KVH_E_SHAPE;
    if (need > capacity) return KVH_E_SIZE;
    // the copy kernel reads the blob in place: both ends must lie in host memory the device can see
    const uint8_t* ends[2] = {static_cast<const uint8_t*>(it.blob_host), static_cast<const uint8_t*>(it.blob_host) + need - 1};
    for (const uint8_t* p : ends) {
      hipPointerAttribute_t at{};
      if (hipPointerGetAttributes(&at, p) != hipSuccess || at.type != hipMemoryTypeHost) {
        (void)hipGetLastError();
        return KVH_E_ARG;
      }
    }
    if ((it.orig_tokens | it.sink | it.window) != 0) {  // a token-dropped blob: n_tokens is what is kept
      if (kvh_kept_tokens(it.orig_tokens, it.sink, it.window) != it.n_tokens) return KVH_E_SHAPE;
    }
    const int64_t span = (it.orig_tokens > it.n_tokens && !it.compact) ? it.orig_tokens : it.n_tokens;
    if (it.dst_token0 + span > INT32_MAX) return KVH_E_ARG;
  }
  return KVH_OK;
}

// Pack consecutive blobs, starting at items[first], into one slot of `capacity` bytes for blobs; returns how many
// went in (at least one: every blob has been checked against the capacity) and their largest token count.
int pack_group(const kvh_load_item* items, int first, int n_items, int l, int c, uint8_t* slot, size_t capacity,
               CopyGroup& g, int& max_tokens) {
  size_t used = 0;
  max_tokens = 0;
  g.n = 0;
  while (first + g.n < n_items && g.n < kMaxGroup) {
    const kvh_load_item& it = items[first + g.n];
    const size_t bytes = kvh_blob_size(l, it.n_tokens, c, it.level);
    if (used + bytes > capacity) break;
    g.src[g.n] = static_cast<const uint8_t*>(it.blob_host);
    g.off[g.n] = kDescBytes + used;
    g.n16[g.n] = bytes / 16;
    g.item[g.n] = kvh_kept_item{slot + kDescBytes + used, it.n_tokens, it.level, it.dst_token0, it.page_table,
                                it.orig_tokens, it.sink, it.window, it.compact};
    if (it.n_tokens > max_tokens) max_tokens = it.n_tokens;
    used += bytes;
    ++g.n;
  }
  return g.n;
}

// ---- the allocation-free variant: its one staging slot lives in the code object -------------------------
// Each device the library runs on holds its own copy of this array, at its own address, until the process ends.
// In host code the name is only a handle for hipGetSymbolAddress; the address kernels and copies use is the one
// that call returns, looked up once per device.
static __device__ __align__(256) uint8_t scratch[KVH_STATIC_SCRATCH_BYTES];
static_assert(KVH_STATIC_SCRATCH_BYTES % 256 == 0 && KVH_STATIC_SCRATCH_BYTES > kDescBytes + kHeaderBytes, "scratch size");

constexpr int kMaxDevices = 64;
std::mutex scratch_mutex;
uint8_t* scratch_ptr[kMaxDevices];  // per device: address of `scratch` there, nullptr until first use

// Address of the current device's scratch array (nullptr on failure).
uint8_t* scratch_on_current_device() {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
  std::lock_guard<std::mutex> lock(scratch_mutex);
  if (scratch_ptr[dev] == nullptr) {
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || p == nullptr) {
      (void)hipGetLastError();
      return nullptr;
    }
    scratch_ptr[dev] = static_cast<uint8_t*>(p);
  }
  return scratch_ptr[dev];
}

}  // namespace
}  // namespace kvh

struct kvh_loader {
  uint8_t* staging;
  size_t slot_bytes;  // capacity of a slot for blobs (the descriptor area is extra)
  size_t slot_pitch;
  int n_slots;
  int next_slot;
  hipStream_t copy_stream;
  hipEvent_t* copied;  // [slot] the slot's group has arrived
  hipEvent_t* freed;   // [slot] the decode that read the slot has finished
  hipEvent_t entered;  // the caller's stream at the start of a run
  bool* in_use;        // [slot] `freed` has been recorded at least once
};

namespace kvh {
namespace {

void destroy(kvh_loader* ld) {
  if (ld == nullptr) return;
  if (ld->copy_stream != nullptr) (void)hipStreamDestroy(ld->copy_stream);
  if (ld->entered != nullptr) (void)hipEventDestroy(ld->entered);
  for (int s = 0; s < ld->n_slots; ++s) {
    if (ld->copied != nullptr && ld->copied[s] != nullptr) (void)hipEventDestroy(ld->copied[s]);
    if (ld->freed != nullptr && ld->freed[s] != nullptr) (void)hipEventDestroy(ld->freed[s]);
  }
  delete[] ld->copied;
  delete[] ld->freed;
  delete[] ld->in_use;
  delete ld;
}

}  // namespace
}  // namespace kvh

using namespace kvh;

extern "C" {

int kvh_loader_create(kvh_loader** out, void* staging_dev, size_t staging_bytes, int n_slots) {
  if (out == nullptr) return KVH_E_ARG;
  *out = nullptr;
  if (staging_dev == nullptr || n_slots < 1 || n_slots > kMaxSlots) return KVH_E_ARG;
  if ((reinterpret_cast<uintptr_t>(staging_dev) & 15u) != 0) return KVH_E_ALIGN;
  const size_t pitch = (staging_bytes / (size_t)n_slots) & ~size_t(15);
  if (pitch < kDescBytes + (size_t)kHeaderBytes) return KVH_E_SIZE;
  kvh_loader* ld = new (std::nothrow) kvh_loader{};
  if (ld == nullptr) return KVH_E_HIP;
  ld->staging = static_cast<uint8_t*>(staging_dev);
  ld->slot_pitch = pitch;
  ld->slot_bytes = pitch - kDescBytes;
  ld->n_slots = n_slots;
  ld->copied = new (std::nothrow) hipEvent_t[n_slots]();
  ld->freed = new (std::nothrow) hipEvent_t[n_slots]();
  ld->in_use = new (std::nothrow) bool[n_slots]();
  bool ok = ld->copied != nullptr && ld->freed != nullptr && ld->in_use != nullptr;
  // default priority; non-blocking so that the legacy default stream does not serialise the copies
  ok = ok && hipStreamCreateWithFlags(&ld->copy_stream, hipStreamNonBlocking) == hipSuccess;
  ok = ok && hipEventCreateWithFlags(&ld->entered, hipEventDisableTiming) == hipSuccess;
  for (int s = 0; ok && s < n_slots; ++s) {
    ok = hipEventCreateWithFlags(&ld->copied[s], hipEventDisableTiming) == hipSuccess &&
         hipEventCreateWithFlags(&ld->freed[s], hipEventDisableTiming) == hipSuccess;
  }
  if (!ok) {
    destroy(ld);
    return KVH_E_HIP;
  }
  *out = ld;
  return KVH_OK;
}

int kvh_loader_destroy(kvh_loader* ld) {
  if (ld == nullptr) return KVH_E_ARG;
  // the copies enqueued by this loader must not outlive its stream
  const bool ok = hipStreamSynchronize(ld->copy_stream) == hipSuccess;
  destroy(ld);
  return ok ? KVH_OK : KVH_E_HIP;
}

size_t kvh_loader_slot_bytes(const kvh_loader* ld) { return ld == nullptr ? 0 : ld->slot_bytes; }

int kvh_loader_run(kvh_loader* ld, const kvh_load_item* items, int n_items, kvh_dtype dt, int l, int c,
                   const kvh_kv_view* dst, int block_tokens, int32_t* status_dev, void* stream) {
  if (ld == nullptr) return KVH_E_ARG;
  if (int rc = validate_load(items, n_items, dt, l, c, dst, block_tokens, ld->slot_bytes)) return rc;
  hipStream_t compute = static_cast<hipStream_t>(stream);
  // Stream order: the copies read host blobs that work already enqueued on the caller's stream may
  // still be writing (an encode straight into pinned memory), so they start after that work.
  if (hipEventRecord(ld->entered, compute) != hipSuccess || hipStreamWaitEvent(ld->copy_stream, ld->entered, 0) != hipSuccess)
    return KVH_E_HIP;
  DecodeParams a{};
  a.k = static_cast<uint16_t*>(dst->k);
  a.v = static_cast<uint16_t*>(dst->v);
  a.layer_stride = dst->layer_stride;
  a.token_stride = dst->token_stride;
  a.l = l;
  a.c = c;
  a.block_tokens = block_tokens;
  a.split = kNoSplit;
  int first = 0;
  while (first < n_items) {
    const int s = ld->next_slot;
    uint8_t* slot = ld->staging + (size_t)s * ld->slot_pitch;
    CopyGroup g{};
    int max_tokens = 0;
    pack_group(items, first, n_items, l, c, slot, ld->slot_bytes, g, max_tokens);
    // the slot may still be read by the decode that used it last (in this run or an earlier one)
    if (ld->in_use[s] && hipStreamWaitEvent(ld->copy_stream, ld->freed[s], 0) != hipSuccess) return KVH_E_HIP;
    hipLaunchKernelGGL(load_group_kernel, dim3(kCopyBlocksPerBlob, (unsigned)g.n), dim3(kCopyThreads), 0,
                       ld->copy_stream, g, slot);
    KVH_HIP_CHECK_LAUNCH();
    if (hipEventRecord(ld->copied[s], ld->copy_stream) != hipSuccess) return KVH_E_HIP;
    if (hipStreamWaitEvent(compute, ld->copied[s], 0) != hipSuccess) return KVH_E_HIP;
    a.kept_items = reinterpret_cast<const kvh_kept_item*>(slot);
    a.status = status_dev != nullptr ? status_dev + first : nullptr;
    if (int rc = launch_decode(a, dt, g.n, max_tokens, compute)) return rc;
    if (hipEventRecord(ld->freed[s], compute) != hipSuccess) return KVH_E_HIP;
    ld->in_use[s] = true;
    ld->next_slot = (s + 1) % ld->n_slots;
    first += g.n;
  }
  return KVH_OK;
}

int kvh_load_static(const kvh_load_item* items, int n_items, kvh_dtype dt, int l, int c, const kvh_kv_view* dst,
                    int block_tokens, int32_t* status_dev, void* stream) {
  constexpr size_t capacity = (size_t)KVH_STATIC_SCRATCH_BYTES - kDescBytes;
  if (int rc = validate_load(items, n_items, dt, l, c, dst, block_tokens, capacity)) return rc;
  uint8_t* slot = scratch_on_current_device();
  if (slot == nullptr) return KVH_E_HIP;
  hipStream_t compute = static_cast<hipStream_t>(stream);
  DecodeParams a{};
  a.k = static_cast<uint16_t*>(dst->k);
  a.v = static_cast<uint16_t*>(dst->v);
  a.layer_stride = dst->layer_stride;
  a.token_stride = dst->token_stride;
  a.l = l;
  a.c = c;
  a.block_tokens = block_tokens;
  a.split = kNoSplit;
  // One slot, one stream: copy group, decode group, copy the next group over it.  Stream order keeps a copy from
  // overtaking the decode that still reads the slot; nothing in the slot has to start at zero (the copy kernel
  // rewrites the descriptors of every group).
  for (int first = 0; first < n_items;) {
    CopyGroup g{};
    int max_tokens = 0;
    pack_group(items, first, n_items, l, c, slot, capacity, g, max_tokens);
    hipLaunchKernelGGL(load_group_kernel, dim3(kCopyBlocksPerBlob, (unsigned)g.n), dim3(kCopyThreads), 0, compute, g,
                       slot);
    KVH_HIP_CHECK_LAUNCH();
    a.kept_items = reinterpret_cast<const kvh_kept_item*>(slot);
    a.status = status_dev != nullptr ? status_dev + first : nullptr;
    if (int rc = launch_decode(a, dt, g.n, max_tokens, compute)) return rc;
    first += g.n;
  }
  return KVH_OK;
}

}  // extern "C"
