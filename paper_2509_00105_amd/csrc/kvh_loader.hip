// Load path: stored blobs in pinned host memory -> device staging slots -> decode, with the copy of
// chunk i + 1 overlapping the decode of chunk i (the paper charges a stored entry size / Bandwidth
// of loading delay plus its decompression overhead; Design section, utility and estimator).  Host
// side only: two HIP streams and a ring of events around the existing decode kernel.
#include <new>

#include "kvh_common.hpp"

struct kvh_loader {
  uint8_t* staging;
  size_t slot_bytes;
  int n_slots;
  int device;
  hipStream_t copy_stream;
  hipEvent_t* copied;  // [slot] the slot's blob has arrived
  hipEvent_t* freed;   // [slot] the decode that read the slot has been enqueued and will have finished
  bool* in_use;        // [slot] `freed` has been recorded at least once
};

namespace kvh {
namespace {

constexpr int kMaxSlots = 64;

void destroy(kvh_loader* ld) {
  if (ld == nullptr) return;
  if (ld->copy_stream != nullptr) (void)hipStreamDestroy(ld->copy_stream);
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
  const size_t slot_bytes = (staging_bytes / (size_t)n_slots) & ~size_t(15);
  if (slot_bytes < (size_t)kHeaderBytes) return KVH_E_SIZE;
  kvh_loader* ld = new (std::nothrow) kvh_loader{};
  if (ld == nullptr) return KVH_E_HIP;
  ld->staging = static_cast<uint8_t*>(staging_dev);
  ld->slot_bytes = slot_bytes;
  ld->n_slots = n_slots;
  ld->copied = new (std::nothrow) hipEvent_t[n_slots]();
  ld->freed = new (std::nothrow) hipEvent_t[n_slots]();
  ld->in_use = new (std::nothrow) bool[n_slots]();
  bool ok = ld->copied != nullptr && ld->freed != nullptr && ld->in_use != nullptr;
  ok = ok && hipGetDevice(&ld->device) == hipSuccess;
  // default priority; non-blocking so that the legacy default stream does not serialise the copies
  ok = ok && hipStreamCreateWithFlags(&ld->copy_stream, hipStreamNonBlocking) == hipSuccess;
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
  if (ld == nullptr || items == nullptr || n_items < 1 || (dt != KVH_F16 && dt != KVH_BF16)) return KVH_E_ARG;
  if (dst == nullptr || dst->k == nullptr || dst->v == nullptr || dst->layer_stride < 0 || dst->token_stride < 0)
    return KVH_E_ARG;
  if (((reinterpret_cast<uintptr_t>(dst->k) | reinterpret_cast<uintptr_t>(dst->v)) & 15u) != 0 ||
      dst->layer_stride % 8 != 0 || dst->token_stride % 8 != 0)
    return KVH_E_ALIGN;
  // validate every item before anything is enqueued
  for (int i = 0; i < n_items; ++i) {
    const kvh_load_item& it = items[i];
    if (it.blob_host == nullptr || it.dst_token0 < 0) return KVH_E_ARG;
    if (level_bits(it.level) < 0) return KVH_E_LEVEL;
    const size_t need = kvh_blob_size(l, it.n_tokens, c, it.level);
    if (need == 0) return KVH_E_SHAPE;
    if (need > ld->slot_bytes) return KVH_E_SIZE;
    if (it.page_table != nullptr && block_tokens < 1) return KVH_E_ARG;
    if (it.dst_token0 + it.n_tokens > INT32_MAX) return KVH_E_ARG;
  }
  hipStream_t compute = static_cast<hipStream_t>(stream);
  DecodeParams a{};
  a.items = nullptr;
  a.k = static_cast<uint16_t*>(dst->k);
  a.v = static_cast<uint16_t*>(dst->v);
  a.layer_stride = dst->layer_stride;
  a.token_stride = dst->token_stride;
  a.l = l;
  a.c = c;
  a.split = kNoSplit;
  for (int i = 0; i < n_items; ++i) {
    const kvh_load_item& it = items[i];
    const int s = i % ld->n_slots;
    uint8_t* slot = ld->staging + (size_t)s * ld->slot_bytes;
    const size_t bytes = kvh_blob_size(l, it.n_tokens, c, it.level);
    // the slot may still be read by the decode that used it last (in this run or the previous one)
    if (ld->in_use[s] && hipStreamWaitEvent(ld->copy_stream, ld->freed[s], 0) != hipSuccess) return KVH_E_HIP;
    if (hipMemcpyAsync(slot, it.blob_host, bytes, hipMemcpyHostToDevice, ld->copy_stream) != hipSuccess) return KVH_E_HIP;
    if (hipEventRecord(ld->copied[s], ld->copy_stream) != hipSuccess) return KVH_E_HIP;
    if (hipStreamWaitEvent(compute, ld->copied[s], 0) != hipSuccess) return KVH_E_HIP;
    a.one = kvh_item{slot, it.n_tokens, it.level, it.dst_token0, it.page_table};
    a.status = status_dev != nullptr ? status_dev + i : nullptr;
    a.block_tokens = it.page_table != nullptr ? block_tokens : 1;
    if (int rc = launch_decode(a, dt, 1, it.n_tokens, compute)) return rc;
    if (hipEventRecord(ld->freed[s], compute) != hipSuccess) return KVH_E_HIP;
    ld->in_use[s] = true;
  }
  return KVH_OK;
}

}  // extern "C"
