// Host-side runtime of libspc: error reporting, the device block cache, packing
// descriptors and coordinate-level bookkeeping.
#include <algorithm>
#include <cstring>
#include <map>
#include <unordered_map>
#include <utility>
#include <vector>

#include "spc_internal.h"

namespace spc {

static thread_local char g_err[512] = "";

int set_error(int code, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
  return code;
}

// ---------------------------------------------------------------- block cache
// Freed blocks are kept for reuse, binned by rounded size AND by the stream whose work
// last touched them: a block is handed out again only to work enqueued on that same
// stream, so stream order alone guarantees that the previous user has finished (blocks
// are returned right after the kernels that use them were enqueued, not after they ran).
namespace {
struct Pool {
  std::mutex mu;
  std::map<std::pair<size_t, hipStream_t>, std::vector<void*>> free_blocks;
  std::unordered_map<void*, size_t> live;  // block -> rounded size
};
Pool& pool() {
  static Pool* p = new Pool;  // never destroyed: device memory is reclaimed by the driver at exit
  return *p;
}
size_t round_size(size_t b) {
  if (b < 4096) return 4096;
  if (b < (size_t(1) << 20)) {  // next power of two below 1 MiB
    size_t r = 4096;
    while (r < b) r <<= 1;
    return r;
  }
  const size_t g = size_t(1) << 20;  // 1 MiB granules above
  return (b + g - 1) / g * g;
}
}  // namespace

void* pool_alloc(size_t bytes, hipStream_t stream) {
  const size_t r = round_size(bytes);
  Pool& P = pool();
  {
    std::lock_guard<std::mutex> lk(P.mu);
    auto it = P.free_blocks.find({r, stream});
    if (it != P.free_blocks.end() && !it->second.empty()) {
      void* p = it->second.back();
      it->second.pop_back();
      P.live[p] = r;
      return p;
    }
  }
  void* p = nullptr;
  hipError_t e = hipMalloc(&p, r);
  if (e != hipSuccess) {
    (void)hipGetLastError();
    pool_release_all();
    e = hipMalloc(&p, r);
  }
  if (e != hipSuccess) {
    set_error(SPC_ERR_NOMEM, "hipMalloc(%zu) failed: %s", r, hipGetErrorString(e));
    return nullptr;
  }
  std::lock_guard<std::mutex> lk(P.mu);
  P.live[p] = r;
  return p;
}

void pool_free(void* p, hipStream_t stream) {
  if (!p) return;
  Pool& P = pool();
  std::lock_guard<std::mutex> lk(P.mu);
  auto it = P.live.find(p);
  if (it == P.live.end()) return;
  P.free_blocks[{it->second, stream}].push_back(p);
  P.live.erase(it);
}

void order_stream_after(hipStream_t waiter, hipStream_t producer) {
  if (waiter == producer) return;
  hipEvent_t e = nullptr;
  if (hipEventCreateWithFlags(&e, hipEventDisableTiming) != hipSuccess) {
    (void)hipGetLastError();
    (void)hipStreamSynchronize(producer);  // no event to be had: wait on the host instead
    return;
  }
  if (hipEventRecord(e, producer) != hipSuccess || hipStreamWaitEvent(waiter, e, 0) != hipSuccess) {
    (void)hipGetLastError();
    (void)hipStreamSynchronize(producer);
  }
  (void)hipEventDestroy(e);  // released once the record has completed
}

int pool_release_all() {
  Pool& P = pool();
  std::vector<void*> blocks;
  {
    std::lock_guard<std::mutex> lk(P.mu);
    for (auto& kv : P.free_blocks)
      for (void* b : kv.second) blocks.push_back(b);
    P.free_blocks.clear();
  }
  if (!blocks.empty()) (void)hipDeviceSynchronize();
  for (void* b : blocks) (void)hipFree(b);
  return SPC_OK;
}

// ---------------------------------------------------------------- descriptors
int check_desc(const spc_pack_desc* d, PackInfo* pi) {
  if (!d) return set_error(SPC_ERR_ARG, "pack descriptor is NULL");
  if (d->key_bits != 32 && d->key_bits != 64) return set_error(SPC_ERR_ARG, "key_bits must be 32 or 64");
  const int b[4] = {d->bits_b, d->bits_x, d->bits_y, d->bits_z};
  int sum = 0;
  for (int i = 0; i < 4; ++i) {
    if (b[i] < 0 || b[i] > 31) return set_error(SPC_ERR_ARG, "field width %d out of [0,31]", b[i]);
    sum += b[i];
  }
  if (d->bits_x < 1 || d->bits_y < 1 || d->bits_z < 1) return set_error(SPC_ERR_ARG, "spatial fields need >= 1 bit");
  if (sum > d->key_bits) return set_error(SPC_ERR_ARG, "fields need %d bits, key has %d", sum, d->key_bits);
  if (d->pad < 0) return set_error(SPC_ERR_ARG, "pad must be >= 0");
  pi->key_bits = d->key_bits;
  pi->bits_b = d->bits_b;
  pi->bits_x = d->bits_x;
  pi->bits_y = d->bits_y;
  pi->bits_z = d->bits_z;
  pi->sh_y = d->bits_z;
  pi->sh_x = d->bits_z + d->bits_y;
  pi->sh_b = d->bits_z + d->bits_y + d->bits_x;
  pi->used_bits = sum;
  return SPC_OK;
}

uint64_t level_mask(const PackInfo& pi, int m) {
  auto field = [&](int bits) -> uint64_t {
    uint64_t all = (bits >= 64) ? ~uint64_t(0) : ((uint64_t(1) << bits) - 1);
    uint64_t low = (m >= bits) ? all : ((uint64_t(1) << m) - 1);
    return all & ~low;
  };
  uint64_t mask = 0;
  mask |= ((pi.bits_b ? ((uint64_t(1) << pi.bits_b) - 1) : 0) << pi.sh_b);
  mask |= field(pi.bits_x) << pi.sh_x;
  mask |= field(pi.bits_y) << pi.sh_y;
  mask |= field(pi.bits_z);
  return mask;
}

bool stream_is_capturing(hipStream_t s) {
  hipStreamCaptureStatus st = hipStreamCaptureStatusNone;
  if (hipStreamIsCapturing(s, &st) != hipSuccess) {
    (void)hipGetLastError();
    return false;
  }
  return st != hipStreamCaptureStatusNone;
}

void level_unref(Level* l) {
  if (!l) return;
  if (l->refs.fetch_sub(1) == 1) {
    // the blocks go back to the producing stream's cache: that stream must not reuse them before the
    // searches that read the keys on other streams have finished
    if (l->owns_keys || l->n_dev)
      for (hipStream_t r : l->readers) order_stream_after(l->stream, r);
    if (l->owns_keys) pool_free(l->keys, l->stream);
    pool_free(l->n_dev, l->stream);
    if (l->ready) (void)hipEventDestroy(l->ready);
    delete l;
  }
}

}  // namespace spc

extern "C" {

const char* spc_last_error(void) { return spc::g_err; }
const char* spc_version(void) { return "spc-gfx950 0.1"; }
int spc_release_cache(void) { return spc::pool_release_all(); }

static int ceil_log2(int64_t v) {  // smallest b with 2^b >= v
  int b = 0;
  while ((int64_t(1) << b) < v) ++b;
  return b;
}

int spc_pack_desc_fit(const int32_t lo[3], const int32_t hi[3], int32_t n_batch, int32_t max_stride,
                      int32_t max_reach, int32_t key_bits, spc_pack_desc* out) {
  if (!lo || !hi || !out) return spc::set_error(SPC_ERR_ARG, "NULL argument");
  if (n_batch < 1 || max_stride < 1 || (max_stride & (max_stride - 1)) || max_reach < 0)
    return spc::set_error(SPC_ERR_ARG, "n_batch >= 1, max_stride a power of two, max_reach >= 0 required");
  if (key_bits != 0 && key_bits != 32 && key_bits != 64) return spc::set_error(SPC_ERR_ARG, "key_bits must be 0, 32 or 64");
  const int64_t S = max_stride;
  const int64_t pad = (int64_t(max_reach) + S - 1) / S * S;
  int bits[3];
  for (int a = 0; a < 3; ++a) {
    if (hi[a] < lo[a]) return spc::set_error(SPC_ERR_ARG, "hi < lo on axis %d", a);
    int64_t l = lo[a];
    int64_t org = (l >= 0 ? l / S : -((-l + S - 1) / S)) * S;  // floor to a multiple of S
    out->origin[a] = static_cast<int32_t>(org);
    bits[a] = std::max(1, ceil_log2(int64_t(hi[a]) - org + 2 * pad + 1));
    if (bits[a] > 31) return spc::set_error(SPC_ERR_RANGE, "axis %d needs %d bits", a, bits[a]);
  }
  out->bits_b = ceil_log2(n_batch);
  out->bits_x = bits[0];
  out->bits_y = bits[1];
  out->bits_z = bits[2];
  out->pad = static_cast<int32_t>(pad);
  const int sum = out->bits_b + bits[0] + bits[1] + bits[2];
  if (sum > 64 || (key_bits == 32 && sum > 32)) return spc::set_error(SPC_ERR_RANGE, "coordinates need %d key bits", sum);
  out->key_bits = key_bits ? key_bits : (sum <= 32 ? 32 : 64);
  return SPC_OK;
}

}  // extern "C"
