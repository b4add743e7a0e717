// On-demand residency of expert weights (MoQE Section 4.4 and the appendix on memory: only the
// selected expert's weights sit in device memory, the others wait in host memory and are copied in
// when the router switches to them).  A cache of `slots` equal device buffers holds the most
// recently used of K blobs; a miss copies the blob host -> device on the caller's stream, which
// also orders the copy behind every kernel that still reads the evicted blob.
#include "moqe_internal.h"

#include <vector>
#include <new>

struct moqe_expert_cache {
  int K = 0, slots = 0;
  size_t slot_bytes = 0;
  std::vector<const void*> host;
  std::vector<size_t> bytes;
  std::vector<int> slot_of;        // expert -> slot or -1
  std::vector<int> expert_in;      // slot -> expert or -1
  std::vector<uint64_t> last_use;  // slot -> tick of last acquire
  uint64_t tick = 0;
  uint8_t* dev = nullptr;
  uint64_t copies = 0, copied_bytes = 0;
};

using namespace moqe;

extern "C" {

int32_t moqe_cache_create(moqe_expert_cache** out, const void* const* host_blobs, const size_t* bytes, int32_t K,
                          int32_t slots) {
  if (!out || !host_blobs || !bytes) return set_error(MOQE_E_NULL, "moqe_cache_create: NULL argument");
  if (K < 1 || slots < 1 || slots > K) return set_error(MOQE_E_SHAPE, "moqe_cache_create: K=%d slots=%d", K, slots);
  size_t mx = 0;
  for (int e = 0; e < K; ++e) {
    if (!host_blobs[e] || bytes[e] == 0) return set_error(MOQE_E_NULL, "moqe_cache_create: blob %d is empty", e);
    mx = bytes[e] > mx ? bytes[e] : mx;
  }
  if (dry_run()) { *out = nullptr; return MOQE_OK; }
  moqe_expert_cache* c = new (std::nothrow) moqe_expert_cache;
  if (!c) return set_error(MOQE_E_WORKSPACE, "moqe_cache_create: out of host memory");
  c->K = K; c->slots = slots; c->slot_bytes = align256(mx);
  c->host.assign(host_blobs, host_blobs + K);
  c->bytes.assign(bytes, bytes + K);
  c->slot_of.assign(K, -1);
  c->expert_in.assign(slots, -1);
  c->last_use.assign(slots, 0);
  const size_t total = c->slot_bytes * size_t(slots);
  hipError_t err = hipMalloc(reinterpret_cast<void**>(&c->dev), total);
  if (err != hipSuccess) {
    delete c;
    return set_error(MOQE_E_HIP, "moqe_cache_create: %zu bytes of device memory: %s", total, hipGetErrorString(err));
  }
  *out = c;
  return MOQE_OK;
}

int32_t moqe_cache_destroy(moqe_expert_cache* c) {
  if (!c) return MOQE_OK;
  hipError_t err = hipFree(c->dev);
  delete c;
  if (err != hipSuccess) return set_error(MOQE_E_HIP, "moqe_cache_destroy: %s", hipGetErrorString(err));
  return MOQE_OK;
}

int32_t moqe_cache_acquire(moqe_expert_cache* c, const int32_t* want, int32_t n, void** dev_ptrs, int32_t* copied,
                           void* stream) {
  if (!c || !want || !dev_ptrs) return set_error(MOQE_E_NULL, "moqe_cache_acquire: NULL argument");
  if (n < 0 || n > c->slots) return set_error(MOQE_E_SHAPE, "moqe_cache_acquire: %d blobs wanted, %d slots", n, c->slots);
  for (int i = 0; i < n; ++i) {
    if (want[i] < 0 || want[i] >= c->K) return set_error(MOQE_E_SHAPE, "moqe_cache_acquire: blob %d outside [0, %d)", want[i], c->K);
    for (int j = 0; j < i; ++j)
      if (want[j] == want[i]) return set_error(MOQE_E_SHAPE, "moqe_cache_acquire: blob %d wanted twice", want[i]);
  }
  const uint64_t now = ++c->tick;
  int ncopied = 0;
  // first pass: hits keep their slots (and must not be evicted for this call's misses)
  for (int i = 0; i < n; ++i)
    if (c->slot_of[want[i]] >= 0) c->last_use[c->slot_of[want[i]]] = now;
  for (int i = 0; i < n; ++i) {
    const int e = want[i];
    int s = c->slot_of[e];
    if (s < 0) {
      s = 0;                                           // least recently used slot (empty slots have tick 0)
      for (int t = 1; t < c->slots; ++t)
        if (c->last_use[t] < c->last_use[s]) s = t;
      if (c->expert_in[s] >= 0) c->slot_of[c->expert_in[s]] = -1;
      hipError_t err = hipMemcpyAsync(c->dev + size_t(s) * c->slot_bytes, c->host[e], c->bytes[e], hipMemcpyHostToDevice,
                                      static_cast<hipStream_t>(stream));
      if (err != hipSuccess) {
        c->expert_in[s] = -1;
        return set_error(MOQE_E_HIP, "moqe_cache_acquire: copy of blob %d: %s", e, hipGetErrorString(err));
      }
      c->expert_in[s] = e;
      c->slot_of[e] = s;
      c->last_use[s] = now;
      c->copies += 1; c->copied_bytes += c->bytes[e];
      ++ncopied;
    }
    dev_ptrs[i] = c->dev + size_t(s) * c->slot_bytes;
  }
  if (copied) *copied = ncopied;
  return MOQE_OK;
}

int32_t moqe_cache_stats(const moqe_expert_cache* c, uint64_t* copies, uint64_t* copied_bytes) {
  if (!c) return set_error(MOQE_E_NULL, "moqe_cache_stats: cache is NULL");
  if (copies) *copies = c->copies;
  if (copied_bytes) *copied_bytes = c->copied_bytes;
  return MOQE_OK;
}

}  // extern "C"
