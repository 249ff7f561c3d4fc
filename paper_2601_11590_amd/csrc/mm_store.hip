// Single-node stand-in for the MM Store (paper section 3.2, "Multimodal Cache Pooling" and
// "Fault-Tolerant and Recomputation"): encoded features are kept in a device pool under the
// hash of the multimodal input; a hit returns the stored rows without running the encoder, a
// miss (never stored, or dropped to make room) recomputes them and stores them again.
//
// The paper names neither the hash nor the replacement rule; fixed here:
//   key   two polynomial hashes modulo P = 2^61 - 1 over the input as 32-bit little-endian
//         words (last word zero-padded) behind four header words (byte length low / high, salt
//         low / high):  H_k = sum_j (s_j + 1) R_k^(L - j) mod P.  Every term carries its own
//         power, so the sum can be taken in any order: a thread folds a run of words with
//         Horner's rule, multiplies by the power its run ends at, and the rest is modular
//         addition -- exact integer arithmetic, bit for bit the value a serial evaluation gives.
//   pool  a byte arena behind a 1 MiB scratch area (partial hashes); entries are contiguous,
//         256-byte aligned; insert drops least-recently-used entries until a first-fit range
//         (lowest address) is free; a hit makes its entry the most recent.
// The bookkeeping is host code and touches no device memory; only epd_store_hash and
// epd_encode_cached launch work.
#include "../../include/epd_encode.h"

#include <hip/hip_runtime.h>

#include <cstdarg>
#include <cstdio>
#include <list>
#include <map>
#include <mutex>
#include <string>
#include <vector>

namespace {

constexpr uint64_t kP = (1ull << 61) - 1;
constexpr uint64_t kBase0 = 0x1D4E2C1B3A596877ull % kP, kBase1 = 0x0F1E2D3C4B5A6978ull % kP;
constexpr uint64_t kAlign = 256;
constexpr uint64_t kScratchBytes = 1ull << 20;
constexpr int kRanges = 32;          // ranges per launch (descriptors travel as kernel arguments)
constexpr int kMaxBlocks = 1024;     // blocks per range
constexpr int kThreads = 256;
constexpr int kMinWords = 64;        // words per thread, at least

struct Key {
  uint64_t a, b;
  bool operator<(const Key& o) const { return a != o.a ? a < o.a : b < o.b; }
};
struct Entry { uint64_t off, bytes; std::list<Key>::iterator lru; };

std::string fmt(const char* f, ...) {
  char buf[512];
  va_list ap;
  va_start(ap, f);
  vsnprintf(buf, sizeof buf, f, ap);
  va_end(ap);
  return buf;
}

// ---------------------------------------------------------------- arithmetic modulo 2^61 - 1
__host__ __device__ inline uint64_t addmod(uint64_t a, uint64_t b) {
  uint64_t r = a + b;                 // < 2^62
  return r >= kP ? r - kP : r;
}
__device__ inline uint64_t mulmod(uint64_t a, uint64_t b) {   // a, b < 2^61
  const uint64_t lo = a * b, hi = __umul64hi(a, b);           // 2^64 = 8 (mod P): a b = 8 hi + lo
  uint64_t r = (lo & kP) + ((lo >> 61) | (hi << 3));          // hi < 2^58
  r = (r & kP) + (r >> 61);
  return r >= kP ? r - kP : r;
}
__device__ inline uint64_t powmod(uint64_t r, uint64_t e) {
  uint64_t acc = 1;
  while (e) {
    if (e & 1) acc = mulmod(acc, r);
    r = mulmod(r, r);
    e >>= 1;
  }
  return acc;
}

struct HashRange {
  const uint8_t* data;
  uint64_t bytes, salt;
  uint32_t words;            // ceil(bytes / 4)
  uint32_t words_per_thread; // multiple of kMinWords
  uint32_t blocks;           // blocks that hold words of this range (>= 1)
};
struct HashArgs {
  int n;
  uint64_t* partial;         // [kRanges][kMaxBlocks][2]
  uint64_t* result;          // [kRanges][2]
  HashRange r[kRanges];
};

__device__ inline uint32_t load_word(const uint8_t* p, uint64_t byte0, uint64_t bytes, bool aligned) {
  if (aligned && byte0 + 4 <= bytes) return *(const uint32_t*)(p + byte0);
  uint32_t w = 0;
  for (int i = 0; i < 4; ++i)
    if (byte0 + i < bytes) w |= (uint32_t)p[byte0 + i] << (8 * i);
  return w;
}

// blockIdx.y = range, blockIdx.x = block of that range (blocks past its need leave at once)
__global__ __launch_bounds__(kThreads) void hash_partial_kernel(HashArgs a) {
  const HashRange g = a.r[blockIdx.y];
  if (blockIdx.x >= g.blocks) return;
  const uint64_t L = 4 + (uint64_t)g.words;                 // sequence length: header + data words
  const bool aligned = ((size_t)g.data & 3) == 0;
  const uint64_t w0 = ((uint64_t)blockIdx.x * kThreads + threadIdx.x) * g.words_per_thread;
  const uint64_t w1 = min(w0 + (uint64_t)g.words_per_thread, (uint64_t)g.words);
  uint64_t h0 = 0, h1 = 0;
  if (w0 < w1) {
    for (uint64_t w = w0; w < w1; ++w) {
      const uint64_t v = (uint64_t)load_word(g.data, w * 4, g.bytes, aligned) + 1;
      h0 = mulmod(addmod(h0, v), kBase0);
      h1 = mulmod(addmod(h1, v), kBase1);
    }
    const uint64_t e = L - (4 + w1);                        // the run ends at sequence position 4 + w1
    h0 = mulmod(h0, powmod(kBase0, e));
    h1 = mulmod(h1, powmod(kBase1, e));
  }
  if (blockIdx.x == 0 && threadIdx.x == 0) {
    // header words s_0 .. s_3 sit at powers L .. L - 3
    const uint64_t hdr[4] = {g.bytes & 0xffffffffull, g.bytes >> 32, g.salt & 0xffffffffull, g.salt >> 32};
    uint64_t t0 = 0, t1 = 0;
    for (int j = 0; j < 4; ++j) {
      t0 = mulmod(addmod(t0, hdr[j] + 1), kBase0);
      t1 = mulmod(addmod(t1, hdr[j] + 1), kBase1);
    }
    h0 = addmod(h0, mulmod(t0, powmod(kBase0, L - 4)));
    h1 = addmod(h1, mulmod(t1, powmod(kBase1, L - 4)));
  }
  __shared__ uint64_t s0[kThreads], s1[kThreads];
  s0[threadIdx.x] = h0;
  s1[threadIdx.x] = h1;
  __syncthreads();
  for (int step = kThreads / 2; step > 0; step >>= 1) {
    if ((int)threadIdx.x < step) {
      s0[threadIdx.x] = addmod(s0[threadIdx.x], s0[threadIdx.x + step]);
      s1[threadIdx.x] = addmod(s1[threadIdx.x], s1[threadIdx.x + step]);
    }
    __syncthreads();
  }
  if (threadIdx.x == 0) {
    uint64_t* out = a.partial + ((size_t)blockIdx.y * kMaxBlocks + blockIdx.x) * 2;
    out[0] = s0[0];
    out[1] = s1[0];
  }
}

// one block per range: modular sum of its blocks' partial hashes
__global__ __launch_bounds__(kThreads) void hash_final_kernel(HashArgs a) {
  const HashRange g = a.r[blockIdx.x];
  uint64_t h0 = 0, h1 = 0;
  for (uint32_t b = threadIdx.x; b < g.blocks; b += kThreads) {
    const uint64_t* p = a.partial + ((size_t)blockIdx.x * kMaxBlocks + b) * 2;
    h0 = addmod(h0, p[0]);
    h1 = addmod(h1, p[1]);
  }
  __shared__ uint64_t s0[kThreads], s1[kThreads];
  s0[threadIdx.x] = h0;
  s1[threadIdx.x] = h1;
  __syncthreads();
  for (int step = kThreads / 2; step > 0; step >>= 1) {
    if ((int)threadIdx.x < step) {
      s0[threadIdx.x] = addmod(s0[threadIdx.x], s0[threadIdx.x + step]);
      s1[threadIdx.x] = addmod(s1[threadIdx.x], s1[threadIdx.x + step]);
    }
    __syncthreads();
  }
  if (threadIdx.x == 0) {
    a.result[blockIdx.x * 2] = s0[0];
    a.result[blockIdx.x * 2 + 1] = s1[0];
  }
}

// Partial-hash scratch of epd_store_hash_noalloc: one slot pair per (range, block) of one launch.
// Every GPU the library runs on holds its own copy of this array, at its own address, until the
// process ends.  In host code the name is only a handle for hipGetSymbolAddress -- it is not a
// device address and never goes into a kernel argument or a copy.
constexpr size_t kStaticScratchWords = (size_t)kRanges * kMaxBlocks * 2;
static __device__ __align__(256) uint64_t scratch[kStaticScratchWords];

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
uint64_t* g_scratch_ptr[kMaxDevices] = {};     // device address of `scratch` on each device, once known

}  // namespace

struct epd_store {
  char* pool = nullptr;          // device; [0, kScratchBytes) scratch, entries behind it
  uint64_t arena = 0;            // bytes available to entries (multiple of kAlign)
  std::map<Key, Entry> entries;
  std::map<uint64_t, uint64_t> by_off;     // offset -> rounded size
  std::list<Key> lru;                      // front = least recently used
  uint64_t hits = 0, misses = 0, evictions = 0;
  std::string err;
};

namespace {

thread_local std::string g_store_error = "";

uint64_t round_up(uint64_t n) { return (n + kAlign - 1) / kAlign * kAlign; }

// lowest offset of a free range of `need` bytes, or UINT64_MAX
uint64_t first_fit(const epd_store* s, uint64_t need) {
  uint64_t pos = 0;
  for (const auto& kv : s->by_off) {
    if (kv.first - pos >= need) return pos;
    pos = kv.first + kv.second;
  }
  return s->arena - pos >= need ? pos : UINT64_MAX;
}

void drop(epd_store* s, std::map<Key, Entry>::iterator it) {
  s->by_off.erase(it->second.off);
  s->lru.erase(it->second.lru);
  s->entries.erase(it);
}

}  // namespace

extern "C" {

epd_status epd_store_create(void* device_pool, uint64_t pool_bytes, epd_store_handle* out) {
  if (!out) { g_store_error = "out is NULL"; return EPD_ERR_INVALID_ARG; }
  if (!device_pool || ((uintptr_t)device_pool % kAlign)) {
    g_store_error = "pool is NULL or not 256-byte aligned"; return EPD_ERR_INVALID_ARG;
  }
  if (pool_bytes < kScratchBytes + kAlign) {
    g_store_error = fmt("pool of %llu bytes is smaller than the %llu-byte scratch area plus one entry",
                        (unsigned long long)pool_bytes, (unsigned long long)kScratchBytes);
    return EPD_ERR_WORKSPACE;
  }
  epd_store* s = new epd_store();
  s->pool = (char*)device_pool;
  s->arena = (pool_bytes - kScratchBytes) / kAlign * kAlign;
  *out = s;
  return EPD_OK;
}

epd_status epd_store_destroy(epd_store_handle s) {
  delete s;
  return EPD_OK;
}

const char* epd_store_last_error(epd_store_handle s) { return s ? s->err.c_str() : g_store_error.c_str(); }

epd_status epd_store_lookup(epd_store_handle s, const uint64_t key[2], void** device_ptr, uint64_t* bytes) {
  if (!s) { g_store_error = "store is NULL"; return EPD_ERR_INVALID_ARG; }
  if (!key || !device_ptr) { s->err = "a required pointer is NULL"; return EPD_ERR_INVALID_ARG; }
  auto it = s->entries.find(Key{key[0], key[1]});
  if (it == s->entries.end()) { ++s->misses; *device_ptr = nullptr; if (bytes) *bytes = 0; return EPD_MISS; }
  ++s->hits;
  s->lru.splice(s->lru.end(), s->lru, it->second.lru);       // most recent at the back
  *device_ptr = s->pool + kScratchBytes + it->second.off;
  if (bytes) *bytes = it->second.bytes;
  return EPD_OK;
}

epd_status epd_store_insert(epd_store_handle s, const uint64_t key[2], uint64_t bytes, void** device_ptr) {
  if (!s) { g_store_error = "store is NULL"; return EPD_ERR_INVALID_ARG; }
  if (!key || !device_ptr) { s->err = "a required pointer is NULL"; return EPD_ERR_INVALID_ARG; }
  const uint64_t need = round_up(bytes);
  if (bytes == 0 || need > s->arena) {
    s->err = fmt("an entry of %llu bytes can never fit a pool of %llu", (unsigned long long)bytes,
                 (unsigned long long)s->arena);
    *device_ptr = nullptr;
    return EPD_ERR_WORKSPACE;
  }
  const Key k{key[0], key[1]};
  auto old = s->entries.find(k);
  if (old != s->entries.end()) drop(s, old);
  uint64_t off;
  while ((off = first_fit(s, need)) == UINT64_MAX) {
    drop(s, s->entries.find(s->lru.front()));
    ++s->evictions;
  }
  s->lru.push_back(k);
  s->entries[k] = Entry{off, bytes, std::prev(s->lru.end())};
  s->by_off[off] = need;
  *device_ptr = s->pool + kScratchBytes + off;
  return EPD_OK;
}

epd_status epd_store_stats(epd_store_handle s, uint64_t* hits, uint64_t* misses, uint64_t* evictions, uint64_t* entries) {
  if (!s) { g_store_error = "store is NULL"; return EPD_ERR_INVALID_ARG; }
  if (hits) *hits = s->hits;
  if (misses) *misses = s->misses;
  if (evictions) *evictions = s->evictions;
  if (entries) *entries = s->entries.size();
  return EPD_OK;
}

// Describes ranges [i0, i0 + m) in `a` and launches the two hash kernels for them: partial hashes
// go to a.partial, the m keys to a.result (both set by the caller).
static void launch_hash(HashArgs& a, const void* device_data, const uint64_t* offsets, const uint64_t* salts, int i0, int m,
                        hipStream_t st) {
  uint32_t max_blocks = 1;
  for (int j = 0; j < m; ++j) {
    HashRange& r = a.r[j];
    r.data = (const uint8_t*)device_data + offsets[i0 + j];
    r.bytes = offsets[i0 + j + 1] - offsets[i0 + j];
    r.salt = salts[i0 + j];
    r.words = (uint32_t)((r.bytes + 3) / 4);
    const uint64_t per_thread = ((uint64_t)r.words + (uint64_t)kMaxBlocks * kThreads - 1) / ((uint64_t)kMaxBlocks * kThreads);
    r.words_per_thread = (uint32_t)((per_thread + kMinWords - 1) / kMinWords * kMinWords);
    if (r.words_per_thread == 0) r.words_per_thread = kMinWords;
    const uint64_t per_block = (uint64_t)r.words_per_thread * kThreads;
    r.blocks = (uint32_t)(((uint64_t)r.words + per_block - 1) / per_block);
    if (r.blocks == 0) r.blocks = 1;
    if (r.blocks > max_blocks) max_blocks = r.blocks;
  }
  a.n = m;
  hipLaunchKernelGGL(hash_partial_kernel, dim3(max_blocks, m), dim3(kThreads), 0, st, a);
  hipLaunchKernelGGL(hash_final_kernel, dim3(m), dim3(kThreads), 0, st, a);
}

static bool ranges_ok(const uint64_t* offsets, int n, std::string& err) {
  for (int i = 0; i < n; ++i)
    if (offsets[i + 1] < offsets[i] || offsets[i + 1] - offsets[i] >= (1ull << 33)) {
      err = fmt("range %d: offsets must not decrease and a range holds less than 8 GiB", i);
      return false;
    }
  return true;
}

epd_status epd_store_hash(epd_store_handle s, const void* device_data, const uint64_t* offsets, const uint64_t* salts,
                          int32_t n, uint64_t* keys_out, void* stream) {
  if (!s) { g_store_error = "store is NULL"; return EPD_ERR_INVALID_ARG; }
  if (!device_data || !offsets || !salts || !keys_out || n <= 0) {
    s->err = "a required pointer is NULL or n <= 0"; return EPD_ERR_INVALID_ARG;
  }
  if (!ranges_ok(offsets, n, s->err)) return EPD_ERR_SHAPE;
  hipStream_t st = (hipStream_t)stream;
  HashArgs a{};
  a.partial = (uint64_t*)s->pool;
  a.result = a.partial + (size_t)kRanges * kMaxBlocks * 2;
  static_assert(((size_t)kRanges * kMaxBlocks * 2 + kRanges * 2) * 8 <= kScratchBytes, "hash scratch");
  for (int i0 = 0; i0 < n; i0 += kRanges) {
    const int m = n - i0 < kRanges ? n - i0 : kRanges;
    launch_hash(a, device_data, offsets, salts, i0, m, st);
    hipError_t e = hipMemcpyAsync(keys_out + (size_t)i0 * 2, a.result, (size_t)m * 16, hipMemcpyDeviceToHost, st);
    if (e == hipSuccess) e = hipStreamSynchronize(st);      // the keys decide what is launched next
    if (e != hipSuccess) { s->err = fmt("hash launch or copy failed: %s", hipGetErrorString(e)); return EPD_ERR_HIP; }
  }
  return EPD_OK;
}

// The same keys for callers that cannot allocate: the partial hashes go to the library's own
// static device array instead of a pool, the keys to a device buffer of the caller, and the host
// is not waited for.  Nothing here allocates or frees memory (device or pinned), copies, or
// synchronises; the two launches are all the GPU work.
epd_status epd_store_hash_noalloc(const void* device_data, const uint64_t* offsets, const uint64_t* salts, int32_t n,
                                  uint64_t* keys_device_out, void* stream) {
  if (!device_data || !offsets || !salts || !keys_device_out || n <= 0) {
    g_store_error = "a required pointer is NULL or n <= 0"; return EPD_ERR_INVALID_ARG;
  }
  if (n > kRanges) {
    g_store_error = fmt("%d ranges: one call of epd_store_hash_noalloc takes at most %d (its scratch array holds that many)", n, kRanges);
    return EPD_ERR_SHAPE;
  }
  if (!ranges_ok(offsets, n, g_store_error)) return EPD_ERR_SHAPE;
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess || dev < 0 || dev >= kMaxDevices) {
    g_store_error = fmt("no usable current device (%s, device %d)", hipGetErrorString(e), dev); return EPD_ERR_HIP;
  }
  uint64_t* ptr;
  {
    // first call on this device: ask the runtime where this device keeps its copy of the array
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
      void* p = nullptr;
      e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
      if (e != hipSuccess || !p) {
        g_store_error = fmt("hipGetSymbolAddress(scratch) failed on device %d: %s", dev, hipGetErrorString(e)); return EPD_ERR_HIP;
      }
      g_scratch_ptr[dev] = (uint64_t*)p;
    }
    ptr = g_scratch_ptr[dev];
  }
  // Nothing in the array has to start at zero: the first kernel writes the slot of every block the
  // second one reads, so the previous call's contents are simply overwritten.
  HashArgs a{};
  a.partial = ptr;
  a.result = keys_device_out;
  launch_hash(a, device_data, offsets, salts, 0, n, (hipStream_t)stream);
  e = hipGetLastError();
  if (e != hipSuccess) { g_store_error = fmt("hash launch failed: %s", hipGetErrorString(e)); return EPD_ERR_HIP; }
  return EPD_OK;
}

}  // extern "C"
