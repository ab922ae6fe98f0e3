// Content-addressed store of launch tables (per-unit descriptors and work lists).
//
// A table is uploaded the first time its contents are seen and keeps its device
// address until the store is destroyed: kernels that were queued earlier, and HIP
// graphs captured earlier, go on reading the address they were given, so storage
// that has been handed out is never moved, overwritten or reused.  When a chunk
// is full another one is chained behind it; chunks are released together at the
// end.  Growth is bounded by a total limit.
//
// The memory back end is a template parameter, so that the bookkeeping can be
// exercised on the host without a device (the unit test plugs in malloc).
//   struct Backend {
//     bool alloc(size_t bytes, uint8_t** dev, uint8_t** host);   // one chunk: device memory + host mirror
//     void release(uint8_t* dev, uint8_t* host);
//     bool upload(uint8_t* dev, const uint8_t* host, size_t bytes, void* stream);  // asynchronous on stream
//     bool may_alloc(void* stream);                              // false while `stream` is being captured
//   };
#pragma once

#include <stddef.h>
#include <stdint.h>
#include <string.h>

#include <unordered_map>
#include <vector>

namespace hack {

enum class TableStatus { kOk, kTooLarge, kFullDuringCapture, kLimit, kAllocFailed, kUploadFailed };

template <typename Backend>
class TableCache {
 public:
  TableCache(Backend backend, size_t chunk_bytes, size_t limit_bytes)
      : be_(backend), chunk_bytes_(chunk_bytes), limit_bytes_(limit_bytes) {}
  TableCache(const TableCache&) = delete;
  TableCache& operator=(const TableCache&) = delete;
  ~TableCache() {
    for (Chunk& c : chunks_) be_.release(c.dev, c.host);
  }

  // Device address of a table with exactly these bytes.
  TableStatus get(const uint8_t* bytes, size_t n, void* stream, const uint8_t** dev) {
    const uint64_t h = fnv1a(bytes, n);
    auto range = index_.equal_range(h);
    for (auto it = range.first; it != range.second; ++it) {
      const Entry& e = it->second;
      if (e.bytes == n && memcmp(chunks_[e.chunk].host + e.offset, bytes, n) == 0) {
        *dev = chunks_[e.chunk].dev + e.offset;
        return TableStatus::kOk;
      }
    }
    const size_t need = (n + kAlign - 1) / kAlign * kAlign;
    if (need > chunk_bytes_) return TableStatus::kTooLarge;
    if (chunks_.empty() || chunks_.back().used + need > chunk_bytes_) {
      if (!be_.may_alloc(stream)) return TableStatus::kFullDuringCapture;
      if ((chunks_.size() + 1) * chunk_bytes_ > limit_bytes_) return TableStatus::kLimit;
      Chunk c{};
      if (!be_.alloc(chunk_bytes_, &c.dev, &c.host)) return TableStatus::kAllocFailed;
      chunks_.push_back(c);
    }
    Chunk& c = chunks_.back();
    const size_t off = c.used;
    memcpy(c.host + off, bytes, n);
    if (!be_.upload(c.dev + off, c.host + off, n, stream)) return TableStatus::kUploadFailed;
    c.used += need;
    index_.emplace(h, Entry{chunks_.size() - 1, off, n});
    *dev = c.dev + off;
    return TableStatus::kOk;
  }

  // Allocates the first chunk ahead of time (so that a first table seen during a
  // stream capture still finds room).  Returns false if the allocation failed.
  bool reserve_first_chunk() {
    if (!chunks_.empty()) return true;
    Chunk c{};
    if (!be_.alloc(chunk_bytes_, &c.dev, &c.host)) return false;
    chunks_.push_back(c);
    return true;
  }

  size_t chunks() const { return chunks_.size(); }
  size_t tables() const { return index_.size(); }

 private:
  static constexpr size_t kAlign = 256;
  struct Chunk {
    uint8_t* dev;
    uint8_t* host;
    size_t used;
  };
  struct Entry {
    size_t chunk, offset, bytes;
  };
  static uint64_t fnv1a(const uint8_t* p, size_t n) {
    uint64_t h = 1469598103934665603ull;
    for (size_t i = 0; i < n; ++i) {
      h ^= p[i];
      h *= 1099511628211ull;
    }
    return h;
  }

  Backend be_;
  size_t chunk_bytes_, limit_bytes_;
  std::vector<Chunk> chunks_;
  std::unordered_multimap<uint64_t, Entry> index_;
};

}  // namespace hack
