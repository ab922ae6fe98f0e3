// Host-only check of the launch-table store (csrc/table_cache.h) with a malloc
// back end: tables that were handed out keep their address and their contents
// when the store grows past a chunk, identical contents are found again, growth
// stops at the limit, and nothing grows while a "capture" is in progress.
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

#include "../../paper_2504_09261_amd/csrc/table_cache.h"

struct HostBackend {
  int* live;
  bool* capturing;
  bool alloc(size_t bytes, uint8_t** dev, uint8_t** host) {
    *dev = static_cast<uint8_t*>(malloc(bytes));
    *host = static_cast<uint8_t*>(malloc(bytes));
    ++*live;
    return *dev && *host;
  }
  void release(uint8_t* dev, uint8_t* host) {
    free(dev);
    free(host);
    --*live;
  }
  bool upload(uint8_t* dev, const uint8_t* host, size_t bytes, void*) {
    memcpy(dev, host, bytes);
    return true;
  }
  bool may_alloc(void*) { return !*capturing; }
};

#define CHECK(c)                                              \
  do {                                                        \
    if (!(c)) {                                               \
      printf("FAILED line %d: %s\n", __LINE__, #c);           \
      return 1;                                               \
    }                                                         \
  } while (0)

static std::vector<uint8_t> table(int id, size_t n) {
  std::vector<uint8_t> t(n);
  for (size_t i = 0; i < n; ++i) t[i] = (uint8_t)((id * 131 + i * 7) & 0xFF);
  memcpy(t.data(), &id, sizeof id);
  return t;
}

int main() {
  int live = 0;
  bool capturing = false;
  {
    const size_t chunk = 4096, limit = 4 * 4096;
    hack::TableCache<HostBackend> tc(HostBackend{&live, &capturing}, chunk, limit);
    CHECK(tc.reserve_first_chunk() && tc.chunks() == 1);
    std::vector<const uint8_t*> addr;
    std::vector<std::vector<uint8_t>> data;
    // 1000-byte tables take 1024 bytes each: four per chunk, so the 13th does not fit three chunks
    for (int id = 0; id < 12; ++id) {
      data.push_back(table(id, 1000));
      const uint8_t* d = nullptr;
      CHECK(tc.get(data.back().data(), 1000, nullptr, &d) == hack::TableStatus::kOk);
      addr.push_back(d);
      // every table handed out so far still sits where it was, unchanged
      for (int j = 0; j <= id; ++j) CHECK(memcmp(addr[j], data[j].data(), 1000) == 0);
    }
    CHECK(tc.chunks() == 3 && tc.tables() == 12);
    // the same contents again: same address, nothing new stored
    for (int id = 0; id < 12; ++id) {
      const uint8_t* d = nullptr;
      CHECK(tc.get(data[id].data(), 1000, nullptr, &d) == hack::TableStatus::kOk && d == addr[id]);
    }
    CHECK(tc.tables() == 12);
    // same length, other contents: a different table
    auto other = table(3, 1000);
    other[999] ^= 1;
    const uint8_t* d = nullptr;
    CHECK(tc.get(other.data(), 1000, nullptr, &d) == hack::TableStatus::kOk && d != addr[3]);
    CHECK(tc.chunks() == 4);
    // a full chunk cannot be followed by a new one during a capture ...
    for (int id = 100; id < 103; ++id) {
      auto t = table(id, 1000);
      CHECK(tc.get(t.data(), 1000, nullptr, &d) == hack::TableStatus::kOk);
    }
    capturing = true;
    auto t = table(200, 1000);
    CHECK(tc.get(t.data(), 1000, nullptr, &d) == hack::TableStatus::kFullDuringCapture);
    // ... while known tables are still served
    CHECK(tc.get(data[0].data(), 1000, nullptr, &d) == hack::TableStatus::kOk && d == addr[0]);
    capturing = false;
    // the limit of four chunks is reached; a table larger than a chunk never fits
    CHECK(tc.get(t.data(), 1000, nullptr, &d) == hack::TableStatus::kLimit);
    auto big = table(300, 5000);
    CHECK(tc.get(big.data(), 5000, nullptr, &d) == hack::TableStatus::kTooLarge);
    for (int j = 0; j < 12; ++j) CHECK(memcmp(addr[j], data[j].data(), 1000) == 0);
    CHECK(live == 4);
  }
  CHECK(live == 0);   // every chunk released with the store
  printf("ok\n");
  return 0;
}
