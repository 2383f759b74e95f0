// Host data path: sharded dataset with an index map, batches formed under the max-tokens cap, a
// reproducible shuffle per epoch, and a background thread that assembles the next batches while the
// current one trains, reading instances through a least-recently-used cache
// (sections "Dataset and Dataloader", "Forward Pass", "Prefetch and Cache").  No device work.
#include <fcntl.h>
#include <sys/stat.h>
#include <unistd.h>

#include <algorithm>
#include <condition_variable>
#include <cstdio>
#include <cstring>
#include <list>
#include <mutex>
#include <string>
#include <thread>
#include <unordered_map>
#include <vector>

#include "common.h"

namespace {

const char kShardMagic[8] = {'H', 'S', 'S', 'H', 'A', 'R', 'D', '1'};

// Philox4x32-10 on the host (same published definition as the device version in common.h)
void philox_host(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3, uint32_t k0, uint32_t k1, uint32_t out[4]) {
  for (int round = 0; round < 10; ++round) {
    const uint64_t p0 = (uint64_t)0xD2511F53u * c0, p1 = (uint64_t)0xCD9E8D57u * c2;
    const uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0, n1 = (uint32_t)p1, n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1, n3 = (uint32_t)p0;
    c0 = n0; c1 = n1; c2 = n2; c3 = n3;
    k0 += 0x9E3779B9u; k1 += 0xBB67AE85u;
  }
  out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

struct Shard {
  std::string path;
  int fd = -1;
  int64_t n_seq = 0, n_tok = 0, first = 0;     // `first`: global index of the shard's first instance
  std::vector<int64_t> tok_off;                // token offset of every instance inside the shard (n_seq + 1 entries)
  int64_t data_pos = 0;                        // file position of the token array
};

struct Batch { int32_t pad_len; std::vector<int64_t> inst; };
struct Ready { std::vector<int32_t> ids, lens; std::vector<int64_t> inst; int32_t B = 0, L = 0; };

}  // namespace

struct hs_dataset {
  std::vector<Shard> shards;
  std::vector<int32_t> lengths;                // of all instances, in global order
  int64_t cache_cap = 0;
  int prefetch = 2;
  // least-recently-used cache of instances (touched by the worker thread only)
  std::list<int64_t> lru;
  std::unordered_map<int64_t, std::pair<std::list<int64_t>::iterator, std::vector<int32_t>>> cache;
  int64_t loads = 0, hits = 0;             // worker thread only
  int64_t pub_loads = 0, pub_hits = 0;     // published with every finished batch (under mu)
  // epoch state
  std::vector<Batch> batches;                  // this worker's batches, in order
  std::vector<Ready> ring;
  int64_t produced = 0, consumed = 0;
  bool stop = false, failed = false;
  std::string fail_msg;
  std::thread worker;
  std::mutex mu;
  std::condition_variable cv;
};

namespace {

bool read_exact(int fd, void* dst, size_t n, int64_t pos) {
  char* p = (char*)dst;
  while (n > 0) {
    const ssize_t r = pread(fd, p, n, pos);
    if (r <= 0) return false;
    p += r; n -= (size_t)r; pos += r;
  }
  return true;
}

// tokens of one instance, through the cache
bool fetch(hs_dataset* d, int64_t inst, const int32_t** tok, std::vector<int32_t>* tmp) {
  if (d->cache_cap > 0) {
    auto it = d->cache.find(inst);
    if (it != d->cache.end()) {
      d->lru.splice(d->lru.end(), d->lru, it->second.first);
      ++d->hits;
      *tok = it->second.second.data();
      return true;
    }
  }
  size_t s = (size_t)(std::upper_bound(d->shards.begin(), d->shards.end(), inst, [](int64_t v, const Shard& sh) { return v < sh.first; }) -
                      d->shards.begin()) - 1;
  const Shard& sh = d->shards[s];
  const int64_t row = inst - sh.first, n = sh.tok_off[row + 1] - sh.tok_off[row];
  std::vector<int32_t> buf((size_t)n);
  if (n > 0 && !read_exact(sh.fd, buf.data(), (size_t)n * 4, sh.data_pos + sh.tok_off[row] * 4)) return false;
  ++d->loads;
  if (d->cache_cap > 0) {
    d->lru.push_back(inst);
    auto ins = d->cache.emplace(inst, std::make_pair(std::prev(d->lru.end()), std::move(buf)));
    *tok = ins.first->second.second.data();
    if ((int64_t)d->cache.size() > d->cache_cap) {
      const int64_t victim = d->lru.front();
      d->lru.pop_front();
      d->cache.erase(victim);
    }
  } else {
    *tmp = std::move(buf);
    *tok = tmp->data();
  }
  return true;
}

void worker_main(hs_dataset* d) {
  const int64_t nb = (int64_t)d->batches.size();
  for (int64_t k = 0; k < nb; ++k) {
    {
      std::unique_lock<std::mutex> lk(d->mu);
      d->cv.wait(lk, [&] { return d->stop || k - d->consumed < (int64_t)d->ring.size(); });
      if (d->stop) return;
    }
    const Batch& b = d->batches[(size_t)k];
    Ready& r = d->ring[(size_t)(k % (int64_t)d->ring.size())];
    r.B = (int32_t)b.inst.size(); r.L = b.pad_len; r.inst = b.inst;
    r.ids.assign((size_t)r.B * r.L, 0);            // PAD = 0
    r.lens.resize((size_t)r.B);
    bool ok = true;
    std::vector<int32_t> tmp;
    for (int32_t i = 0; i < r.B && ok; ++i) {
      const int32_t* tok = nullptr;
      ok = fetch(d, b.inst[(size_t)i], &tok, &tmp);
      const int32_t n = d->lengths[(size_t)b.inst[(size_t)i]];
      r.lens[(size_t)i] = n;
      if (ok && n > 0) memcpy(&r.ids[(size_t)i * r.L], tok, (size_t)n * 4);
    }
    std::lock_guard<std::mutex> lk(d->mu);
    if (!ok) { d->failed = true; d->fail_msg = "dataset: read error"; d->cv.notify_all(); return; }
    d->produced = k + 1;
    d->pub_loads = d->loads; d->pub_hits = d->hits;
    d->cv.notify_all();
  }
}

void stop_worker(hs_dataset* d) {
  if (d->worker.joinable()) {
    { std::lock_guard<std::mutex> lk(d->mu); d->stop = true; }
    d->cv.notify_all();
    d->worker.join();
  }
  d->stop = false;
}

}  // namespace

extern "C" {

hs_status hs_shard_write(const char* path, const int32_t* lengths, int64_t n_seq, const int32_t* tokens) {
  if (!path || n_seq < 0 || (n_seq > 0 && !lengths)) return hs_fail(nullptr, HS_ERR_INVALID_ARG, "hs_shard_write: bad argument");
  int64_t n_tok = 0;
  for (int64_t i = 0; i < n_seq; ++i) {
    if (lengths[i] < 0) return hs_fail(nullptr, HS_ERR_INVALID_ARG, "hs_shard_write: negative length");
    n_tok += lengths[i];
  }
  if (n_tok > 0 && !tokens) return hs_fail(nullptr, HS_ERR_INVALID_ARG, "hs_shard_write: tokens is NULL");
  FILE* f = fopen(path, "wb");
  if (!f) return hs_fail(nullptr, HS_ERR_STATE, std::string("hs_shard_write: cannot create ") + path);
  bool ok = fwrite(kShardMagic, 1, 8, f) == 8 && fwrite(&n_seq, 8, 1, f) == 1 && fwrite(&n_tok, 8, 1, f) == 1 &&
            (n_seq == 0 || fwrite(lengths, 4, (size_t)n_seq, f) == (size_t)n_seq) && (n_tok == 0 || fwrite(tokens, 4, (size_t)n_tok, f) == (size_t)n_tok);
  ok = (fclose(f) == 0) && ok;
  if (!ok) return hs_fail(nullptr, HS_ERR_STATE, std::string("hs_shard_write: could not write ") + path);
  return HS_OK;
}

hs_status hs_dataset_close(hs_dataset* d) {
  if (!d) return HS_OK;
  stop_worker(d);
  for (Shard& s : d->shards) if (s.fd >= 0) close(s.fd);
  delete d;
  return HS_OK;
}

hs_status hs_dataset_open(const char* const* paths, int32_t n_shards, int64_t cache_instances, int32_t prefetch_batches, hs_dataset** out) {
  if (!out) return hs_fail(nullptr, HS_ERR_INVALID_ARG, "hs_dataset_open: out is NULL");
  *out = nullptr;
  if (!paths || n_shards < 1 || cache_instances < 0 || prefetch_batches < 1 || prefetch_batches > 64)
    return hs_fail(nullptr, HS_ERR_INVALID_ARG, "hs_dataset_open: need >= 1 shard, cache >= 0, 1 <= prefetch <= 64");
  hs_dataset* d = new hs_dataset();
  d->cache_cap = cache_instances;
  d->prefetch = prefetch_batches;
  int64_t first = 0;
  for (int32_t s = 0; s < n_shards; ++s) {
    Shard sh;
    sh.path = paths[s] ? paths[s] : "";
    sh.fd = open(sh.path.c_str(), O_RDONLY);
    char magic[8];
    int64_t hdr[2];
    if (sh.fd < 0 || !read_exact(sh.fd, magic, 8, 0) || memcmp(magic, kShardMagic, 8) != 0 || !read_exact(sh.fd, hdr, 16, 8) || hdr[0] < 0 || hdr[1] < 0) {
      if (sh.fd >= 0) close(sh.fd);
      hs_dataset_close(d);
      return hs_fail(nullptr, HS_ERR_STATE, "hs_dataset_open: cannot read shard " + sh.path);
    }
    sh.n_seq = hdr[0]; sh.n_tok = hdr[1]; sh.first = first;
    std::vector<int32_t> len((size_t)sh.n_seq);
    struct stat st;
    const int64_t want = 24 + 4 * sh.n_seq + 4 * sh.n_tok;
    if ((sh.n_seq > 0 && !read_exact(sh.fd, len.data(), (size_t)sh.n_seq * 4, 24)) || fstat(sh.fd, &st) != 0 || (int64_t)st.st_size != want) {
      close(sh.fd);
      hs_dataset_close(d);
      return hs_fail(nullptr, HS_ERR_STATE, "hs_dataset_open: truncated shard " + sh.path);
    }
    sh.tok_off.resize((size_t)sh.n_seq + 1);
    sh.tok_off[0] = 0;
    for (int64_t i = 0; i < sh.n_seq; ++i) {
      if (len[(size_t)i] < 0) { close(sh.fd); hs_dataset_close(d); return hs_fail(nullptr, HS_ERR_STATE, "hs_dataset_open: negative length in " + sh.path); }
      sh.tok_off[(size_t)i + 1] = sh.tok_off[(size_t)i] + len[(size_t)i];
    }
    if (sh.tok_off[(size_t)sh.n_seq] != sh.n_tok) { close(sh.fd); hs_dataset_close(d); return hs_fail(nullptr, HS_ERR_STATE, "hs_dataset_open: lengths do not add up in " + sh.path); }
    sh.data_pos = 24 + 4 * sh.n_seq;
    d->lengths.insert(d->lengths.end(), len.begin(), len.end());
    first += sh.n_seq;
    d->shards.push_back(std::move(sh));
  }
  *out = d;
  return HS_OK;
}

int64_t hs_dataset_size(const hs_dataset* d) { return d ? (int64_t)d->lengths.size() : 0; }

hs_status hs_dataset_lengths(const hs_dataset* d, int32_t* out) {
  if (!d || !out) return hs_fail(nullptr, HS_ERR_INVALID_ARG, "hs_dataset_lengths: NULL argument");
  memcpy(out, d->lengths.data(), d->lengths.size() * 4);
  return HS_OK;
}

hs_status hs_dataset_locate(const hs_dataset* d, int64_t instance, int32_t* shard_out, int64_t* row_out) {
  if (!d || !shard_out || !row_out || instance < 0 || instance >= (int64_t)d->lengths.size())
    return hs_fail(nullptr, HS_ERR_INVALID_ARG, "hs_dataset_locate: bad argument");
  const size_t s = (size_t)(std::upper_bound(d->shards.begin(), d->shards.end(), instance, [](int64_t v, const Shard& sh) { return v < sh.first; }) -
                            d->shards.begin()) - 1;
  *shard_out = (int32_t)s; *row_out = instance - d->shards[s].first;
  return HS_OK;
}

hs_status hs_dataset_begin_epoch(hs_dataset* d, uint64_t seed, int64_t epoch, int32_t bucket_width, int64_t max_tokens, int32_t cap_mode,
                                 int32_t world, int32_t rank, int64_t* n_batches_out) {
  if (!d || !n_batches_out) return hs_fail(nullptr, HS_ERR_INVALID_ARG, "hs_dataset_begin_epoch: NULL argument");
  *n_batches_out = 0;
  if (world < 1 || rank < 0 || rank >= world || epoch < 0) return hs_fail(nullptr, HS_ERR_INVALID_ARG, "hs_dataset_begin_epoch: bad world/rank/epoch");
  stop_worker(d);
  const int64_t n = (int64_t)d->lengths.size();
  std::vector<int32_t> seq_index((size_t)n), pads((size_t)n);
  std::vector<int64_t> offs((size_t)n + 1);
  int64_t nb = 0;
  hs_status st = hs_make_batches(d->lengths.data(), n, bucket_width, max_tokens, cap_mode, seq_index.data(), offs.data(), pads.data(), &nb);
  if (st != HS_OK) return st;
  // Fisher-Yates driven by the generator: for i = nb-1 .. 1 swap i with word 0 of block (i, epoch, tag) mod (i + 1)
  std::vector<int64_t> order((size_t)nb);
  for (int64_t i = 0; i < nb; ++i) order[(size_t)i] = i;
  for (int64_t i = nb - 1; i >= 1; --i) {
    uint32_t w[4];
    philox_host((uint32_t)i, (uint32_t)((uint64_t)i >> 32), (uint32_t)epoch, 0x5AFF1Eu, (uint32_t)seed, (uint32_t)(seed >> 32), w);
    const int64_t j = (int64_t)(w[0] % (uint64_t)(i + 1));
    std::swap(order[(size_t)i], order[(size_t)j]);
  }
  d->batches.clear();
  for (int64_t k = rank; k < nb; k += world) {
    const int64_t b = order[(size_t)k];
    Batch bt;
    bt.pad_len = pads[(size_t)b];
    for (int64_t q = offs[(size_t)b]; q < offs[(size_t)b + 1]; ++q) bt.inst.push_back(seq_index[(size_t)q]);
    d->batches.push_back(std::move(bt));
  }
  d->ring.assign((size_t)d->prefetch, Ready());
  d->produced = d->consumed = 0;
  d->failed = false;
  *n_batches_out = (int64_t)d->batches.size();
  d->worker = std::thread(worker_main, d);
  return HS_OK;
}

hs_status hs_dataset_peek(hs_dataset* d, int32_t* B_out, int32_t* L_out) {
  if (!d || !B_out || !L_out) return hs_fail(nullptr, HS_ERR_INVALID_ARG, "hs_dataset_peek: NULL argument");
  *B_out = *L_out = 0;
  if (d->consumed >= (int64_t)d->batches.size()) return HS_OK;      // end of the epoch
  const Batch& b = d->batches[(size_t)d->consumed];
  *B_out = (int32_t)b.inst.size(); *L_out = b.pad_len;
  return HS_OK;
}

hs_status hs_dataset_next(hs_dataset* d, int32_t* ids_out, int32_t* lens_out, int64_t* instance_out) {
  if (!d || !ids_out || !lens_out) return hs_fail(nullptr, HS_ERR_INVALID_ARG, "hs_dataset_next: NULL argument");
  if (d->consumed >= (int64_t)d->batches.size()) return hs_fail(nullptr, HS_ERR_STATE, "hs_dataset_next: the epoch is over");
  const int64_t k = d->consumed;
  std::unique_lock<std::mutex> lk(d->mu);
  d->cv.wait(lk, [&] { return d->failed || d->produced > k; });
  if (d->failed) return hs_fail(nullptr, HS_ERR_STATE, d->fail_msg);
  const Ready& r = d->ring[(size_t)(k % (int64_t)d->ring.size())];
  memcpy(ids_out, r.ids.data(), r.ids.size() * 4);
  memcpy(lens_out, r.lens.data(), r.lens.size() * 4);
  if (instance_out) memcpy(instance_out, r.inst.data(), r.inst.size() * 8);
  d->consumed = k + 1;
  lk.unlock();
  d->cv.notify_all();
  return HS_OK;
}

hs_status hs_dataset_stats(hs_dataset* d, int64_t* loads_out, int64_t* hits_out) {
  if (!d || !loads_out || !hits_out) return hs_fail(nullptr, HS_ERR_INVALID_ARG, "hs_dataset_stats: NULL argument");
  std::lock_guard<std::mutex> lk(d->mu);     // (counts of the batches produced so far)
  *loads_out = d->pub_loads; *hits_out = d->pub_hits;
  return HS_OK;
}

}  // extern "C"
