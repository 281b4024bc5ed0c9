// Priority-ordered residency of K,V caches in slots lent by the serving framework (arxiv 2412.16434, Sec. 3.3:
// priority-based K,V cache, cooperative memory management).  Host code; semantics are stated in symph_pool.h.
//
// Structures: the announced sessions ordered as one layer admits them (larger cache first, then smaller id), the
// resident units ordered as the framework may overwrite them (later layer first, then smaller cache, then larger id:
// the reverse of the admission order), a bitmap of the free slots.  Admission walks layer by layer over the
// sessions that were admitted in the layer before: all layers of a session have one size and the room only shrinks,
// so a session refused once stays refused and leaves the walk.
#include <functional>
#include <new>
#include <set>
#include <tuple>
#include <unordered_map>
#include <utility>
#include <vector>

#include "symph.h"
#include "symph_pool.h"

namespace {

enum : int8_t { kFree = 0, kLent = 1, kFramework = 2 };

struct Session {
  int64_t id;
  int32_t n_tokens;
  int32_t blocks;                            // slots per layer
  std::vector<std::vector<int32_t>> tables;  // one per resident layer, layers 0 .. size()-1
  int32_t resident() const { return (int32_t)tables.size(); }
};

struct AdmitKey {  // order inside one layer
  int32_t blocks;
  int64_t id;
  bool operator<(const AdmitKey& o) const { return blocks != o.blocks ? blocks > o.blocks : id < o.id; }
};

struct GiveUpKey {  // first = first to be overwritten
  int32_t layer, blocks;
  int64_t id;
  bool operator<(const GiveUpKey& o) const {
    if (layer != o.layer) return layer > o.layer;
    if (blocks != o.blocks) return blocks < o.blocks;
    return id > o.id;
  }
};

struct Gone {
  int64_t id;
  int32_t layer, blocks;
};

}  // namespace

struct symph_pool {
  int32_t n_layers, n_slots, block_size;
  int32_t n_free, n_lent, n_framework;
  std::vector<int8_t> state;
  // Free slots as a bitmap; every word below first_word is empty, so taking the lowest free slot is a short scan
  // (a heap of a million slot numbers cost 75 ns per slot, this costs 2).
  std::vector<uint64_t> free_bits;
  size_t first_word;

  void push_free(int32_t slot) {
    const size_t w = (size_t)slot >> 6;
    free_bits[w] |= (uint64_t)1 << (slot & 63);
    if (w < first_word) first_word = w;
  }
  int32_t pop_lowest_free() {  // the caller knows that n_free > 0
    while (free_bits[first_word] == 0) ++first_word;
    const int bit = __builtin_ctzll(free_bits[first_word]);
    free_bits[first_word] &= free_bits[first_word] - 1;
    return (int32_t)(first_word * 64 + bit);
  }
  std::unordered_map<int64_t, Session> sessions;
  std::set<AdmitKey> admit_order;
  std::set<GiveUpKey> give_up_order;
  std::vector<Gone> gone;  // units given up since the last settle

  void release_top_layer(Session& s) {
    const int32_t layer = s.resident() - 1;
    for (int32_t slot : s.tables.back()) {
      state[slot] = kFree;
      push_free(slot);
    }
    n_free += s.blocks;
    n_lent -= s.blocks;
    give_up_order.erase(GiveUpKey{layer, s.blocks, s.id});
    gone.push_back(Gone{s.id, layer, s.blocks});
    s.tables.pop_back();
  }

  // resident layers per session for the slots the framework does not own, in admit_order
  std::vector<std::pair<Session*, int32_t>> target() {
    std::vector<std::pair<Session*, int32_t>> out;
    out.reserve(admit_order.size());
    for (const AdmitKey& k : admit_order) out.emplace_back(&sessions.find(k.id)->second, 0);
    std::vector<int32_t> walk(out.size()), next;
    for (size_t i = 0; i < walk.size(); ++i) walk[i] = (int32_t)i;
    int64_t room = (int64_t)n_slots - n_framework;
    for (int32_t layer = 0; layer < n_layers && !walk.empty(); ++layer) {
      next.clear();
      for (int32_t i : walk) {
        if (out[i].first->blocks <= room) {
          room -= out[i].first->blocks;
          out[i].second = layer + 1;
          next.push_back(i);
        }
      }
      walk.swap(next);
    }
    return out;
  }
};

namespace {

template <class F>
int32_t guarded(F&& f) {
  try {
    return f();
  } catch (const std::bad_alloc&) {
    return SYMPH_ENOMEM;
  } catch (...) {
    return SYMPH_EINVAL;
  }
}

}  // namespace

extern "C" {

int32_t symph_pool_create(int32_t n_layers, int32_t n_slots, int32_t block_size, symph_pool** out) {
  if (!out || n_layers < 1 || n_slots < 1 || block_size < 1) return SYMPH_EINVAL;
  return guarded([&]() -> int32_t {
    symph_pool* p = new symph_pool();
    try {
      p->n_layers = n_layers;
      p->n_slots = n_slots;
      p->block_size = block_size;
      p->n_free = n_slots;
      p->n_lent = p->n_framework = 0;
      p->state.assign((size_t)n_slots, kFree);
      p->free_bits.assign(((size_t)n_slots + 63) / 64, ~(uint64_t)0);
      if (n_slots & 63) p->free_bits.back() = (((uint64_t)1 << (n_slots & 63)) - 1);
      p->first_word = 0;
    } catch (...) {
      delete p;
      throw;
    }
    *out = p;
    return SYMPH_OK;
  });
}

void symph_pool_destroy(symph_pool* pool) { delete pool; }

int32_t symph_pool_advise(symph_pool* pool, int64_t session, int32_t n_tokens) {
  if (!pool || n_tokens < 1) return SYMPH_EINVAL;
  return guarded([&]() -> int32_t {
    auto it = pool->sessions.find(session);
    if (it != pool->sessions.end()) return it->second.n_tokens == n_tokens ? SYMPH_OK : SYMPH_EINVAL;
    const int32_t blocks = (int32_t)(((int64_t)n_tokens + pool->block_size - 1) / pool->block_size);
    Session s{session, n_tokens, blocks, {}};
    s.tables.reserve((size_t)pool->n_layers);
    auto ins = pool->admit_order.insert(AdmitKey{blocks, session});
    try {
      pool->sessions.emplace(session, std::move(s));
    } catch (...) {
      pool->admit_order.erase(ins.first);
      throw;
    }
    return SYMPH_OK;
  });
}

int32_t symph_pool_drop(symph_pool* pool, int64_t session) {
  if (!pool) return SYMPH_EINVAL;
  return guarded([&]() -> int32_t {
    auto it = pool->sessions.find(session);
    if (it == pool->sessions.end()) return SYMPH_EINVAL;
    Session& s = it->second;
    pool->gone.reserve(pool->gone.size() + (size_t)s.resident());  // what follows cannot fail half way
    while (s.resident() > 0) pool->release_top_layer(s);
    pool->admit_order.erase(AdmitKey{s.blocks, s.id});
    pool->sessions.erase(it);
    return SYMPH_OK;
  });
}

int32_t symph_pool_claim(symph_pool* pool, int64_t session, int32_t* h_slots, int32_t max_slots,
                         int32_t* n_resident_layers) {
  if (!pool || !n_resident_layers || max_slots < 0) return SYMPH_EINVAL;
  return guarded([&]() -> int32_t {
    auto it = pool->sessions.find(session);
    if (it == pool->sessions.end()) return SYMPH_EINVAL;
    Session& s = it->second;
    const int64_t need = (int64_t)s.resident() * s.blocks;
    if (need > max_slots) return SYMPH_EWORKSPACE;
    if (need > 0 && !h_slots) return SYMPH_EINVAL;
    int64_t k = 0;
    for (int32_t layer = 0; layer < s.resident(); ++layer) {
      for (int32_t slot : s.tables[layer]) {
        pool->state[slot] = kFramework;
        h_slots[k++] = slot;
      }
      pool->give_up_order.erase(GiveUpKey{layer, s.blocks, s.id});
    }
    pool->n_lent -= (int32_t)need;
    pool->n_framework += (int32_t)need;
    *n_resident_layers = s.resident();
    pool->admit_order.erase(AdmitKey{s.blocks, s.id});
    pool->sessions.erase(it);
    return SYMPH_OK;
  });
}

int32_t symph_pool_framework_take(symph_pool* pool, int32_t n, int32_t* h_slots) {
  if (!pool || n < 0 || (n > 0 && !h_slots)) return SYMPH_EINVAL;
  if (n > pool->n_slots - pool->n_framework) return SYMPH_EWORKSPACE;
  return guarded([&]() -> int32_t {
    pool->gone.reserve(pool->gone.size() + pool->give_up_order.size());
    while (pool->n_free < n) {
      const GiveUpKey k = *pool->give_up_order.begin();  // not empty: n_free + n_lent >= n
      pool->release_top_layer(pool->sessions.find(k.id)->second);
    }
    for (int32_t i = 0; i < n; ++i) {
      const int32_t slot = pool->pop_lowest_free();
      pool->state[slot] = kFramework;
      h_slots[i] = slot;
    }
    pool->n_free -= n;
    pool->n_framework += n;
    return SYMPH_OK;
  });
}

int32_t symph_pool_framework_give(symph_pool* pool, int32_t n, const int32_t* h_slots) {
  if (!pool || n < 0 || (n > 0 && !h_slots)) return SYMPH_EINVAL;
  return guarded([&]() -> int32_t {
    // validate first (a slot listed twice is caught by marking), then commit
    int32_t i = 0;
    bool ok = true;
    for (; i < n; ++i) {
      const int32_t slot = h_slots[i];
      if (slot < 0 || slot >= pool->n_slots || pool->state[slot] != kFramework) { ok = false; break; }
      pool->state[slot] = kFree;
    }
    if (!ok) {
      for (int32_t j = 0; j < i; ++j) pool->state[h_slots[j]] = kFramework;
      return SYMPH_EINVAL;
    }
    for (i = 0; i < n; ++i) pool->push_free(h_slots[i]);
    pool->n_free += n;
    pool->n_framework -= n;
    return SYMPH_OK;
  });
}

int32_t symph_pool_settle(symph_pool* pool, symph_pool_change* h_changes, int32_t max_changes, int32_t* h_slots,
                          int32_t max_slots, int32_t* n_changes, int32_t* n_slots) {
  if (!pool || !n_changes || !n_slots || max_changes < 0 || max_slots < 0) return SYMPH_EINVAL;
  return guarded([&]() -> int32_t {
    auto want = pool->target();
    int64_t changes = (int64_t)pool->gone.size(), slots = 0, new_gone = 0;
    for (auto& [s, r] : want) {
      const int32_t have = s->resident();
      if (r < have) new_gone += have - r;
      if (r > have) { changes += r - have; slots += (int64_t)(r - have) * s->blocks; }
    }
    changes += new_gone;
    if (changes > INT32_MAX || slots > INT32_MAX) return SYMPH_EUNSUPPORTED;
    if (changes > max_changes || slots > max_slots) {
      *n_changes = (int32_t)changes;
      *n_slots = (int32_t)slots;
      return SYMPH_EWORKSPACE;
    }
    if ((changes > 0 && !h_changes) || (slots > 0 && !h_slots)) return SYMPH_EINVAL;
    // the loads in the order of admission: layer by layer, inside a layer as admit_order says
    std::vector<std::pair<Session*, int32_t>> loads;
    loads.reserve((size_t)(changes - (int64_t)pool->gone.size() - new_gone));
    for (int32_t layer = 0; layer < pool->n_layers; ++layer) {
      bool any_above = false;
      for (auto& [s, r] : want) {
        if (r > layer + 1) any_above = true;
        if (layer >= s->resident() && layer < r) loads.emplace_back(s, layer);
      }
      if (!any_above) break;
    }
    // every allocation the commit needs, before the first change
    pool->gone.reserve(pool->gone.size() + (size_t)new_gone);
    std::vector<std::vector<int32_t>> fresh;
    fresh.reserve(loads.size());
    for (auto& [s, layer] : loads) fresh.emplace_back((size_t)s->blocks);
    for (auto& [s, r] : want) s->tables.reserve((size_t)pool->n_layers);

    for (auto& [s, r] : want)
      while (s->resident() > r) pool->release_top_layer(*s);
    int32_t c = 0, k = 0;
    for (const Gone& g : pool->gone) h_changes[c++] = symph_pool_change{g.id, g.layer, SYMPH_POOL_EVICTED, g.blocks, -1};
    pool->gone.clear();
    for (size_t i = 0; i < loads.size(); ++i) {
      Session* s = loads[i].first;
      const int32_t layer = loads[i].second;  // == s->resident(): a session's layers come in ascending order
      std::vector<int32_t>& t = fresh[i];
      for (int32_t b = 0; b < s->blocks; ++b) {
        const int32_t slot = pool->pop_lowest_free();
        pool->state[slot] = kLent;
        t[b] = slot;
        h_slots[k + b] = slot;
      }
      h_changes[c++] = symph_pool_change{s->id, layer, SYMPH_POOL_LOAD, s->blocks, k};
      k += s->blocks;
      pool->n_free -= s->blocks;
      pool->n_lent += s->blocks;
      pool->give_up_order.insert(GiveUpKey{layer, s->blocks, s->id});
      s->tables.push_back(std::move(t));
    }
    *n_changes = c;
    *n_slots = k;
    return SYMPH_OK;
  });
}

int32_t symph_pool_resident_layers(const symph_pool* pool, int64_t session) {
  if (!pool) return SYMPH_EINVAL;
  auto it = pool->sessions.find(session);
  return it == pool->sessions.end() ? (int32_t)SYMPH_EINVAL : it->second.resident();
}

int32_t symph_pool_unit_slots(const symph_pool* pool, int64_t session) {
  if (!pool) return SYMPH_EINVAL;
  auto it = pool->sessions.find(session);
  return it == pool->sessions.end() ? (int32_t)SYMPH_EINVAL : it->second.blocks;
}

int32_t symph_pool_table(const symph_pool* pool, int64_t session, int32_t layer, int32_t* h_slots, int32_t max_slots) {
  if (!pool || layer < 0) return SYMPH_EINVAL;
  auto it = pool->sessions.find(session);
  if (it == pool->sessions.end() || layer >= it->second.resident()) return SYMPH_EINVAL;
  const Session& s = it->second;
  if (s.blocks > max_slots) return SYMPH_EWORKSPACE;
  if (!h_slots) return SYMPH_EINVAL;
  for (int32_t b = 0; b < s.blocks; ++b) h_slots[b] = s.tables[layer][b];
  return s.blocks;
}

int32_t symph_pool_counts(const symph_pool* pool, int32_t* n_free, int32_t* n_lent, int32_t* n_framework) {
  if (!pool) return SYMPH_EINVAL;
  if (n_free) *n_free = pool->n_free;
  if (n_lent) *n_lent = pool->n_lent;
  if (n_framework) *n_framework = pool->n_framework;
  return SYMPH_OK;
}

}  // extern "C"
