// Paged activation store: the bookkeeping of Sec. 3.4 (budgets, greedy reduction, page
// allocation, the two ordered indices of Algorithm 3, dynamic memory budget).  Host code
// only; the arena's memory belongs to the caller.
#include <algorithm>
#include <cmath>
#include <cstdint>
#include <deque>
#include <map>
#include <new>
#include <unordered_map>
#include <vector>

#include "daf.h"
#include "daf_store.h"

namespace {

// Order of an index: ratio ascending, then id ascending.  The first element is the one that
// gives way first.
struct Key {
  double ratio;
  int64_t id;
};
inline bool key_less(const Key& a, const Key& b) {
  return a.ratio < b.ratio || (a.ratio == b.ratio && a.id < b.id);
}

// ------------------------------------------------------------------------------------------
// Red-black tree over the activation slots (Sec. 3.4 "Page Table Maintenance").  Node z is
// slot z of the store (slots start at 1); node 0 is the shared black sentinel, whose parent
// field is scratch space for the deletion fix-up.  Every slot is in the tree at most once.
// ------------------------------------------------------------------------------------------
class RbTree {
 public:
  RbTree() { t_.push_back(Node{0, 0, 0, false, Key{0.0, 0}}); }
  void clear() {
    root_ = 0;
    count_ = 0;
    t_.resize(1);
    t_[0] = Node{0, 0, 0, false, Key{0.0, 0}};
  }
  int size() const { return count_; }

  void insert(int z, Key k) {
    if ((int)t_.size() <= z) t_.resize((size_t)z + 1, Node{0, 0, 0, false, Key{0.0, 0}});
    t_[z] = Node{0, 0, 0, true, k};
    int y = 0, x = root_;
    while (x) {
      y = x;
      x = key_less(k, t_[x].k) ? t_[x].l : t_[x].r;
    }
    t_[z].p = y;
    if (!y) root_ = z;
    else if (key_less(k, t_[y].k)) t_[y].l = z;
    else t_[y].r = z;
    ++count_;
    // restore: no red node has a red parent
    while (t_[t_[z].p].red) {
      int p = t_[z].p, g = t_[p].p;
      if (p == t_[g].l) {
        const int u = t_[g].r;
        if (t_[u].red) {
          t_[p].red = false; t_[u].red = false; t_[g].red = true;
          z = g;
        } else {
          if (z == t_[p].r) { z = p; rotate_left(z); p = t_[z].p; g = t_[p].p; }
          t_[p].red = false; t_[g].red = true;
          rotate_right(g);
        }
      } else {
        const int u = t_[g].l;
        if (t_[u].red) {
          t_[p].red = false; t_[u].red = false; t_[g].red = true;
          z = g;
        } else {
          if (z == t_[p].l) { z = p; rotate_right(z); p = t_[z].p; g = t_[p].p; }
          t_[p].red = false; t_[g].red = true;
          rotate_left(g);
        }
      }
    }
    t_[root_].red = false;
  }

  void erase(int z) {
    int y = z, x;
    bool y_was_red = t_[y].red;
    if (!t_[z].l) {
      x = t_[z].r;
      transplant(z, x);
    } else if (!t_[z].r) {
      x = t_[z].l;
      transplant(z, x);
    } else {
      y = minimum(t_[z].r);
      y_was_red = t_[y].red;
      x = t_[y].r;
      if (t_[y].p == z) {
        t_[x].p = y;                       // also when x is the sentinel
      } else {
        transplant(y, x);
        t_[y].r = t_[z].r;
        t_[t_[y].r].p = y;
      }
      transplant(z, y);
      t_[y].l = t_[z].l;
      t_[t_[y].l].p = y;
      t_[y].red = t_[z].red;
    }
    --count_;
    if (!y_was_red) erase_fixup(x);
    t_[0] = Node{0, 0, 0, false, Key{0.0, 0}};
  }

  int first() const { return root_ ? minimum(root_) : 0; }
  int next(int x) const {
    if (t_[x].r) return minimum(t_[x].r);
    int y = t_[x].p;
    while (y && x == t_[y].r) { x = y; y = t_[y].p; }
    return y;
  }
  const Key& key(int z) const { return t_[z].k; }

  // Checks the search order and the red-black properties; returns false on any violation.
  bool validate() const {
    if (t_[0].red) return false;
    if (!root_) return count_ == 0;
    if (t_[root_].red || t_[root_].p != 0) return false;
    int black_height = -1, seen = 0;
    if (!validate_node(root_, 0, black_height, seen)) return false;
    if (seen != count_) return false;
    for (int x = first(), prev = 0; x; prev = x, x = next(x))
      if (prev && !key_less(t_[prev].k, t_[x].k)) return false;
    return true;
  }

 private:
  struct Node {
    int p, l, r;
    bool red;
    Key k;
  };
  std::vector<Node> t_;
  int root_ = 0;
  int count_ = 0;

  int minimum(int x) const {
    while (t_[x].l) x = t_[x].l;
    return x;
  }
  void rotate_left(int x) {
    const int y = t_[x].r;
    t_[x].r = t_[y].l;
    if (t_[y].l) t_[t_[y].l].p = x;
    t_[y].p = t_[x].p;
    if (!t_[x].p) root_ = y;
    else if (x == t_[t_[x].p].l) t_[t_[x].p].l = y;
    else t_[t_[x].p].r = y;
    t_[y].l = x;
    t_[x].p = y;
  }
  void rotate_right(int x) {
    const int y = t_[x].l;
    t_[x].l = t_[y].r;
    if (t_[y].r) t_[t_[y].r].p = x;
    t_[y].p = t_[x].p;
    if (!t_[x].p) root_ = y;
    else if (x == t_[t_[x].p].r) t_[t_[x].p].r = y;
    else t_[t_[x].p].l = y;
    t_[y].r = x;
    t_[x].p = y;
  }
  void transplant(int u, int v) {
    if (!t_[u].p) root_ = v;
    else if (u == t_[t_[u].p].l) t_[t_[u].p].l = v;
    else t_[t_[u].p].r = v;
    t_[v].p = t_[u].p;                     // the sentinel remembers its parent for the fix-up
  }
  void erase_fixup(int x) {
    while (x != root_ && !t_[x].red) {
      const int p = t_[x].p;
      if (x == t_[p].l) {
        int w = t_[p].r;
        if (t_[w].red) {
          t_[w].red = false; t_[p].red = true;
          rotate_left(p);
          w = t_[p].r;
        }
        if (!t_[t_[w].l].red && !t_[t_[w].r].red) {
          t_[w].red = true;
          x = p;
        } else {
          if (!t_[t_[w].r].red) {
            t_[t_[w].l].red = false; t_[w].red = true;
            rotate_right(w);
            w = t_[p].r;
          }
          t_[w].red = t_[p].red; t_[p].red = false; t_[t_[w].r].red = false;
          rotate_left(p);
          x = root_;
        }
      } else {
        int w = t_[p].l;
        if (t_[w].red) {
          t_[w].red = false; t_[p].red = true;
          rotate_right(p);
          w = t_[p].l;
        }
        if (!t_[t_[w].l].red && !t_[t_[w].r].red) {
          t_[w].red = true;
          x = p;
        } else {
          if (!t_[t_[w].l].red) {
            t_[t_[w].r].red = false; t_[w].red = true;
            rotate_left(w);
            w = t_[p].l;
          }
          t_[w].red = t_[p].red; t_[p].red = false; t_[t_[w].l].red = false;
          rotate_right(p);
          x = root_;
        }
      }
    }
    t_[x].red = false;
  }
  bool validate_node(int x, int blacks, int& black_height, int& seen) const {
    if (!x) {
      if (black_height < 0) black_height = blacks;
      return black_height == blacks;
    }
    ++seen;
    if (t_[x].red && (t_[t_[x].l].red || t_[t_[x].r].red)) return false;
    if (t_[x].l && t_[t_[x].l].p != x) return false;
    if (t_[x].r && t_[t_[x].r].p != x) return false;
    const int b = blacks + (t_[x].red ? 0 : 1);
    return validate_node(t_[x].l, b, black_height, seen) && validate_node(t_[x].r, b, black_height, seen);
  }
};

// The sorting-based index Sec. 4.3.2 measures against: membership is a flat list, and every
// selection sorts all of it.
class SortIndex {
 public:
  void clear() { slots_.clear(); keys_.clear(); }
  void insert(int z, Key k) {
    if ((int)keys_.size() <= z) keys_.resize((size_t)z + 1, Key{0.0, 0});
    keys_[z] = k;
    slots_.push_back(z);
  }
  void erase(int z) {
    for (size_t i = 0; i < slots_.size(); ++i)
      if (slots_[i] == z) { slots_[i] = slots_.back(); slots_.pop_back(); return; }
  }
  int size() const { return (int)slots_.size(); }
  template <class Pred>
  int select(Pred pred) {
    std::sort(slots_.begin(), slots_.end(), [&](int a, int b) { return key_less(keys_[a], keys_[b]); });
    for (int z : slots_)
      if (pred(z)) return z;
    return 0;
  }

 private:
  std::vector<int> slots_;
  std::vector<Key> keys_;
};

struct Act {
  int64_t id;
  int32_t n_w;
  int32_t widths[DAF_STORE_MAX_WIDTHS];
  int64_t bytes[DAF_STORE_MAX_WIDTHS];
  int64_t time[DAF_STORE_MAX_WIDTHS];
  int32_t w;
  double importance;
  int32_t state;
  int64_t offset, pages;   // in pages, valid while allocated
};

struct Extent {
  int64_t off, len;
};

}  // namespace

struct daf_store_s {
  int64_t P = 0, B_mem = 0, B_time = 0 /* <= 0: none */, step_pages = 0, capacity = 0;
  int kind = DAF_STORE_INDEX_RBTREE;
  std::vector<Act> acts;                         // slot s is acts[s - 1]
  std::unordered_map<int64_t, int> slot_of;
  RbTree mem_tree, time_tree;
  SortIndex mem_sort, time_sort;
  int64_t used_mem = 0, used_time = 0, n_select = 0;
  std::deque<int64_t> evicted;
  std::vector<Extent> free_list;                 // inside [0, capacity), by offset, merged
  std::map<int64_t, int> alloc_by_off;           // allocated runs: first page -> slot

  Act& act(int slot) { return acts[(size_t)slot - 1]; }
  int64_t pages_of(const Act& a) const { return (a.bytes[a.w] + P - 1) / P; }
  int64_t limit() const { return B_mem / P; }
  bool over() const { return used_mem > B_mem || (B_time > 0 && used_time > B_time); }
  bool tighter_is_mem() const {
    const double r_mem = (double)(B_mem - used_mem) / (double)B_mem;
    const double r_time = B_time > 0 ? (double)(B_time - used_time) / (double)B_time : 1.0;
    return r_mem <= r_time;
  }
  Key key_of(const Act& a, bool mem) const {
    return Key{a.importance / (double)(mem ? a.bytes[a.w] : a.time[a.w]), a.id};
  }

  void index_insert(int slot) {
    const Act& a = act(slot);
    if (kind == DAF_STORE_INDEX_RBTREE) {
      mem_tree.insert(slot, key_of(a, true));
      time_tree.insert(slot, key_of(a, false));
    } else {
      mem_sort.insert(slot, key_of(a, true));
      time_sort.insert(slot, key_of(a, false));
    }
  }
  void index_erase(int slot) {
    if (kind == DAF_STORE_INDEX_RBTREE) {
      mem_tree.erase(slot);
      time_tree.erase(slot);
    } else {
      mem_sort.erase(slot);
      time_sort.erase(slot);
    }
  }
  // First slot in the order of the chosen index that satisfies pred; 0 if none.
  template <class Pred>
  int select(bool mem, Pred pred) {
    ++n_select;
    if (kind == DAF_STORE_INDEX_RBTREE) {
      const RbTree& t = mem ? mem_tree : time_tree;
      for (int z = t.first(); z; z = t.next(z))
        if (pred(z)) return z;
      return 0;
    }
    return (mem ? mem_sort : time_sort).select(pred);
  }
  void count(const Act& a) { used_mem += pages_of(a) * P; used_time += a.time[a.w]; }
  void uncount(const Act& a) { used_mem -= pages_of(a) * P; used_time -= a.time[a.w]; }

  // ---- free pages -------------------------------------------------------------------------
  void rebuild_free_list() {
    free_list.clear();
    int64_t pos = 0;
    for (const auto& kv : alloc_by_off) {
      const Act& a = acts[(size_t)kv.second - 1];
      const int64_t gap_end = std::min(a.offset, capacity);
      if (gap_end > pos) free_list.push_back(Extent{pos, gap_end - pos});
      pos = std::max(pos, a.offset + a.pages);
    }
    if (capacity > pos) free_list.push_back(Extent{pos, capacity - pos});
  }
  void free_range(int64_t off, int64_t len) {
    const int64_t end = std::min(off + len, capacity);
    if (off >= end) return;
    auto it = std::lower_bound(free_list.begin(), free_list.end(), off,
                               [](const Extent& e, int64_t o) { return e.off < o; });
    it = free_list.insert(it, Extent{off, end - off});
    if (it + 1 != free_list.end() && it->off + it->len == (it + 1)->off) {
      it->len += (it + 1)->len;
      free_list.erase(it + 1);
    }
    if (it != free_list.begin() && (it - 1)->off + (it - 1)->len == it->off) {
      (it - 1)->len += it->len;
      free_list.erase(it);
    }
  }
  // Lowest run of `need` pages, growing the arena by whole steps while nothing fits; -1 if
  // nothing fits at full size.  Does not take the run.
  int64_t first_fit(int64_t need) {
    for (;;) {
      for (const Extent& e : free_list)
        if (e.len >= need) return e.off;
      if (capacity >= limit()) return -1;
      capacity = std::min(capacity + step_pages, limit());
      rebuild_free_list();
    }
  }
  void take(int slot, int64_t off, int64_t need) {
    for (size_t i = 0; i < free_list.size(); ++i) {
      if (free_list[i].off == off) {
        if (free_list[i].len == need) free_list.erase(free_list.begin() + (std::ptrdiff_t)i);
        else { free_list[i].off += need; free_list[i].len -= need; }
        break;
      }
    }
    Act& a = act(slot);
    a.state = DAF_STORE_ALLOCATED;
    a.offset = off;
    a.pages = need;
    alloc_by_off[off] = slot;
  }
  void detach(int slot) {                        // allocated -> its pages are free
    Act& a = act(slot);
    alloc_by_off.erase(a.offset);
    free_range(a.offset, a.pages);
  }

  void evict(int slot) {
    Act& a = act(slot);
    index_erase(slot);
    uncount(a);
    if (a.state == DAF_STORE_ALLOCATED) {
      detach(slot);
      evicted.push_back(a.id);
    }
    a.state = DAF_STORE_EVICTED;
    a.offset = -1;
    a.pages = 0;
  }
  void reduce() {
    while (over()) {
      const bool mem = tighter_is_mem();
      const int v = select(mem, [](int) { return true; });
      if (!v) break;
      Act& a = act(v);
      if (mem && a.state == DAF_STORE_PLANNED && a.w + 1 < a.n_w) {
        index_erase(v);
        uncount(a);
        ++a.w;
        count(a);
        index_insert(v);
      } else {
        evict(v);
      }
    }
  }
};

extern "C" {

int daf_store_create(int64_t page_bytes, int64_t mem_budget_bytes, int64_t time_budget_ns, int64_t step_bytes,
                     int index_kind, daf_store_t** out_store) {
  if (!out_store) return DAF_EINVAL;
  *out_store = nullptr;
  if (page_bytes <= 0 || mem_budget_bytes <= 0 || step_bytes < page_bytes || step_bytes % page_bytes != 0)
    return DAF_EINVAL;
  if (index_kind != DAF_STORE_INDEX_RBTREE && index_kind != DAF_STORE_INDEX_SORT) return DAF_EINVAL;
  daf_store_t* s = new (std::nothrow) daf_store_t();
  if (!s) return DAF_ENOMEM;
  s->P = page_bytes;
  s->B_mem = mem_budget_bytes;
  s->B_time = time_budget_ns > 0 ? time_budget_ns : 0;
  s->step_pages = step_bytes / page_bytes;
  s->kind = index_kind;
  *out_store = s;
  return DAF_OK;
}

void daf_store_destroy(daf_store_t* store) { delete store; }

int daf_store_reset(daf_store_t* s) {
  if (!s) return DAF_EINVAL;
  s->acts.clear();
  s->slot_of.clear();
  s->mem_tree.clear();
  s->time_tree.clear();
  s->mem_sort.clear();
  s->time_sort.clear();
  s->used_mem = s->used_time = 0;
  s->evicted.clear();
  s->alloc_by_off.clear();
  s->rebuild_free_list();
  return DAF_OK;
}

int daf_store_add(daf_store_t* s, int64_t id, const int32_t* widths, const int64_t* bytes_per_width,
                  const int64_t* time_ns_per_width, int32_t n_widths, double moving_avg_importance) {
  if (!s || !widths || !bytes_per_width || !time_ns_per_width) return DAF_EINVAL;
  if (n_widths < 1 || n_widths > DAF_STORE_MAX_WIDTHS) return DAF_EINVAL;
  if (!std::isfinite(moving_avg_importance) || moving_avg_importance < 0.0) return DAF_EINVAL;
  if (s->slot_of.count(id)) return DAF_EINVAL;
  for (int i = 0; i < n_widths; ++i)
    if (bytes_per_width[i] <= 0 || time_ns_per_width[i] <= 0 || widths[i] <= 0) return DAF_EINVAL;
  try {
    Act a{};
    a.id = id;
    a.n_w = n_widths;
    for (int i = 0; i < n_widths; ++i) {
      a.widths[i] = widths[i];
      a.bytes[i] = bytes_per_width[i];
      a.time[i] = time_ns_per_width[i];
    }
    a.w = 0;
    a.importance = moving_avg_importance;
    a.state = DAF_STORE_PLANNED;
    a.offset = -1;
    a.pages = 0;
    s->acts.push_back(a);
    const int slot = (int)s->acts.size();
    s->slot_of[id] = slot;
    s->count(s->act(slot));
    s->index_insert(slot);
    s->reduce();
  } catch (const std::bad_alloc&) {
    return DAF_ENOMEM;
  }
  return DAF_OK;
}

int daf_store_receive(daf_store_t* s, int64_t id, double importance, int32_t* out_bits, int64_t* out_offset_bytes,
                      int64_t* out_size_bytes) {
  if (!s || !out_bits || !out_offset_bytes || !out_size_bytes) return DAF_EINVAL;
  if (!std::isfinite(importance) || importance < 0.0) return DAF_EINVAL;
  const auto it = s->slot_of.find(id);
  if (it == s->slot_of.end()) return DAF_EINVAL;
  const int slot = it->second;
  *out_bits = 0;
  *out_offset_bytes = -1;
  *out_size_bytes = 0;
  if (s->act(slot).state == DAF_STORE_EVICTED) return DAF_OK;
  if (s->act(slot).state != DAF_STORE_PLANNED) return DAF_EINVAL;
  try {
    s->index_erase(slot);
    s->act(slot).importance = importance;
    s->index_insert(slot);
    s->reduce();
    if (s->act(slot).state == DAF_STORE_EVICTED) return DAF_OK;
    const int64_t need = s->pages_of(s->act(slot));
    int64_t off = s->first_fit(need);
    while (off < 0) {
      const int v = s->select(true, [&](int z) { return s->act(z).state == DAF_STORE_ALLOCATED; });
      if (!v) {
        s->evict(slot);
        return DAF_OK;
      }
      s->evict(v);
      off = s->first_fit(need);
    }
    s->take(slot, off, need);
    const Act& a = s->act(slot);
    *out_bits = a.widths[a.w];
    *out_offset_bytes = off * s->P;
    *out_size_bytes = a.bytes[a.w];
  } catch (const std::bad_alloc&) {
    return DAF_ENOMEM;
  }
  return DAF_OK;
}

int daf_store_add_many(daf_store_t* s, int64_t n, const int64_t* ids, const int32_t* widths,
                       const int64_t* bytes_per_width, const int64_t* time_ns_per_width, int32_t n_widths,
                       const double* moving_avg_importance) {
  if (!s || n < 0 || (n > 0 && (!ids || !widths || !bytes_per_width || !time_ns_per_width || !moving_avg_importance)))
    return DAF_EINVAL;
  if (n_widths < 1 || n_widths > DAF_STORE_MAX_WIDTHS) return DAF_EINVAL;
  for (int64_t i = 0; i < n; ++i) {
    const int rc = daf_store_add(s, ids[i], widths, bytes_per_width + i * n_widths, time_ns_per_width + i * n_widths,
                                 n_widths, moving_avg_importance[i]);
    if (rc != DAF_OK) return rc;
  }
  return DAF_OK;
}

int daf_store_receive_many(daf_store_t* s, int64_t n, const int64_t* ids, const double* importance, int32_t* out_bits,
                           int64_t* out_offset_bytes, int64_t* out_size_bytes) {
  if (!s || n < 0 || (n > 0 && (!ids || !importance || !out_bits || !out_offset_bytes || !out_size_bytes)))
    return DAF_EINVAL;
  for (int64_t i = 0; i < n; ++i) {
    const int rc = daf_store_receive(s, ids[i], importance[i], out_bits + i, out_offset_bytes + i, out_size_bytes + i);
    if (rc != DAF_OK) return rc;
  }
  return DAF_OK;
}

int daf_store_release(daf_store_t* s, int64_t id) {
  if (!s) return DAF_EINVAL;
  const auto it = s->slot_of.find(id);
  if (it == s->slot_of.end() || s->act(it->second).state != DAF_STORE_ALLOCATED) return DAF_EINVAL;
  const int slot = it->second;
  Act& a = s->act(slot);
  s->index_erase(slot);
  s->uncount(a);
  s->detach(slot);
  a.state = DAF_STORE_RELEASED;
  a.offset = -1;
  a.pages = 0;
  return DAF_OK;
}

int daf_store_set_mem_budget(daf_store_t* s, int64_t mem_budget_bytes, daf_store_move_t* out_moves, int32_t max_moves,
                             int32_t* out_n_moves) {
  if (!s || !out_n_moves || mem_budget_bytes <= 0 || max_moves < 0) return DAF_EINVAL;
  if ((size_t)max_moves < s->alloc_by_off.size() || (max_moves > 0 && !out_moves)) return DAF_EINVAL;
  *out_n_moves = 0;
  try {
    s->B_mem = mem_budget_bytes;
    s->reduce();
    bool shrunk = false;
    while (s->capacity > s->limit()) {
      s->capacity = std::max<int64_t>(s->capacity - s->step_pages, 0);
      shrunk = true;
    }
    if (shrunk) s->rebuild_free_list();
    std::vector<int> beyond;
    for (const auto& kv : s->alloc_by_off) {
      const Act& a = s->act(kv.second);
      if (a.offset + a.pages > s->capacity) beyond.push_back(kv.second);
    }
    for (int slot : beyond) {
      Act& a = s->act(slot);
      const int64_t old = a.offset, need = a.pages;
      s->detach(slot);
      const int64_t off = s->first_fit(need);
      if (off < 0) {
        s->index_erase(slot);
        s->uncount(a);
        s->evicted.push_back(a.id);
        a.state = DAF_STORE_EVICTED;
        a.offset = -1;
        a.pages = 0;
      } else {
        s->take(slot, off, need);
        if (off != old) {
          out_moves[*out_n_moves] = daf_store_move_t{a.id, old * s->P, off * s->P, a.bytes[a.w]};
          ++*out_n_moves;
        }
      }
    }
  } catch (const std::bad_alloc&) {
    return DAF_ENOMEM;
  }
  return DAF_OK;
}

int daf_store_set_time_budget(daf_store_t* s, int64_t time_budget_ns) {
  if (!s) return DAF_EINVAL;
  try {
    s->B_time = time_budget_ns > 0 ? time_budget_ns : 0;
    s->reduce();
  } catch (const std::bad_alloc&) {
    return DAF_ENOMEM;
  }
  return DAF_OK;
}

int daf_store_query(const daf_store_t* s, int64_t id, int32_t* out_state, int32_t* out_bits, int64_t* out_offset_bytes,
                    int64_t* out_size_bytes) {
  if (!s || !out_state || !out_bits || !out_offset_bytes || !out_size_bytes) return DAF_EINVAL;
  const auto it = s->slot_of.find(id);
  if (it == s->slot_of.end()) return DAF_EINVAL;
  const Act& a = s->acts[(size_t)it->second - 1];
  *out_state = a.state;
  const bool live = a.state == DAF_STORE_PLANNED || a.state == DAF_STORE_ALLOCATED;
  *out_bits = live ? a.widths[a.w] : 0;
  *out_offset_bytes = a.state == DAF_STORE_ALLOCATED ? a.offset * s->P : -1;
  *out_size_bytes = live ? a.bytes[a.w] : 0;
  return DAF_OK;
}

int32_t daf_store_pop_evicted(daf_store_t* s, int64_t* out_ids, int32_t max_ids) {
  if (!s || !out_ids || max_ids <= 0) return 0;
  int32_t n = 0;
  while (n < max_ids && !s->evicted.empty()) {
    out_ids[n++] = s->evicted.front();
    s->evicted.pop_front();
  }
  return n;
}

int64_t daf_store_capacity_bytes(const daf_store_t* s) { return s ? s->capacity * s->P : 0; }
int64_t daf_store_used_bytes(const daf_store_t* s) { return s ? s->used_mem : 0; }
int64_t daf_store_used_time_ns(const daf_store_t* s) { return s ? s->used_time : 0; }
int64_t daf_store_num_selections(const daf_store_t* s) { return s ? s->n_select : 0; }

int daf_store_validate(const daf_store_t* s) {
  if (!s) return DAF_EINVAL;
  int live = 0;
  int64_t mem = 0, time = 0;
  for (const Act& a : s->acts) {
    if (a.state == DAF_STORE_PLANNED || a.state == DAF_STORE_ALLOCATED) {
      ++live;
      mem += s->pages_of(a) * s->P;
      time += a.time[a.w];
    }
  }
  if (mem != s->used_mem || time != s->used_time) return DAF_EINVAL;
  if (s->kind == DAF_STORE_INDEX_RBTREE) {
    if (!s->mem_tree.validate() || !s->time_tree.validate()) return DAF_EINVAL;
    if (s->mem_tree.size() != live || s->time_tree.size() != live) return DAF_EINVAL;
  } else if (s->mem_sort.size() != live || s->time_sort.size() != live) {
    return DAF_EINVAL;
  }
  // allocated runs are disjoint; free extents are exactly the gaps inside the arena
  int64_t pos = 0;
  std::vector<Extent> gaps;
  for (const auto& kv : s->alloc_by_off) {
    const Act& a = s->acts[(size_t)kv.second - 1];
    if (a.state != DAF_STORE_ALLOCATED || a.offset != kv.first || a.offset < pos) return DAF_EINVAL;
    if (a.pages != s->pages_of(a) || a.offset + a.pages > s->capacity) return DAF_EINVAL;
    if (a.offset > pos) gaps.push_back(Extent{pos, a.offset - pos});
    pos = a.offset + a.pages;
  }
  if (s->capacity > pos) gaps.push_back(Extent{pos, s->capacity - pos});
  if (gaps.size() != s->free_list.size()) return DAF_EINVAL;
  for (size_t i = 0; i < gaps.size(); ++i)
    if (gaps[i].off != s->free_list[i].off || gaps[i].len != s->free_list[i].len) return DAF_EINVAL;
  return DAF_OK;
}

}  // extern "C"
