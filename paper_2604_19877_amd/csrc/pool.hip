// Unified page pool: host-side bookkeeping of one device arena shared by KV caches and recurrent states.
//
// Section 6 of the paper ("Heterogeneous state") pads every per-layer state allocation to a common page
// size so that one paged memory manager serves FA (growing), SWA (bounded at the window) and GDN / KDA
// (fixed) layers alike.  Here the common page is one recurrent state, H*dk*dv*4 bytes; an attention layer
// packs the K blocks and then the V blocks of page_bytes / (2 * block bytes) 16-token pages into it, laid
// out so that the attention kernels address the arena as an ordinary (sparse) pool of 16-token pages.
#include <cstring>
#include <string>
#include <vector>

#include "common.h"

struct sa_pool {
  int n_pages = 0, n_layers = 0;
  size_t page_bytes = 0;
  int kv_pages_per_page = 0;        // 16-token pages per unified page
  int tokens_per_page = 0;
  std::vector<int32_t> free_list;   // stack of free unified pages
  struct Seq {
    bool live = false;
    std::string placement;
    int len = 0;
    // per layer: attention -> unified page of token block j (or -1); recurrent -> one state page
    std::vector<std::vector<int32_t>> pages;
  };
  std::vector<Seq> seqs;
};

namespace {

bool is_attention(char c) { return c == 'F' || c == 'S'; }

sa_pool::Seq* find(sa_pool* pool, int id) {
  if (!pool || id < 0 || id >= static_cast<int>(pool->seqs.size()) || !pool->seqs[id].live) return nullptr;
  return &pool->seqs[id];
}

}  // namespace

extern "C" sa_status sa_pool_create(int n_pages, const sa_shapes* sh, int n_layers, sa_pool** pool_out) {
  const char* name = "sa_pool_create";
  SA_REQUIRE(pool_out, SA_EINVAL, "%s: pool_out is null", name);
  *pool_out = nullptr;
  SA_REQUIRE(sh && n_pages >= 1 && n_layers >= 1, SA_EINVAL, "%s: need shapes, n_pages >= 1 and n_layers >= 1", name);
  SA_REQUIRE(sh->H >= 1 && sh->dk >= 1 && sh->dv >= 1 && sh->Hkv >= 1 && sh->D >= 1 && sh->page_size == 16, SA_EINVAL,
             "%s: bad shapes (page_size must be 16)", name);
  const size_t state_bytes = static_cast<size_t>(sh->H) * sh->dk * sh->dv * sizeof(float);
  const size_t block_pair = 2 * static_cast<size_t>(sh->Hkv) * sh->page_size * sh->D * 2;   // K + V of one 16-token page
  SA_REQUIRE(state_bytes % block_pair == 0, SA_EUNSUPPORTED,
             "%s: a state of %zu bytes is not a whole number of 16-token K+V pages (%zu bytes)", name, state_bytes, block_pair);
  SA_REQUIRE(static_cast<long long>(n_pages) * 2 * (state_bytes / block_pair) <= 0x7fffffffLL, SA_EUNSUPPORTED,
             "%s: too many pages for 32-bit kernel page ids", name);
  sa_pool* pool = new sa_pool;
  pool->n_pages = n_pages;
  pool->n_layers = n_layers;
  pool->page_bytes = state_bytes;
  pool->kv_pages_per_page = static_cast<int>(state_bytes / block_pair);
  pool->tokens_per_page = pool->kv_pages_per_page * sh->page_size;
  pool->free_list.resize(n_pages);
  for (int i = 0; i < n_pages; ++i) pool->free_list[i] = n_pages - 1 - i;   // page 0 is handed out first
  *pool_out = pool;
  return SA_OK;
}

extern "C" void sa_pool_destroy(sa_pool* pool) { delete pool; }
extern "C" size_t sa_pool_page_bytes(const sa_pool* pool) { return pool ? pool->page_bytes : 0; }
extern "C" int sa_pool_tokens_per_page(const sa_pool* pool) { return pool ? pool->tokens_per_page : 0; }
extern "C" int sa_pool_kv_id_stride(const sa_pool* pool) { return pool ? 2 * pool->kv_pages_per_page : 0; }
// One past the largest 16-token page id whose K block and V block both lie inside the arena: the ids of the last unified
// page stop at its middle, because the V block of id i sits half a unified page behind its K block.
extern "C" int sa_pool_kernel_pages(const sa_pool* pool) {
  return pool ? (2 * pool->n_pages - 1) * pool->kv_pages_per_page : 0;
}
extern "C" int sa_pool_free_pages(const sa_pool* pool) { return pool ? static_cast<int>(pool->free_list.size()) : 0; }

extern "C" sa_status sa_pool_seq_create(sa_pool* pool, const char* placement, int* seq_id_out) {
  const char* name = "sa_pool_seq_create";
  SA_REQUIRE(pool && placement && seq_id_out, SA_EINVAL, "%s: null argument", name);
  SA_REQUIRE(static_cast<int>(std::strlen(placement)) == pool->n_layers, SA_EINVAL,
             "%s: the placement has %zu characters, the pool was made for %d layers", name, std::strlen(placement), pool->n_layers);
  int recurrent = 0;
  for (int l = 0; l < pool->n_layers; ++l) {
    const char c = placement[l];
    SA_REQUIRE(c == 'F' || c == 'S' || c == 'K' || c == 'G', SA_EINVAL, "%s: layer %d: unknown mixer '%c'", name, l, c);
    recurrent += !is_attention(c);
  }
  SA_REQUIRE(recurrent <= static_cast<int>(pool->free_list.size()), SA_ENOMEM,
             "%s: %d state pages needed, %zu free", name, recurrent, pool->free_list.size());
  int id = -1;
  for (size_t i = 0; i < pool->seqs.size(); ++i)
    if (!pool->seqs[i].live) {
      id = static_cast<int>(i);
      break;
    }
  if (id < 0) {
    id = static_cast<int>(pool->seqs.size());
    pool->seqs.emplace_back();
  }
  sa_pool::Seq& s = pool->seqs[id];
  s.live = true;
  s.placement = placement;
  s.len = 0;
  s.pages.assign(pool->n_layers, {});
  for (int l = 0; l < pool->n_layers; ++l)
    if (!is_attention(placement[l])) {
      s.pages[l].push_back(pool->free_list.back());
      pool->free_list.pop_back();
    }
  *seq_id_out = id;
  return SA_OK;
}

extern "C" sa_status sa_pool_seq_reserve(sa_pool* pool, int seq_id, int len, int window, int slack) {
  const char* name = "sa_pool_seq_reserve";
  sa_pool::Seq* s = find(pool, seq_id);
  SA_REQUIRE(s, SA_EINVAL, "%s: unknown sequence %d", name, seq_id);
  SA_REQUIRE(len >= 0 && window >= 1 && slack >= 0, SA_EINVAL, "%s: need len >= 0, window >= 1, slack >= 0", name);
  const int tpp = pool->tokens_per_page;
  const int n_blocks = (len + tpp - 1) / tpp;
  const long long keep_from = static_cast<long long>(len) - window - slack;        // S layers: first token still needed
  const int first_s = keep_from > 0 ? static_cast<int>(keep_from / tpp) : 0;
  // first pass: count what must be taken and what comes back
  long long need = 0, give = 0;
  for (int l = 0; l < pool->n_layers; ++l) {
    const char c = s->placement[l];
    if (!is_attention(c)) continue;
    const std::vector<int32_t>& pg = s->pages[l];
    const int first = c == 'S' ? first_s : 0;
    for (int j = 0; j < n_blocks; ++j) {
      const bool mapped = j < static_cast<int>(pg.size()) && pg[j] >= 0;
      if (j >= first && !mapped) ++need;
      if (j < first && mapped) ++give;
    }
  }
  SA_REQUIRE(need <= static_cast<long long>(pool->free_list.size()) + give, SA_ENOMEM,
             "%s: %lld pages needed, %zu free (+%lld released by the window)", name, need, pool->free_list.size(), give);
  // Second pass, in two sweeps over the layers: first every sliding-window layer returns the pages behind its window,
  // then pages are taken.  The count above is over the whole sequence, so a layer may only take once every layer has
  // given (taking layer by layer could empty the free list before a later layer's release refills it).
  for (int l = 0; l < pool->n_layers; ++l) {
    if (s->placement[l] != 'S') continue;
    std::vector<int32_t>& pg = s->pages[l];
    for (int j = 0; j < first_s && j < static_cast<int>(pg.size()); ++j)
      if (pg[j] >= 0) {
        pool->free_list.push_back(pg[j]);
        pg[j] = -1;
      }
  }
  for (int l = 0; l < pool->n_layers; ++l) {
    const char c = s->placement[l];
    if (!is_attention(c)) continue;
    std::vector<int32_t>& pg = s->pages[l];
    if (static_cast<int>(pg.size()) < n_blocks) pg.resize(n_blocks, -1);
    for (int j = c == 'S' ? first_s : 0; j < n_blocks; ++j)
      if (pg[j] < 0) {
        pg[j] = pool->free_list.back();   // cannot be empty: need <= free + give was checked above
        pool->free_list.pop_back();
      }
  }
  if (len > s->len) s->len = len;
  return SA_OK;
}

extern "C" sa_status sa_pool_seq_free(sa_pool* pool, int seq_id) {
  sa_pool::Seq* s = find(pool, seq_id);
  SA_REQUIRE(s, SA_EINVAL, "sa_pool_seq_free: unknown sequence %d", seq_id);
  for (std::vector<int32_t>& pg : s->pages)
    for (int32_t p : pg)
      if (p >= 0) pool->free_list.push_back(p);
  s->pages.clear();
  s->live = false;
  return SA_OK;
}

extern "C" int sa_pool_seq_pages(const sa_pool* pool, int seq_id) {
  const sa_pool::Seq* s = find(const_cast<sa_pool*>(pool), seq_id);
  if (!s) return -1;
  int n = 0;
  for (const std::vector<int32_t>& pg : s->pages)
    for (int32_t p : pg) n += p >= 0;
  return n;
}

extern "C" sa_status sa_pool_layer_tables(const sa_pool* pool, const int32_t* seq_ids, int B, int layer, int32_t* page_table,
                                          int max_pages, int32_t* slot) {
  const char* name = "sa_pool_layer_tables";
  SA_REQUIRE(pool && (B == 0 || seq_ids), SA_EINVAL, "%s: null argument", name);
  SA_REQUIRE(layer >= 0 && layer < pool->n_layers && B >= 0 && max_pages >= 0, SA_EINVAL, "%s: bad layer or sizes", name);
  for (int b = 0; b < B; ++b) SA_REQUIRE(find(const_cast<sa_pool*>(pool), seq_ids[b]), SA_EINVAL, "%s: unknown sequence %d", name, seq_ids[b]);
  const int per = pool->kv_pages_per_page, stride = 2 * per;
  for (int b = 0; b < B; ++b) {
    const sa_pool::Seq& s = pool->seqs[seq_ids[b]];
    const bool attn = is_attention(s.placement[layer]);
    if (slot) slot[b] = attn ? -1 : s.pages[layer][0];
    if (!page_table) continue;
    int32_t* row = page_table + static_cast<size_t>(b) * max_pages;
    for (int k = 0; k < max_pages; ++k) {
      const int j = k / per;
      const bool mapped = attn && j < static_cast<int>(s.pages[layer].size()) && s.pages[layer][j] >= 0;
      row[k] = mapped ? s.pages[layer][j] * stride + k % per : -1;
    }
  }
  return SA_OK;
}
