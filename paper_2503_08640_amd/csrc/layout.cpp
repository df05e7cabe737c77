// Host block-layout builder: pool structure (+ per-query group selections) ->
// per-Q-tile lists of KV tiles.  Integer work only, no GPU calls.
//
// Stage 1 (Sec. 2.1): a group attends the anchor, a fixed number of preceding
// groups, and itself causally, so the list of a Q tile is: every sink tile, every
// tile of the preceding groups in the window, and the own group's tiles that start
// at or before the tile's last row.  Stage 2 (Sec. 2.2): the selected groups' KV is
// used in place -- the list simply names their tiles behind the sink's -- followed
// by the query's own tiles up to the diagonal.
#include "layout.hpp"

#include <algorithm>
#include <climits>
#include <numeric>
#include <utility>

namespace {

struct Seg {
  int32_t begin, end;
};

inline int32_t pack_len_kind(int32_t len, int32_t kind) { return len | (kind << 16); }

// Append the tiles of [seg.begin, seg.end) cut every `bn` tokens, all with `kind`.
void push_whole_segment(std::vector<int32_t>& ent, Seg seg, int32_t bn, int32_t kind) {
  for (int64_t k0 = seg.begin; k0 < seg.end; k0 += bn) {
    ent.push_back(static_cast<int32_t>(k0));
    ent.push_back(pack_len_kind(static_cast<int32_t>(std::min<int64_t>(bn, seg.end - k0)), kind));
  }
}

// Append the tiles of `seg` a Q tile [q0, q0+qn) sees under a causal rule inside the
// segment: a tile is listed when its first key is not after the tile's last row; it
// needs no mask when its last key is not after the tile's first row.
void push_causal_segment(std::vector<int32_t>& ent, Seg seg, int32_t bn, int32_t q0, int32_t qn, int32_t kind_full,
                         int32_t kind_causal) {
  const int64_t q_last = static_cast<int64_t>(q0) + qn - 1;
  for (int64_t k0 = seg.begin; k0 < seg.end && k0 <= q_last; k0 += bn) {
    const int64_t kn = std::min<int64_t>(bn, seg.end - k0);
    const bool full = (k0 + kn - 1) <= q0;
    ent.push_back(static_cast<int32_t>(k0));
    ent.push_back(pack_len_kind(static_cast<int32_t>(kn), full ? kind_full : kind_causal));
  }
}

bool strictly_increasing(const int32_t* a, int64_t n) {
  for (int64_t i = 1; i < n; ++i)
    if (a[i] <= a[i - 1]) return false;
  return true;
}

}  // namespace

int dbsa_build_host_lists(const dbsa_pool_desc* pool, const dbsa_select_desc* sel, int32_t first_group, int32_t block_m, int32_t block_n,
                          dbsa_layout* L) {
  if (!pool || !L || block_m <= 0 || block_n <= 0 || block_n >= (1 << 16)) return DBSA_ERR_INVALID_ARG;
  if (!pool->demo_offsets || !pool->group_demo_offsets || pool->n_demos < 1 || pool->n_groups < 1 ||
      pool->sink_len < 0 || pool->prev_window < 0)
    return DBSA_ERR_INVALID_ARG;
  const int32_t S = pool->sink_len;
  const int32_t* doff = pool->demo_offsets;
  const int32_t* gdo = pool->group_demo_offsets;
  if (doff[0] != S || !strictly_increasing(doff, static_cast<int64_t>(pool->n_demos) + 1)) return DBSA_ERR_BAD_BOUNDS;
  if (gdo[0] != 0 || gdo[pool->n_groups] != pool->n_demos ||
      !strictly_increasing(gdo, static_cast<int64_t>(pool->n_groups) + 1))
    return DBSA_ERR_BAD_BOUNDS;

  const int32_t G = pool->n_groups;
  if (first_group >= 0 && (sel || first_group >= G)) return DBSA_ERR_INVALID_ARG;
  std::vector<Seg> group(G);
  for (int32_t g = 0; g < G; ++g) group[g] = Seg{doff[gdo[g]], doff[gdo[g + 1]]};
  const Seg sink{0, S};

  L->block_m = block_m;
  L->block_n = block_n;
  L->sink_len = S;
  L->n_tokens = doff[pool->n_demos];
  L->n_groups = G;
  L->prev_window = pool->prev_window;
  L->query_stage = (sel != nullptr);
  L->list_ptr.assign(1, 0);

  auto close_tile = [&](int32_t q0, int32_t qn, int32_t owner) {
    L->qtile_tab.insert(L->qtile_tab.end(), {q0, qn, owner, 0});
    L->list_ptr.push_back(static_cast<int64_t>(L->list_ent.size() / 2));
  };

  // where the segments sit in the tensors the query-stage calls will be given (the pool itself
  // unless the caller keeps groups in arena pages)
  Seg sink_at = sink;
  std::vector<Seg> group_at = group;

  if (!sel) {
    // ---- stage 1 ----
    // An appended group sees the sink, its window of preceding groups and itself; nothing
    // already encoded sees it (Sec. 2.1), so encoding it means walking its own Q tiles only.
    for (int64_t q0 = 0; q0 < S && first_group < 0; q0 += block_m) {
      const int32_t qn = static_cast<int32_t>(std::min<int64_t>(block_m, S - q0));
      push_causal_segment(L->list_ent, sink, block_n, static_cast<int32_t>(q0), qn, DBSA_TILE_FULL, DBSA_TILE_CAUSAL);
      close_tile(static_cast<int32_t>(q0), qn, -1);
    }
    for (int32_t g = std::max(first_group, 0); g < G; ++g) {
      const int32_t first_prev = std::max<int64_t>(0, static_cast<int64_t>(g) - pool->prev_window);
      for (int64_t q0 = group[g].begin; q0 < group[g].end; q0 += block_m) {
        const int32_t qn = static_cast<int32_t>(std::min<int64_t>(block_m, group[g].end - q0));
        push_whole_segment(L->list_ent, sink, block_n, DBSA_TILE_FULL);
        for (int32_t p = first_prev; p < g; ++p) push_whole_segment(L->list_ent, group[p], block_n, DBSA_TILE_FULL);
        push_causal_segment(L->list_ent, group[g], block_n, static_cast<int32_t>(q0), qn, DBSA_TILE_FULL,
                            DBSA_TILE_CAUSAL);
        close_tile(static_cast<int32_t>(q0), qn, g);
      }
    }
  } else {
    // ---- stage 2 ----
    if (sel->n_queries < 1 || !sel->cu_qlens || !sel->sel_ptr || sel->n_split < 0) return DBSA_ERR_INVALID_ARG;
    const int32_t B = sel->n_queries;
    if (sel->cu_qlens[0] != 0 || !strictly_increasing(sel->cu_qlens, static_cast<int64_t>(B) + 1))
      return DBSA_ERR_BAD_BOUNDS;
    if (sel->sel_ptr[0] != 0) return DBSA_ERR_BAD_BOUNDS;
    for (int32_t u = 0; u < B; ++u)
      if (sel->sel_ptr[u + 1] < sel->sel_ptr[u]) return DBSA_ERR_BAD_BOUNDS;
    if (sel->sel_ptr[B] > 0 && !sel->sel_idx) return DBSA_ERR_INVALID_ARG;
    std::vector<int32_t> seen(G, -1);
    for (int32_t u = 0; u < B; ++u)
      for (int32_t e = sel->sel_ptr[u]; e < sel->sel_ptr[u + 1]; ++e) {
        const int32_t g = sel->sel_idx[e];
        if (g < 0 || g >= G || seen[g] == u) return DBSA_ERR_BAD_SELECTION;
        seen[g] = u;
      }

    if (sel->page_start) {
      const int32_t* ps = sel->page_start;
      std::vector<std::pair<int64_t, int64_t>> resident;
      if (S > 0) {
        if (ps[0] < 0) return DBSA_ERR_BAD_BOUNDS;  // the anchor is part of every query's cache
        sink_at = Seg{ps[0], ps[0] + S};
        resident.emplace_back(ps[0], static_cast<int64_t>(ps[0]) + S);
      }
      for (int32_t g = 0; g < G; ++g) {
        const int32_t len = group[g].end - group[g].begin;
        if (ps[g + 1] < 0) continue;
        if (static_cast<int64_t>(ps[g + 1]) + len > INT32_MAX) return DBSA_ERR_BAD_BOUNDS;
        group_at[g] = Seg{ps[g + 1], ps[g + 1] + len};
        resident.emplace_back(ps[g + 1], static_cast<int64_t>(ps[g + 1]) + len);
      }
      std::sort(resident.begin(), resident.end());
      for (size_t i = 1; i < resident.size(); ++i)
        if (resident[i].first < resident[i - 1].second) return DBSA_ERR_BAD_BOUNDS;
      for (int32_t e = 0; e < sel->sel_ptr[B]; ++e)
        if (ps[sel->sel_idx[e] + 1] < 0) return DBSA_ERR_BAD_SELECTION;
    }

    L->n_queries = B;
    L->n_query_tokens = sel->cu_qlens[B];
    L->dec_ptr.assign(1, 0);
    size_t shortest = SIZE_MAX;
    std::vector<int32_t> dec_shift;  // per decode-list entry of the current query
    for (int32_t u = 0; u < B; ++u) {
      // pool part, shared by all Q tiles of the query and by decode
      const size_t dec_begin = L->dec_ent.size();
      push_whole_segment(L->dec_ent, sink_at, block_n, DBSA_TILE_FULL);
      for (int32_t e = sel->sel_ptr[u]; e < sel->sel_ptr[u + 1]; ++e)
        push_whole_segment(L->dec_ent, group_at[sel->sel_idx[e]], block_n, DBSA_TILE_FULL);
      L->dec_ptr.push_back(static_cast<int64_t>(L->dec_ent.size() / 2));
      shortest = std::min(shortest, (L->dec_ent.size() - dec_begin) / 2);
      // new ids (Sec. 2.2): the sink keeps 0 .. S-1, the k-th selected group follows the (k-1)-th,
      // the query follows the cache.  A run whose first key moves from id j to id j' leaves the
      // query row (at id cache_len + a) to be rotated at id cache_len + a - (j' - j).
      int64_t cache_len = S;
      for (int32_t e = sel->sel_ptr[u]; e < sel->sel_ptr[u + 1]; ++e)
        cache_len += group[sel->sel_idx[e]].end - group[sel->sel_idx[e]].begin;
      L->cache_len.push_back(static_cast<int32_t>(cache_len));
      dec_shift.clear();
      dec_shift.insert(dec_shift.end(), (static_cast<size_t>(S) + block_n - 1) / block_n, static_cast<int32_t>(cache_len));
      int64_t new_first = S;
      for (int32_t e = sel->sel_ptr[u]; e < sel->sel_ptr[u + 1]; ++e) {
        const Seg gs = group[sel->sel_idx[e]];
        const size_t n_t = (static_cast<size_t>(gs.end - gs.begin) + block_n - 1) / block_n;
        dec_shift.insert(dec_shift.end(), n_t, static_cast<int32_t>(cache_len - (new_first - gs.begin)));
        new_first += gs.end - gs.begin;
      }

      L->dec_shift.insert(L->dec_shift.end(), dec_shift.begin(), dec_shift.end());

      const Seg self{sel->cu_qlens[u], sel->cu_qlens[u + 1]};
      for (int64_t q0 = self.begin; q0 < self.end; q0 += block_m) {
        const int32_t qn = static_cast<int32_t>(std::min<int64_t>(block_m, self.end - q0));
        L->list_ent.insert(L->list_ent.end(), L->dec_ent.begin() + dec_begin, L->dec_ent.end());
        push_causal_segment(L->list_ent, self, block_n, static_cast<int32_t>(q0), qn, DBSA_TILE_SELF_FULL,
                            DBSA_TILE_SELF_CAUSAL);
        const int32_t a0 = static_cast<int32_t>(q0 - self.begin);  // local index of the tile's first row
        for (int32_t s : dec_shift) L->list_shift.push_back(s + a0);
        L->list_shift.resize(L->list_ent.size() / 2, a0);           // own keys sit at their local index
        close_tile(static_cast<int32_t>(q0), qn, u);
      }
    }
    // split count: enough (query, split) pairs to cover the chip a few times over
    // once multiplied by the KV heads, but never more splits than tiles.
    int32_t ns = sel->n_split;
    if (ns == 0) {
      ns = std::max(1, std::min(32, (256 + B - 1) / B));
      ns = static_cast<int32_t>(std::max<size_t>(1, std::min<size_t>(ns, shortest)));
    }
    L->n_split = ns;
    L->split_ptr.resize(static_cast<size_t>(B) * (ns + 1));
    for (int32_t u = 0; u < B; ++u) {
      const int64_t base = L->dec_ptr[u], len = L->dec_ptr[u + 1] - base;
      for (int32_t s = 0; s <= ns; ++s) L->split_ptr[static_cast<size_t>(u) * (ns + 1) + s] = base + (s * len) / ns;
    }
  }

  // runs cut to measure for the steps that run as a contraction (below): [segment][batch of 64 users] -> run
  // boundaries, the segments' users, the rotation shift of (query, segment), the share of rows that carry a query
  std::vector<std::vector<std::vector<int64_t>>> plan_cuts;
  std::vector<std::vector<int32_t>> plan_users;
  std::vector<int32_t> plan_shift;
  float plan_fill = 0.f;
  if (sel) {
    // ---- group-major decode schedule ----
    // Queries that selected the same group read the same KV, so at decode a chunk of a
    // segment (the sink, a group) is one work item for up to kItemQueries of its users:
    // its keys are fetched once and scored against all of them.  Every (item, user) pair
    // owns one partial-softmax slot; a query's last slot is for its own cached keys.
    constexpr int32_t kItemQueries = 32;
    const int32_t B = sel->n_queries;
    std::vector<std::vector<int32_t>> users(static_cast<size_t>(G) + 1);
    if (S > 0)
      for (int32_t u = 0; u < B; ++u) users[0].push_back(u);
    for (int32_t u = 0; u < B; ++u)
      for (int32_t e = sel->sel_ptr[u]; e < sel->sel_ptr[u + 1]; ++e) users[sel->sel_idx[e] + 1].push_back(u);
    for (auto& v : users) std::sort(v.begin(), v.end());
    L->gm_seg_ptr.assign(1, 0);
    push_whole_segment(L->gm_seg_ent, sink_at, block_n, DBSA_TILE_FULL);
    L->gm_seg_ptr.push_back(static_cast<int64_t>(L->gm_seg_ent.size() / 2));
    for (int32_t g = 0; g < G; ++g) {
      push_whole_segment(L->gm_seg_ent, group_at[g], block_n, DBSA_TILE_FULL);
      L->gm_seg_ptr.push_back(static_cast<int64_t>(L->gm_seg_ent.size() / 2));
    }
    int64_t max_tiles = 1, tile_batches = 0;
    for (int32_t s = 0; s <= G; ++s) {
      const int64_t t = L->gm_seg_ptr[s + 1] - L->gm_seg_ptr[s];
      if (users[s].empty() || t == 0) continue;
      max_tiles = std::max(max_tiles, t);
      tile_batches += t * ((static_cast<int64_t>(users[s].size()) + kItemQueries - 1) / kItemQueries);
    }
    // single-wave workgroups the chip holds per KV head of an 8-KV-head model (six per compute
    // unit), three quarters of them for pool runs: the rest is for the queries' own caches and for
    // items that take a second batch of queries
    const int64_t run_slots = std::max<int64_t>(1, static_cast<int64_t>(L->compute_units) * 6 / 8 * 3 / 4);
    int64_t chunk = sel->n_split > 0 ? (max_tiles + sel->n_split - 1) / sel->n_split
                                     : std::min<int64_t>(32, (tile_batches + run_slots - 1) / run_slots);
    chunk = std::max<int64_t>(1, chunk);
    // Steps that will run their pool items as a contraction (64 queries per wave, one persistent
    // workgroup per compute unit and KV head: mx_rec below) are bound by arithmetic, and what counts is
    // that every worker gets the same work.  Runs of ONE length cannot do that (90 runs of 32 tiles over
    // 32 workers: three rounds for 2.8 rounds of work), so such a layout cuts its runs to measure: the
    // (segment, 64 queries) units are walked in order and dealt to W workers (W = compute units / 8 per
    // KV head, fewer when a worker's share would fall below kMinShare tiles), each taking tiles until
    // its cost (tiles + kRunCost per run, what starting and finishing a run costs in tiles) reaches the
    // mean; a unit that does not fit is cut there, but no run is shorter than kSnap tiles: a worker
    // rather stops a little early or takes the few tiles that are left.  Worker c takes the runs
    // mx_plan_ptr[c] .. mx_plan_ptr[c+1]-1, in order.  plan_cuts[s][b] = the run boundaries of the b-th
    // batch of 64 queries of segment s.
    if (sel->n_split == 0) {
      double rows = 0.0, used = 0.0;
      int64_t line = 0, n_units = 0;
      for (int32_t s = 0; s <= G; ++s) {
        const int64_t t = L->gm_seg_ptr[s + 1] - L->gm_seg_ptr[s];
        const int64_t n_u = static_cast<int64_t>(users[s].size());
        if (n_u == 0 || t == 0) continue;
        rows += 64.0 * static_cast<double>(t) * static_cast<double>((n_u + 63) / 64);
        used += static_cast<double>(t) * static_cast<double>(n_u);
        line += t * ((n_u + 63) / 64);
        n_units += (n_u + 63) / 64;
      }
      if (rows > 0.0 && used / rows >= kMatrixRowFill) {
        constexpr int64_t kMinShare = 12, kSnap = 4;
        constexpr double kRunCost = 4.5;
        const int64_t nominal = std::max<int64_t>(1, L->compute_units / 8);
        const int64_t workers = std::max<int64_t>(1, std::min<int64_t>(nominal, line / kMinShare));
        int64_t n_rec = 0, longest = 1;
        // one walk for a given share; returns what is left for the last worker, who takes the rest
        auto deal = [&](double target) {
          plan_cuts.assign(static_cast<size_t>(G) + 1, {});
          L->mx_plan_ptr.assign(1, 0);
          n_rec = 0;
          longest = 1;
          double acc = 0.0;
          auto next_worker = [&]() {
            L->mx_plan_ptr.push_back(static_cast<int32_t>(n_rec));
            acc = 0.0;
          };
          for (int32_t s = 0; s <= G; ++s) {
            const int64_t t0 = L->gm_seg_ptr[s], t = L->gm_seg_ptr[s + 1] - t0;
            const int64_t n_u = static_cast<int64_t>(users[s].size());
            if (n_u == 0 || t == 0) continue;
            for (int64_t b = 0; b < (n_u + 63) / 64; ++b) {
              std::vector<int64_t> bounds(1, t0);
              int64_t pos = 0;
              while (pos < t) {
                const bool last = static_cast<int64_t>(L->mx_plan_ptr.size()) >= workers;
                const double room = target - acc - kRunCost;
                const int64_t rem = t - pos;
                if (last || static_cast<double>(rem) <= room + static_cast<double>(kSnap)) {
                  acc += kRunCost + static_cast<double>(rem);  // the rest of the unit is one run
                  longest = std::max(longest, rem);
                  pos = t;
                } else if (room < static_cast<double>(kSnap) && acc > 0.0) {
                  next_worker();  // no room worth a run
                } else {
                  const int64_t take = std::min(rem - kSnap, std::max<int64_t>(kSnap, static_cast<int64_t>(room)));
                  pos += take;
                  bounds.push_back(t0 + pos);
                  longest = std::max(longest, take);
                  n_rec += 1;
                  next_worker();
                }
              }
              bounds.push_back(t0 + t);
              n_rec += 1;
              plan_cuts[static_cast<size_t>(s)].push_back(std::move(bounds));
            }
          }
          const double last_cost = static_cast<int64_t>(L->mx_plan_ptr.size()) >= workers ? acc : 0.0;
          while (static_cast<int64_t>(L->mx_plan_ptr.size()) < workers) L->mx_plan_ptr.push_back(static_cast<int32_t>(n_rec));
          L->mx_plan_ptr.push_back(static_cast<int32_t>(n_rec));
          return last_cost;
        };
        L->mx_plan_workers = static_cast<int32_t>(nominal);
        // the smallest share with which the last worker is left no more than the others (the number of
        // runs, and with it the total cost, depends on the share itself)
        double lo = static_cast<double>(line) / static_cast<double>(workers);
        // (a worker stops less than kRunCost + kSnap short of the share, and there are at most units + W runs:
        // with this share the last worker is sure to be left no more than the others)
        double hi = (static_cast<double>(line) + kRunCost * static_cast<double>(n_units + workers)) / static_cast<double>(workers) +
                    kRunCost + 2.0 * static_cast<double>(kSnap);
        for (int it = 0; it < 24; ++it) {
          const double mid = 0.5 * (lo + hi);
          (deal(mid) <= mid + static_cast<double>(kSnap) ? hi : lo) = mid;
        }
        deal(hi);
        plan_fill = static_cast<float>(used / rows);
      }
    }
    L->gm_chunk_tiles = static_cast<int32_t>(chunk);
    // displacement of segment s for user u, as in list_shift but without a tile offset
    std::vector<int32_t> seg_shift(static_cast<size_t>(B) * (G + 1), 0);
    for (int32_t u = 0; u < B; ++u) {
      seg_shift[static_cast<size_t>(u) * (G + 1)] = L->cache_len[u];
      int64_t new_first = S;
      for (int32_t e = sel->sel_ptr[u]; e < sel->sel_ptr[u + 1]; ++e) {
        const int32_t g = sel->sel_idx[e];
        seg_shift[static_cast<size_t>(u) * (G + 1) + g + 1] = static_cast<int32_t>(L->cache_len[u] - (new_first - group[g].begin));
        new_first += group[g].end - group[g].begin;
      }
    }
    std::vector<int64_t> n_slots(B, 0);
    // first pass: count slots per query; second pass: emit items with absolute slot numbers
    for (int pass = 0; pass < 2; ++pass) {
      std::vector<int64_t> next(B, 0);
      if (pass == 1) {
        L->gm_slot_ptr.assign(static_cast<size_t>(B) + 1, 0);
        for (int32_t u = 0; u < B; ++u) L->gm_slot_ptr[u + 1] = L->gm_slot_ptr[u] + n_slots[u] + 1;  // + own cache
      }
      for (int32_t s = 0; s <= G; ++s) {
        const int64_t t0 = L->gm_seg_ptr[s], t1 = L->gm_seg_ptr[s + 1];
        if (users[s].empty()) continue;
        // the segment's tiles are cut into ceil(tiles / chunk) runs of equal length (to within one
        // tile): a short last run would leave its workgroup idle while the full ones finish
        const int64_t n_runs = (t1 - t0 + chunk - 1) / chunk;
        for (int64_t run = 0; run < n_runs; ++run) {
          const int64_t c0 = t0 + run * (t1 - t0) / n_runs, c1 = t0 + (run + 1) * (t1 - t0) / n_runs;
          for (size_t b0 = 0; b0 < users[s].size(); b0 += kItemQueries) {
            const size_t b1 = std::min(users[s].size(), b0 + kItemQueries);
            if (pass == 1)
              L->gm_items.insert(L->gm_items.end(),
                                 {static_cast<int32_t>(c0), static_cast<int32_t>(c1 - c0),
                                  static_cast<int32_t>(L->gm_qrefs.size() / 2), static_cast<int32_t>(b1 - b0)});
            for (size_t k = b0; k < b1; ++k) {
              const int32_t u = users[s][k];
              if (pass == 0)
                ++n_slots[u];
              else {
                L->gm_qrefs.push_back(u);
                L->gm_qrefs.push_back(static_cast<int32_t>(L->gm_slot_ptr[u] + next[u]++));
                L->gm_qshift.push_back(seg_shift[static_cast<size_t>(u) * (G + 1) + s]);
              }
            }
          }
        }
      }
    }
    if (!plan_cuts.empty()) {
      plan_users = users;
      plan_shift = seg_shift;
    }
  }

  for (size_t i = 3; i < L->gm_items.size(); i += 4) L->gm_max_queries = std::max(L->gm_max_queries, L->gm_items[i]);
  for (const int32_t shift : L->gm_qshift) L->max_decode_shift = std::max<int64_t>(L->max_decode_shift, shift);
  if (!plan_cuts.empty()) {
    // Records of the runs cut to measure, with references and slots of their own (the work items above keep
    // their runs of one length for the steps that do not run as a contraction): per unit, run by run, the
    // unit's users with one slot each; a query's last slot is again its own cache.
    const int32_t B = L->n_queries;
    std::vector<int64_t> n_slots(static_cast<size_t>(B), 0), next(static_cast<size_t>(B), 0);
    for (int pass = 0; pass < 2; ++pass) {
      if (pass == 1) {
        L->mx_slot_ptr.assign(static_cast<size_t>(B) + 1, 0);
        for (int32_t u = 0; u < B; ++u) L->mx_slot_ptr[u + 1] = L->mx_slot_ptr[u] + n_slots[u] + 1;
      }
      for (size_t s = 0; s < plan_cuts.size(); ++s)
        for (size_t b = 0; b < plan_cuts[s].size(); ++b)
          for (size_t run = 0; run + 1 < plan_cuts[s][b].size(); ++run) {
            const size_t b0 = 64 * b, b1 = std::min(plan_users[s].size(), b0 + 64);
            if (pass == 1)
              L->mx_rec.insert(L->mx_rec.end(),
                               {static_cast<int32_t>(L->mx_qrefs.size() / 2), static_cast<int32_t>(b1 - b0),
                                static_cast<int32_t>(plan_cuts[s][b][run]),
                                static_cast<int32_t>(plan_cuts[s][b][run + 1] - plan_cuts[s][b][run])});
            for (size_t k = b0; k < b1; ++k) {
              const int32_t u = plan_users[s][k];
              if (pass == 0) {
                ++n_slots[static_cast<size_t>(u)];
              } else {
                L->mx_qrefs.push_back(u);
                L->mx_qrefs.push_back(static_cast<int32_t>(L->mx_slot_ptr[u] + next[static_cast<size_t>(u)]++));
                L->mx_qshift.push_back(plan_shift[static_cast<size_t>(u) * plan_cuts.size() + s]);
              }
            }
          }
    }
    L->mx_row_fill = plan_fill;
  } else {
    // No plan: the work items' runs with up to 64 queries each: consecutive items of one run (its batches of
    // 32 queries, whose references follow each other) are taken in pairs.  Slots do not change.
    const size_t n_items = L->gm_items.size() / 4;
    double rows = 0.0, used = 0.0;
    for (size_t it = 0; it < n_items; ++it) {
      const int32_t* a = &L->gm_items[4 * it];
      int32_t n_q = a[3];
      if (it + 1 < n_items) {
        const int32_t* b = a + 4;
        if (b[0] == a[0] && b[1] == a[1] && b[2] == a[2] + a[3] && a[3] == 32) {
          n_q += b[3];
          ++it;
        }
      }
      L->mx_rec.insert(L->mx_rec.end(), {a[2], n_q, a[0], a[1]});
      rows += 64.0 * a[1];
      used += static_cast<double>(n_q) * a[1];
    }
    L->mx_row_fill = rows > 0.0 ? static_cast<float>(used / rows) : 0.f;
  }
  {
    const size_t n_items = L->gm_items.size() / 4;
    L->gm_item_run.resize(n_items * 4);
    L->gm_ref_pad.resize(n_items * 32 * 4);
    for (size_t it = 0; it < n_items; ++it) {
      const int32_t ent_begin = L->gm_items[4 * it], ent_count = L->gm_items[4 * it + 1];
      const int32_t ref_begin = L->gm_items[4 * it + 2], n_q = L->gm_items[4 * it + 3];
      // tiles of one segment follow each other without gaps and all but the last are full
      L->gm_item_run[4 * it + 0] = L->gm_seg_ent[2 * ent_begin];
      L->gm_item_run[4 * it + 1] = block_n * (ent_count - 1) + (L->gm_seg_ent[2 * (ent_begin + ent_count - 1) + 1] & 0xFFFF);
      L->gm_item_run[4 * it + 2] = n_q;
      L->gm_item_run[4 * it + 3] = 0;
      for (int32_t j = 0; j < 32; ++j) {
        const int32_t ref = ref_begin + std::min(j, n_q - 1);
        int32_t* dst = &L->gm_ref_pad[(it * 32 + j) * 4];
        dst[0] = L->gm_qrefs[2 * ref];
        dst[1] = L->gm_qrefs[2 * ref + 1];
        dst[2] = L->gm_qshift[ref];
        dst[3] = 0;
      }
    }
  }
  if (L->query_stage) {
    const int32_t n_items = static_cast<int32_t>(L->gm_items.size() / 4);
    const int32_t pool_blocks = (n_items + 7) / 8, self_blocks = (L->n_queries + 7) / 8;
    for (int k = 0; k < 6; ++k) {
      const int32_t per_wave = 32 >> k;
      L->gm_rows_off[k] = static_cast<int32_t>(L->gm_rows.size());
      for (int32_t b = 0; b < pool_blocks; ++b) {
        int32_t most = 0;
        for (int32_t it = 8 * b; it < std::min(n_items, 8 * b + 8); ++it) most = std::max(most, L->gm_items[4 * it + 3]);
        for (int32_t z = 0; z * per_wave < most; ++z) L->gm_rows.push_back((b << 8) | z);
      }
      L->gm_pool_rows[k] = static_cast<int32_t>(L->gm_rows.size()) - L->gm_rows_off[k];
      // how often a key of the pool items is walked when a wave takes per_wave queries
      double keys = 0.0, walked = 0.0;
      for (int32_t it = 0; it < n_items; ++it) {
        const double n = L->gm_item_run[4 * it + 1];
        keys += n;
        walked += n * ((L->gm_item_run[4 * it + 2] + per_wave - 1) / per_wave);
      }
      L->gm_walks_per_key[k] = keys > 0.0 ? static_cast<float>(walked / keys) : 1.f;
      for (int32_t b = 0; b < self_blocks; ++b) L->gm_rows.push_back((pool_blocks + b) << 8);
    }
    L->gm_rows_off[6] = static_cast<int32_t>(L->gm_rows.size());
  }
  L->shortest_list = INT64_MAX;
  for (int64_t t = 0; t < L->n_qtiles(); ++t) {
    L->shortest_list = std::min(L->shortest_list, L->list_ptr[t + 1] - L->list_ptr[t]);
    if (!L->list_shift.empty())
      for (int64_t e = L->list_ptr[t]; e < L->list_ptr[t + 1]; ++e)
        L->max_rotation_id = std::max<int64_t>(L->max_rotation_id,
                                               static_cast<int64_t>(L->list_shift[e]) + L->qtile_tab[4 * t + 1] - 1);
  }
  if (L->n_qtiles() == 0) L->shortest_list = 0;

  // launch order: owner by owner (a group at pre-encoding, a query at the query stage), the
  // longest list of an owner first.  Q tiles of one owner walk the same KV, so keeping them
  // adjacent keeps that KV in the L2 of the XCD that runs them.
  // At the query stage the owners themselves are put in the order of their selections (the lists
  // of selected groups compared word by word, then the query index): queries that start with the
  // same groups then run side by side and walk the same keys at about the same time, which is what
  // lets many queries with small selections share the L2 of the XCD that serves a KV head.
  const int64_t nt = L->n_qtiles();
  std::vector<int32_t> owner_rank;
  if (L->query_stage && sel) {
    std::vector<int32_t> by_sel(static_cast<size_t>(sel->n_queries));
    std::iota(by_sel.begin(), by_sel.end(), 0);
    std::stable_sort(by_sel.begin(), by_sel.end(), [&](int32_t a, int32_t b) {
      return std::lexicographical_compare(sel->sel_idx + sel->sel_ptr[a], sel->sel_idx + sel->sel_ptr[a + 1],
                                          sel->sel_idx + sel->sel_ptr[b], sel->sel_idx + sel->sel_ptr[b + 1]);
    });
    owner_rank.resize(by_sel.size());
    for (size_t i = 0; i < by_sel.size(); ++i) owner_rank[static_cast<size_t>(by_sel[i])] = static_cast<int32_t>(i);
  }
  auto rank_of = [&](int32_t owner) {
    return owner >= 0 && static_cast<size_t>(owner) < owner_rank.size() ? owner_rank[static_cast<size_t>(owner)] : owner;
  };
  L->order.resize(nt);
  std::iota(L->order.begin(), L->order.end(), 0);
  std::stable_sort(L->order.begin(), L->order.end(), [&](int32_t a, int32_t b) {
    const int32_t oa = rank_of(L->qtile_tab[4 * a + 2]), ob = rank_of(L->qtile_tab[4 * b + 2]);
    if (oa != ob) return oa < ob;
    return (L->list_ptr[a + 1] - L->list_ptr[a]) > (L->list_ptr[b + 1] - L->list_ptr[b]);
  });
  return DBSA_OK;
}

void dbsa_balance_records(const std::vector<int32_t>& rec_in, int32_t n_classes, std::vector<int32_t>* class_ptr,
                          std::vector<int32_t>* rec) {
  constexpr int64_t kTileCost = 3;  // what a record costs beyond its list, in list entries
  const int64_t nt = static_cast<int64_t>(rec_in.size() / 4);
  std::vector<int64_t> load(static_cast<size_t>(n_classes), 0);
  std::vector<std::vector<int32_t>> recs_of(static_cast<size_t>(n_classes));
  std::vector<int32_t> round, by_load(static_cast<size_t>(n_classes));
  auto entries = [&](int32_t t) { return static_cast<int64_t>(rec_in[4 * static_cast<size_t>(t) + 3]); };
  for (int64_t a = 0; a < nt; a += n_classes) {
    const int64_t b = std::min<int64_t>(nt, a + n_classes);
    round.resize(static_cast<size_t>(b - a));
    std::iota(round.begin(), round.end(), static_cast<int32_t>(a));
    std::stable_sort(round.begin(), round.end(), [&](int32_t x, int32_t y) { return entries(x) > entries(y); });
    std::iota(by_load.begin(), by_load.end(), 0);
    std::stable_sort(by_load.begin(), by_load.end(), [&](int32_t x, int32_t y) { return load[x] < load[y]; });
    for (size_t i = 0; i < round.size(); ++i) {
      const int32_t c = by_load[i];
      recs_of[c].push_back(round[i]);
      load[c] += entries(round[i]) + kTileCost;
    }
  }
  class_ptr->assign(static_cast<size_t>(n_classes) + 1, 0);
  rec->clear();
  rec->reserve(rec_in.size());
  for (int32_t c = 0; c < n_classes; ++c) {
    for (int32_t t : recs_of[c]) rec->insert(rec->end(), rec_in.begin() + 4 * static_cast<size_t>(t), rec_in.begin() + 4 * static_cast<size_t>(t) + 4);
    (*class_ptr)[c + 1] = static_cast<int32_t>(rec->size() / 4);
  }
}

void dbsa_balance_schedule(const dbsa_layout* L, int32_t n_classes, std::vector<int32_t>* class_ptr,
                           std::vector<int32_t>* rec) {
  const int64_t nt = L->n_qtiles();
  std::vector<int32_t> in_order;
  in_order.reserve(static_cast<size_t>(nt) * 4);
  for (int64_t i = 0; i < nt; ++i) {
    const int32_t t = L->order[static_cast<size_t>(i)];
    in_order.push_back(L->qtile_tab[4 * t + 0]);
    in_order.push_back(L->qtile_tab[4 * t + 1]);
    in_order.push_back(static_cast<int32_t>(L->list_ptr[t]));
    in_order.push_back(static_cast<int32_t>(L->list_ptr[t + 1] - L->list_ptr[t]));
  }
  dbsa_balance_records(in_order, n_classes, class_ptr, rec);
}
