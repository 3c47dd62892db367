// Runs every oracle routine once on a small synthetic workload so that a build with
// -fsanitize=address,undefined can catch out-of-bounds accesses, overflow and other
// undefined behaviour inside the oracle (TEST INFRASTRUCTURE, like the oracle itself).
//
//   g++ -O1 -g -std=c++17 -fsanitize=address,undefined -fno-sanitize-recover=all \
//       sanitize_driver.cpp -o sanitize_driver && ./sanitize_driver
//
// The inputs come from a plain linear congruential generator: they are arbitrary data of the
// right shape, not part of the method.  The driver checks only that the calls return
// normally and agree with each other where two routines compute the same thing.
#include "ginex_oracle.cpp"

#include <cstdio>
#include <cstdlib>

namespace {

uint64_t g_state = 0x2545F4914F6CDD1Dull;
uint32_t next_u32() {
  g_state = g_state * 6364136223846793005ull + 1442695040888963407ull;
  return (uint32_t)(g_state >> 33);
}

void fail(const char* what) {
  std::fprintf(stderr, "sanitize_driver: %s\n", what);
  std::exit(1);
}

struct Lists {
  std::vector<int32_t> init, in, out, pos;
  std::vector<int64_t> off, miss;
  int64_t init_count = 0;
};

bool same(const Lists& a, const Lists& b) {
  const int64_t n = a.off.back();
  return a.init_count == b.init_count && a.off == b.off && a.miss == b.miss &&
         std::equal(a.init.begin(), a.init.begin() + a.init_count, b.init.begin()) &&
         std::equal(a.in.begin(), a.in.begin() + n, b.in.begin()) &&
         std::equal(a.out.begin(), a.out.begin() + n, b.out.begin()) &&
         std::equal(a.pos.begin(), a.pos.begin() + n, b.pos.begin());
}

typedef int32_t (*changeset_fn)(int64_t, const int32_t*, const int64_t*, int32_t, int64_t, int32_t*,
                                int64_t*, int32_t*, int32_t*, int32_t*, int64_t, int64_t*, int64_t*);

Lists run(changeset_fn fn, int64_t n, const std::vector<int32_t>& ids,
          const std::vector<int64_t>& off, int64_t cap) {
  const int32_t S = (int32_t)off.size() - 1;
  Lists r;
  const int64_t c = std::max<int64_t>((int64_t)ids.size(), 1);
  r.init.assign(std::max<int64_t>(cap, 1), 0);
  r.in.assign(c, 0); r.out.assign(c, 0); r.pos.assign(c, 0);
  r.off.assign(S + 1, 0); r.miss.assign(std::max(S, 1), 0);
  if (fn(n, ids.data(), off.data(), S, cap, r.init.data(), &r.init_count, r.in.data(),
         r.out.data(), r.pos.data(), c, r.off.data(), r.miss.data()) != 0)
    fail("a changeset routine returned an error");
  r.miss.resize(S);
  return r;
}

void whole_path(int64_t n, int64_t e, int32_t S, int32_t batch, int64_t cap, bool off64) {
  // multigraph CSR with a few heavy rows, rows sorted
  std::vector<int64_t> deg(n, 0);
  for (int64_t j = 0; j < e; ++j) {
    const uint32_t r = next_u32();
    ++deg[(r & 7) == 0 ? r % 5 : r % n];
  }
  std::vector<int64_t> off(n + 1, 0);
  for (int64_t v = 0; v < n; ++v) off[v + 1] = off[v] + deg[v];
  std::vector<int32_t> ind(std::max<int64_t>(e, 1));
  for (int64_t v = 0; v < n; ++v) {
    for (int64_t j = off[v]; j < off[v + 1]; ++j) ind[j] = (int32_t)(next_u32() % n);
    std::sort(ind.begin() + off[v], ind.begin() + off[v + 1]);
  }
  std::vector<int32_t> off32(off.begin(), off.end());
  const void* offsets = off64 ? (const void*)off.data() : (const void*)off32.data();

  const int32_t fanout[3] = {10, 10, 10};
  std::vector<int32_t> seeds((size_t)S * batch);
  std::vector<int64_t> seed_off(S + 1);
  for (int32_t b = 0; b <= S; ++b) seed_off[b] = (int64_t)b * batch;
  for (auto& s : seeds) s = (int32_t)(next_u32() % n);   // repeats inside a batch are allowed
  int64_t cap_ids = 0, cap_rows = 0, cap_cols = 0;
  for (int32_t b = 0; b < S; ++b) {
    int64_t cur = std::min<int64_t>(batch, n);
    for (int h = 0; h < 3; ++h) {
      cap_rows += cur + 1; cap_cols += cur * fanout[h];
      cur = std::min<int64_t>(cur * (1 + fanout[h]), n);
    }
    cap_ids += cur;
  }
  std::vector<int32_t> ids(cap_ids), col(cap_cols);
  std::vector<int64_t> rowptr(cap_rows), ids_off(S + 1), hops((size_t)S * 4), ro(S * 3 + 1),
      co(S * 3 + 1), need(3);
  if (oracle_sample_superbatch(n, offsets, off64, ind.data(), seeds.data(), seed_off.data(), S,
                               fanout, 3, 7, 3, ids.data(), cap_ids, ids_off.data(), hops.data(),
                               rowptr.data(), cap_rows, col.data(), cap_cols, ro.data(), co.data(),
                               need.data()) != 0)
    fail("oracle_sample_superbatch failed");
  ids.resize(need[0]);

  // neighbour cache, and sampling through it
  std::vector<int64_t> at(n);
  std::vector<int32_t> ca(std::max<int64_t>(e / 3, 1));
  int64_t cached = 0, used = 0;
  oracle_neighbor_cache_build(n, offsets, off64, ind.data(), e / 3, at.data(), ca.data(), &cached,
                              &used);
  for (int64_t v = 0; v < n; ++v) {
    int64_t d = 0;
    const int64_t where = oracle_neighbor_lookup(at.data(), ca.data(), (int32_t)v, &d);
    if (where >= 0 && d != off[v + 1] - off[v]) fail("neighbour cache record has the wrong length");
  }
  std::vector<int32_t> ids2(cap_ids);
  std::vector<int64_t> ids_off2(S + 1), need2(3), lookups(2);
  oracle_sample_superbatch_cached(n, offsets, off64, ind.data(), at.data(), ca.data(), seeds.data(),
                                  seed_off.data(), S, fanout, 3, 7, 3, ids2.data(), cap_ids,
                                  ids_off2.data(), hops.data(), rowptr.data(), cap_rows, col.data(),
                                  cap_cols, ro.data(), co.data(), need2.data(), lookups.data());
  ids2.resize(need2[0]);
  if (ids2 != ids || ids_off2 != ids_off) fail("sampling through the neighbour cache differs");

  std::vector<int32_t> nxt(std::max<size_t>(ids.size(), 1)), first(n);
  oracle_next_use(n, ids.data(), ids_off.data(), S, nxt.data(), first.data());

  const Lists heap = run(oracle_changeset, n, ids, ids_off, cap);
  if (!same(heap, run(oracle_changeset_by_sorting, n, ids, ids_off, cap)))
    fail("Belady: heap and sort-based variants differ");
  const Lists lru = run(oracle_changeset_lru, n, ids, ids_off, cap);
  if (!same(lru, run(oracle_changeset_lru_by_sorting, n, ids, ids_off, cap)))
    fail("LRU: heap and sort-based variants differ");
  oracle_lru_misses(n, ids.data(), ids_off.data(), S, cap, heap.init.data(), heap.init_count);

  // resumed from the standard prefetch: must reproduce the standard lists
  {
    Lists r;
    const int64_t c = std::max<int64_t>((int64_t)ids.size(), 1);
    r.init.assign(std::max<int64_t>(cap, 1), 0);
    r.in.assign(c, 0); r.out.assign(c, 0); r.pos.assign(c, 0);
    r.off.assign(S + 1, 0); r.miss.assign(S, 0);
    std::vector<int32_t> fin(std::max<int64_t>(cap, 1));
    for (int variant = 0; variant < 2; ++variant) {
      auto fn = variant ? oracle_changeset_resume_by_sorting : oracle_changeset_resume;
      if (fn(n, ids.data(), ids_off.data(), S, cap, heap.init.data(), heap.init_count, fin.data(),
             r.init.data(), &r.init_count, r.in.data(), r.out.data(), r.pos.data(), c,
             r.off.data(), r.miss.data()) != 0)
        fail("a resumed changeset returned an error");
      if (heap.init_count == cap && (r.off != heap.off || r.miss != heap.miss))
        fail("resumed from the standard prefetch, the lists differ from the standard ones");
    }
  }

  // static policy
  std::vector<int32_t> sel(std::max<int64_t>(std::min(cap, n), 1));
  const int64_t n_sel = oracle_static_select(n, ind.data(), e, cap, sel.data());
  oracle_static_misses(n, ids.data(), (int64_t)ids.size(), sel.data(), n_sel);

  // executor replay
  const int64_t R = 48;
  std::vector<uint8_t> slow((size_t)n * R), cache((size_t)std::max<int64_t>(cap, 1) * R);
  for (auto& x : slow) x = (uint8_t)next_u32();
  std::vector<int32_t> addr(n);
  oracle_cache_init(cache.data(), addr.data(), n, slow.data(), R, heap.init.data(), heap.init_count);
  for (int32_t i = 0; i < S; ++i) {
    const int64_t lo = ids_off[i], cnt = ids_off[i + 1] - lo, c0 = heap.off[i];
    std::vector<uint8_t> out((size_t)std::max<int64_t>(cnt, 1) * R), want(out.size());
    oracle_gather_update(cache.data(), addr.data(), slow.data(), R, ids.data() + lo, cnt, out.data(),
                         heap.in.data() + c0, heap.out.data() + c0, heap.pos.data() + c0,
                         heap.off[i + 1] - c0);
    oracle_gather(slow.data(), R, ids.data() + lo, cnt, want.data());
    if (out != want) fail("gather through the cache differs from the slow tier's rows");
  }
}

}  // namespace

int main() {
  // Philox / Floyd corner cases: tiny and huge degrees, k = 1 and the maximum
  int64_t picks[64];
  for (int64_t deg : {0ll, 1ll, 9ll, 10ll, 11ll, 64ll, 65ll, 1000003ll, (1ll << 40)})
    for (int k : {1, 10, 64}) {
      const int c = oracle_floyd_picks(5, 17, 2, 1, deg, k, picks);
      if (c != (deg < k ? (int)deg : k)) fail("floyd_picks returned the wrong count");
      for (int s = 0; s < c; ++s)
        if (picks[s] < 0 || picks[s] >= deg || (s && picks[s] <= picks[s - 1]))
          fail("floyd_picks: out of range or not ascending");
    }
  whole_path(3000, 40000, 6, 64, 300, false);     // cache under pressure
  whole_path(3000, 40000, 6, 64, 100000, true);   // everything fits, 64-bit offsets
  whole_path(500, 0, 3, 16, 10, false);           // no edges at all
  whole_path(40, 2000, 4, 40, 7, true);           // every batch covers the whole graph
  whole_path(2000, 30000, 1, 50, 0, false);       // S = 1, no cache
  std::puts("sanitize_driver: ok");
  return 0;
}
