// Replays a script of pool operations against the host library (CPU build, sanitizers on) and
// compares every status, id, slot list and the whole pool state with the expected values the
// script carries (written by the Python test from the pool model).  Exit code 0 = all equal.
//
// Script = whitespace-separated integers:
//   0 num_blocks n_layers device(0/1) max_q n_order order...      create the pool (first line)
//   1 expect_pid                                                   prefix_create
//   2 pid layer n pos0 expect_status                               prefix_append
//   3 parent n expect_status expect_pid                            prefix_fork
//   4 pid expect_status                                            prefix_release
//   5 pid kind expect_status expect_sid                            stream_create
//   6 sid expect_status                                            stream_release
//   7 sid new_len expect_status                                    stream_rewind
//   8 flags n_items (sid n_new)* expect_status n_slots slot*       batch_build (+ one step, destroy)
//   9 skip k                                                       after `skip` device calls, k fail
//  10 nb ref* nfree free* ns (sid pid kind len nblk blk*)* np (pid len nblk sealed nstreams blk*)*
#include "../../include/oxy.h"

#include <cstdio>
#include <cstdlib>
#include <vector>

extern "C" void oxy_stub_fail_next(int skip, int k);

static FILE* g_in;
static long g_line = 0;
static bool next_int(long* v) { return fscanf(g_in, "%ld", v) == 1; }
static long need() {
  long v;
  if (!next_int(&v)) {
    fprintf(stderr, "script ended inside op %ld\n", g_line);
    exit(3);
  }
  return v;
}
#define CHECK(cond, ...)                               \
  do {                                                 \
    if (!(cond)) {                                     \
      fprintf(stderr, "op %ld: ", g_line);             \
      fprintf(stderr, __VA_ARGS__);                    \
      fprintf(stderr, " [%s]\n", oxy_last_error());    \
      exit(1);                                         \
    }                                                  \
  } while (0)

int main(int argc, char** argv) {
  if (argc < 2 || !(g_in = fopen(argv[1], "r"))) return 2;
  oxy_pool* pool = nullptr;
  std::vector<char> kv, ws, scratch;
  int n_layers = 1;
  bool device = false;
  long op;
  while (next_int(&op)) {
    ++g_line;
    switch (op) {
      case 0: {
        oxy_pool_config c = {};
        c.num_blocks = (int32_t)need();
        c.n_layers = n_layers = (int32_t)need();
        device = need() != 0;
        c.max_q_tokens = (int32_t)need();
        c.n_q_heads = 8, c.n_kv_heads = 1, c.head_dim = 256, c.page_size = 16;
        std::vector<int32_t> order((size_t)need());
        for (auto& o : order) o = (int32_t)need();
        c.free_order = order.empty() ? nullptr : order.data();
        c.max_partials = 4096;
        c.max_work_items = 4096;
        if (device) {   // "device" buffers are host memory of exactly the requested size
          kv.resize(256);   // never touched: the launches are stand-ins
          ws.resize(oxy_workspace_bytes(&c) + 256);
          c.kv_base = (void*)(((uintptr_t)kv.data() + 255) & ~(uintptr_t)255);
          c.kv_base = (void*)0x100000;   // only ever used for address arithmetic
          c.kv_bytes = oxy_kv_bytes(&c);
          c.workspace = (void*)(((uintptr_t)ws.data() + 255) & ~(uintptr_t)255);
          c.workspace_bytes = oxy_workspace_bytes(&c);
        } else {
          c.flags = OXY_POOL_HOST_ONLY;
        }
        CHECK(oxy_pool_create(&c, &pool) == OXY_OK, "pool_create");
        break;
      }
      case 1: {
        int32_t pid = -1;
        CHECK(oxy_prefix_create(pool, &pid) == OXY_OK && pid == need(), "prefix_create -> %d", pid);
        break;
      }
      case 2: {
        long pid = need(), layer = need(), n = need(), pos0 = need(), exp = need();
        int32_t st = oxy_prefix_append(pool, (int32_t)pid, (int32_t)layer, (void*)16, (void*)16,
                                       (int32_t)n, (int32_t)pos0, nullptr);
        CHECK(st == exp, "prefix_append %d != %ld", st, exp);
        break;
      }
      case 3: {
        long parent = need(), n = need(), exp = need(), exp_pid = need();
        int32_t pid = -1;
        int32_t st = oxy_prefix_fork(pool, (int32_t)parent, (int32_t)n, &pid);
        CHECK(st == exp && (st != OXY_OK || pid == exp_pid), "prefix_fork %d (%d)", st, pid);
        break;
      }
      case 4: {
        long pid = need(), exp = need();
        int32_t st = oxy_prefix_release(pool, (int32_t)pid);
        CHECK(st == exp, "prefix_release %d != %ld", st, exp);
        break;
      }
      case 5: {
        long pid = need(), kind = need(), exp = need(), exp_sid = need();
        int32_t sid = -1;
        int32_t st = oxy_stream_create(pool, (int32_t)pid, (int32_t)kind, &sid);
        CHECK(st == exp && (st != OXY_OK || sid == exp_sid), "stream_create %d (%d)", st, sid);
        break;
      }
      case 6: {
        long sid = need(), exp = need();
        int32_t st = oxy_stream_release(pool, (int32_t)sid);
        CHECK(st == exp, "stream_release %d != %ld", st, exp);
        break;
      }
      case 7: {
        long sid = need(), len = need(), exp = need();
        int32_t st = oxy_stream_rewind(pool, (int32_t)sid, (int32_t)len);
        CHECK(st == exp, "stream_rewind %d != %ld", st, exp);
        break;
      }
      case 8: {
        long flags = need(), n_items = need();
        std::vector<oxy_item> items((size_t)n_items);
        for (auto& it : items) {
          it.stream_id = (int32_t)need();
          it.n_new = (int32_t)need();
        }
        long exp = need(), n_slots = need();
        std::vector<int64_t> exp_slots((size_t)n_slots);
        for (auto& s : exp_slots) s = need();
        oxy_batch* b = nullptr;
        int32_t st = oxy_batch_build(pool, items.data(), (int32_t)n_items, (int32_t)flags, nullptr, &b);
        CHECK(st == exp, "batch_build %d != %ld", st, exp);
        if (st != OXY_OK) break;
        int32_t n_tok = 0, n_work = 0;
        CHECK(oxy_batch_info(b, nullptr, &n_tok, &n_work, nullptr) == OXY_OK && n_tok == n_slots,
              "batch_info: %d tokens, expected %ld", n_tok, n_slots);
        std::vector<int64_t> got((size_t)n_tok + 1);
        CHECK(oxy_batch_slots(b, got.data(), n_tok) == OXY_OK, "batch_slots");
        for (long i = 0; i < n_slots; ++i)
          CHECK(got[i] == exp_slots[i], "slot %ld: %lld != %lld", i, (long long)got[i],
                (long long)exp_slots[i]);
        std::vector<int32_t> work((size_t)n_work * 8 + 8);
        if (!(flags & OXY_BATCH_APPEND_ONLY))
          CHECK(oxy_batch_work(b, work.data(), n_work) == OXY_OK, "batch_work");
        if (device) {   // the launches are stand-ins; what runs is the host side of each call
          void* p = (void*)16;
          CHECK(oxy_stream_append(pool, b, 0, p, p, nullptr) == OXY_OK, "stream_append");
          if (!(flags & OXY_BATCH_APPEND_ONLY)) {
            CHECK(oxy_mixed_attention(pool, b, n_layers - 1, p, p, nullptr, 0.0625f, nullptr) == OXY_OK,
                  "mixed_attention");
            for (int f = 0; f < 8; ++f)   // every launch schedule, issued and recorded
              CHECK(oxy_step_layers(pool, b, 0, n_layers, p, p, 0, p, p, 0, nullptr, 0, 0.0625f, f,
                                    nullptr, nullptr) == OXY_OK, "step_layers flags %d", f);
          }
        }
        CHECK(oxy_batch_destroy(b) == OXY_OK, "batch_destroy");
        break;
      }
      case 9:
      {
        const int skip = (int)need();
        oxy_stub_fail_next(skip, (int)need());
        break;
      }
      case 10: {
        long nb = need();
        std::vector<int32_t> buf((size_t)nb + 1);
        CHECK(oxy_block_refcounts(pool, buf.data(), (int32_t)nb) == OXY_OK, "refcounts");
        for (long i = 0; i < nb; ++i) CHECK(buf[i] == need(), "refcount of block %ld", i);
        long nfree = need();
        int32_t free_now = -1, n_px = -1, n_st = -1;
        CHECK(oxy_pool_stats(pool, &free_now, &n_px, &n_st) == OXY_OK && free_now == nfree,
              "free blocks %d != %ld", free_now, nfree);
        CHECK(oxy_free_blocks(pool, buf.data(), (int32_t)nb) == OXY_OK, "free_blocks");
        for (long i = 0; i < nfree; ++i) CHECK(buf[i] == need(), "free stack position %ld", i);
        long ns = need();
        CHECK(ns == n_st, "live streams %d != %ld", n_st, ns);
        for (long s = 0; s < ns; ++s) {
          long sid = need(), pid = need(), kind = need(), len = need(), nblk = need();
          int32_t g_pid, g_kind, g_len, g_nblk;
          CHECK(oxy_stream_info(pool, (int32_t)sid, &g_pid, &g_kind, &g_len, &g_nblk) == OXY_OK &&
                    g_pid == pid && g_kind == kind && g_len == len && g_nblk == nblk,
                "stream %ld info", sid);
          CHECK(oxy_stream_blocks(pool, (int32_t)sid, buf.data(), (int32_t)nb) == OXY_OK, "stream_blocks");
          for (long i = 0; i < nblk; ++i) CHECK(buf[i] == need(), "stream %ld block %ld", sid, i);
        }
        long np = need();
        CHECK(np == n_px, "live prefixes %d != %ld", n_px, np);
        for (long q = 0; q < np; ++q) {
          long pid = need(), len = need(), nblk = need(), sealed = need(), nstr = need();
          int32_t g_len, g_nblk, g_sealed, g_nstr;
          CHECK(oxy_prefix_info(pool, (int32_t)pid, &g_len, &g_nblk, &g_sealed, &g_nstr) == OXY_OK &&
                    g_len == len && g_nblk == nblk && g_sealed == sealed && g_nstr == nstr,
                "prefix %ld info", pid);
          CHECK(oxy_prefix_blocks(pool, (int32_t)pid, buf.data(), (int32_t)nb) == OXY_OK, "prefix_blocks");
          for (long i = 0; i < nblk; ++i) CHECK(buf[i] == need(), "prefix %ld block %ld", pid, i);
        }
        break;
      }
      default:
        fprintf(stderr, "unknown op %ld at %ld\n", op, g_line);
        return 2;
    }
  }
  if (pool) CHECK(oxy_pool_destroy(pool) == OXY_OK, "pool_destroy");
  printf("OK %ld ops\n", g_line);
  return 0;
}
