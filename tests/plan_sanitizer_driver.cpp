// Drives the host-side planning of libfastcache (csrc/fc_plan.cpp: validation,
// prefix sums, descriptors, work lists) with cases read from stdin and prints
// every plan as text, in a build with AddressSanitizer and
// UndefinedBehaviorSanitizer; the sanitizers abort on any finding.  Built, fed
// and checked by test_plan_sanitizers.py.
//
// Input, one case per block of lines (all integers):
//   compress nl nh d n_free mode in_place n_req max_blocks per_req
//            window pool_kernel need_lse q_ok lse_ok null_mask
//     then lines: seq_lens, methods, budgets, and with per_req = 1 windows, pool_kernels
//   lse nl nh d n_req max_blocks window has_method        then seq_lens [, methods]
//   mlp nl nh d n_free n_req max_blocks k tile_rows has_enable   then lens, begins, ends [, enable]
//   append nl nh d n_free n_req max_blocks has_enable     then lens [, enable]
//   decode nl nh d n_req max_blocks has_budget            then lens [, budgets]
#include <cstdint>
#include <cstdio>
#include <string>
#include <vector>

#include "../paper_2503_08461_amd/csrc/fc_plan.h"

using namespace fc;

static bool read_ints(std::vector<int32_t>* v, int n) {
  v->resize(n);
  for (int i = 0; i < n; ++i) {
    long long x;
    if (scanf("%lld", &x) != 1) return false;
    (*v)[i] = (int32_t)x;
  }
  return true;
}

static void print_desc(const ReqDesc& d) {
  printf("D %d %d %d %d %d %d %d %d %lld %lld %lld %lld %d %d %d %d %d %d %d\n", d.table_row,
         d.seq_len, d.budget, d.method, d.n_old, d.n_new, d.old_off, d.new_off,
         (long long)d.score_off, (long long)d.raw_off, (long long)d.kept_off, (long long)d.q_off,
         d.window, d.pool_kernel, d.img_begin, d.img_end, d.chunks_text0, d.chunks_image,
         d.chunks_text1);
}

int main() {
  char kind[32];
  while (scanf("%31s", kind) == 1) {
    const std::string k = kind;
    PoolView pv;
    if (k == "compress") {
      int mode, in_place, n_req, max_blocks, per_req, need_lse, q_ok, lse_ok, null_mask;
      CompressArgs a;
      if (scanf("%d %d %d %d %d %d %d %d %d %d %d %d %d %d %d", &pv.n_layers, &pv.n_heads,
                &pv.head_dim, &pv.n_free, &mode, &in_place, &n_req, &max_blocks, &per_req,
                &a.window, &a.pool_kernel, &need_lse, &q_ok, &lse_ok, &null_mask) != 15)
        return 2;
      pv.score_mode = mode;
      pv.in_place = in_place != 0;
      std::vector<int32_t> lens, methods, budgets, windows, pks;
      const int n = n_req > 0 ? n_req : 0;
      if (!read_ints(&lens, n) || !read_ints(&methods, n) || !read_ints(&budgets, n)) return 2;
      if (per_req && (!read_ints(&windows, n) || !read_ints(&pks, n))) return 2;
      a.n_req = n_req;
      a.max_blocks = max_blocks;
      a.seq_lens = (null_mask & 1) ? nullptr : lens.data();
      a.method = (null_mask & 2) ? nullptr : methods.data();
      a.budget = (null_mask & 4) ? nullptr : budgets.data();
      a.window_per_req = per_req ? windows.data() : nullptr;
      a.pool_kernel_per_req = (per_req && !(null_mask & 8)) ? pks.data() : nullptr;
      a.need_lse = need_lse != 0;
      a.q_ok = q_ok != 0;
      a.lse_ok = lse_ok != 0;
      CompressPlan plan;
      const int rc = plan_compress(pv, a, &plan);
      printf("R %d %d %d %d %d %d %zu %zu %zu %d %zu\n", rc, plan.code, plan.total_new,
             plan.total_old, plan.total_released, plan.top_after, plan.kept_entries,
             plan.score_entries, plan.raw_floats, plan.window_hi, plan.descs.size());
      if (rc != PLAN_OK) continue;
      for (const ReqDesc& d : plan.descs) print_desc(d);
      for (int i = 0; i < N_LISTS; ++i) {
        printf("L %d %d %zu", i, plan.max_len[i], plan.lists[i].size());
        for (int32_t x : plan.lists[i]) printf(" %d", x);
        printf("\n");
      }
    } else if (k == "lse") {
      int n_req, max_blocks, window, has_method;
      if (scanf("%d %d %d %d %d %d %d", &pv.n_layers, &pv.n_heads, &pv.head_dim, &n_req,
                &max_blocks, &window, &has_method) != 7)
        return 2;
      std::vector<int32_t> lens, methods;
      const int n = n_req > 0 ? n_req : 0;
      if (!read_ints(&lens, n) || (has_method && !read_ints(&methods, n))) return 2;
      LsePlan plan;
      const int rc = plan_window_lse(pv, n_req, max_blocks, lens.data(),
                                     has_method ? methods.data() : nullptr, window, &plan);
      printf("R %d %zu\n", rc, plan.descs.size());
      if (rc == PLAN_OK)
        for (const ReqDesc& d : plan.descs) print_desc(d);
    } else if (k == "mlp") {
      int n_req, max_blocks, kk, tile_rows, has_enable;
      if (scanf("%d %d %d %d %d %d %d %d %d", &pv.n_layers, &pv.n_heads, &pv.head_dim, &pv.n_free,
                &n_req, &max_blocks, &kk, &tile_rows, &has_enable) != 9)
        return 2;
      std::vector<int32_t> lens, ib, ie, en;
      const int n = n_req > 0 ? n_req : 0;
      if (!read_ints(&lens, n) || !read_ints(&ib, n) || !read_ints(&ie, n) ||
          (has_enable && !read_ints(&en, n)))
        return 2;
      MlpPlan plan;
      const int rc = plan_mlp(pv, n_req, max_blocks, lens.data(), ib.data(), ie.data(),
                              has_enable ? en.data() : nullptr, kk, tile_rows, &plan);
      printf("R %d %d %d %lld %d %zu %zu\n", rc, plan.total_new, plan.total_old, plan.n_tiles,
             plan.top_after, plan.descs.size(), plan.jobs.size());
      if (rc != PLAN_OK) continue;
      for (const ReqDesc& d : plan.descs) print_desc(d);
      for (const MlpJob& j : plan.jobs) printf("J %d %d %d %d\n", j.desc, j.modality, j.chunks, j.tile_start);
    } else if (k == "append" || k == "decode") {
      int n_req, max_blocks, has_extra;
      if (k == "append") {
        if (scanf("%d %d %d %d %d %d %d", &pv.n_layers, &pv.n_heads, &pv.head_dim, &pv.n_free,
                  &n_req, &max_blocks, &has_extra) != 7)
          return 2;
      } else if (scanf("%d %d %d %d %d %d", &pv.n_layers, &pv.n_heads, &pv.head_dim, &n_req,
                       &max_blocks, &has_extra) != 6) {
        return 2;
      }
      std::vector<int32_t> lens, extra;
      const int n = n_req > 0 ? n_req : 0;
      if (!read_ints(&lens, n) || (has_extra && !read_ints(&extra, n))) return 2;
      DecodePlan plan;
      const int rc = k == "append"
                         ? plan_append(pv, n_req, max_blocks, lens.data(),
                                       has_extra ? extra.data() : nullptr, &plan)
                         : plan_decode_attention(pv, n_req, max_blocks, lens.data(),
                                                 has_extra ? extra.data() : nullptr, &plan);
      printf("R %d %d %zu %zu\n", rc, plan.n_pop, plan.kept_entries, plan.reqs.size());
      if (rc != PLAN_OK) continue;
      for (const DecodeReq& q : plan.reqs)
        printf("Q %d %d %d %lld\n", q.table_row, q.seq_len, q.pop_index, (long long)q.kept_off);
    } else {
      return 3;
    }
  }
  return 0;
}
