// Host-side check program for the sanitizer build: linked with the library's own sources compiled with
// AddressSanitizer + UndefinedBehaviorSanitizer on the host side, it drives the planner entry points on inputs
// read from a file and walks the argument checks of every device entry point (calls that are refused before
// anything is launched, so no GPU is needed).  Results go to stdout as integers; a sanitizer report aborts.
#include <cstdio>
#include <cstdlib>
#include <vector>

#include "vlcache.h"

static int planner(const char* path) {
  FILE* f = fopen(path, "r");
  if (!f) return 2;
  int L, G, n_seg, has_k;
  long long budget, cap;
  if (fscanf(f, "%d %d %lld", &L, &G, &budget) != 3) return 2;
  std::vector<double> sens((size_t)L * (G + 1));
  for (auto& v : sens)
    if (fscanf(f, "%lf", &v) != 1) return 2;
  if (fscanf(f, "%d", &n_seg) != 1) return 2;
  std::vector<vlc_segment> seg(n_seg);
  for (auto& s : seg)
    if (fscanf(f, "%d %d %d %d %d %d %d", &s.start, &s.length, &s.is_image, &s.pos, &s.old_pos, &s.cache_row,
               &s.kv_start) != 7)
      return 2;
  if (fscanf(f, "%d %lld", &has_k, &cap) != 2) return 2;
  std::vector<int32_t> sel(L);
  for (auto& v : sel)
    if (fscanf(f, "%d", &v) != 1) return 2;
  fclose(f);

  // exactly-sized buffers: an overrun of one element is a sanitizer report
  std::vector<int32_t> k1(L), k2(L);
  int rc = vlc_plan_layer_rates(L, G, sens.data(), budget, k1.data());
  printf("rates %d", rc);
  for (int v : k1) printf(" %d", v);
  rc = vlc_plan_layer_rates_blocks(L, G, sens.data(), budget, k2.data());
  printf("\nblocks %d", rc);
  for (int v : k2) printf(" %d", v);
  const int32_t* k = has_k ? sel.data() : nullptr;
  const int32_t* over = has_k ? nullptr : sel.data();
  std::vector<int32_t> n_rows(L), slot((size_t)L * cap), map((size_t)L * cap), pos((size_t)L * cap),
      kvs((size_t)L * cap), kvl((size_t)L * cap), nxt((size_t)L * cap, -7);
  rc = vlc_plan_token_indices(n_seg, seg.data(), L, k, over, cap, n_rows.data(), slot.data(), map.data(), pos.data(),
                              kvs.data(), kvl.data());
  printf("\nindices %d", rc);
  if (rc == 0) {
    for (int l = 0; l < L; ++l) {
      printf("\nn %d", n_rows[l]);
      const int32_t* arrs[5] = {slot.data(), map.data(), pos.data(), kvs.data(), kvl.data()};
      for (auto a : arrs) {
        printf("\n");
        for (int i = 0; i < n_rows[l]; ++i) printf("%d ", a[(size_t)l * cap + i]);
      }
    }
    rc = vlc_plan_next_rows(n_seg, seg.data(), L, k, over, cap, nxt.data());
    printf("\nnext %d", rc);
    for (int l = 0; l < L; ++l) {
      printf("\n");
      for (int i = 0; i < n_rows[l]; ++i) printf("%d ", nxt[(size_t)l * cap + i]);
    }
  }
  long long n_img = 0;
  for (auto& s : seg) n_img += s.is_image ? s.length : 0;
  const long long rcap = n_img > 0 ? n_img : 1;
  std::vector<int32_t> n_reuse(L), src((size_t)L * rcap), dst((size_t)L * rcap), dl((size_t)L * rcap);
  rc = vlc_plan_reuse_rows(n_seg, seg.data(), L, k, over, rcap, n_reuse.data(), src.data(), dst.data(), dl.data());
  printf("\nreuse %d", rc);
  if (rc == 0)
    for (int l = 0; l < L; ++l) {
      printf("\nm %d", n_reuse[l]);
      const int32_t* arrs[3] = {src.data(), dst.data(), dl.data()};
      for (auto a : arrs) {
        printf("\n");
        for (int i = 0; i < n_reuse[l]; ++i) printf("%d ", a[(size_t)l * rcap + i]);
      }
    }
  int64_t steps = -1;
  rc = vlc_plan_budget_steps(500, L, &steps);
  printf("\nbudget %d %lld\n", rc, (long long)steps);
  return 0;
}

// Every call below must be refused by the host-side checks (or be a no-op); none may reach a kernel launch.
static int errors() {
  char buf[4096] __attribute__((aligned(256)));
  void* p = buf;                 // a non-NULL, aligned stand-in: refused calls never dereference device pointers
  int32_t i32[8] = {0};
  double sens[6] = {3, 2, 1, 3, 2, 1};
  vlc_segment seg[2] = {{0, 10, 0, 0, 0, 0, 0}, {10, 50, 1, 10, 0, 0, 0}};
  vlc_segment bad_seg[2] = {{0, 10, 0, 0, 0, 0, 0}, {5, 5, 0, 5, 0, 0, 0}};
  int32_t k_up[2] = {10, 20}, k_ok[2] = {20, 10}, k_big[1] = {501};
  int32_t out[2 * 64];
  std::vector<int> rc;
  rc.push_back(vlc_plan_layer_rates(2, 2, nullptr, 3, i32));
  rc.push_back(vlc_plan_layer_rates(0, 2, sens, 3, i32));
  rc.push_back(vlc_plan_layer_rates(2, 501, sens, 3, i32));
  rc.push_back(vlc_plan_layer_rates(2, 2, sens, -1, i32));
  rc.push_back(vlc_plan_layer_rates_blocks(2, 2, sens, -1, i32));
  rc.push_back(vlc_plan_token_indices(2, seg, 2, k_up, nullptr, 64, i32, out, nullptr, nullptr, nullptr, nullptr));
  rc.push_back(vlc_plan_token_indices(2, bad_seg, 1, k_ok, nullptr, 64, i32, out, nullptr, nullptr, nullptr, nullptr));
  rc.push_back(vlc_plan_token_indices(2, seg, 1, k_big, nullptr, 64, i32, out, nullptr, nullptr, nullptr, nullptr));
  rc.push_back(vlc_plan_token_indices(2, seg, 2, k_ok, nullptr, 11, i32, out, nullptr, nullptr, nullptr, nullptr));
  rc.push_back(vlc_plan_token_indices(2, seg, 2, nullptr, nullptr, 64, i32, out, nullptr, nullptr, nullptr, nullptr));
  rc.push_back(vlc_plan_reuse_rows(2, seg, 2, k_ok, nullptr, 10, i32, out, nullptr, nullptr));
  rc.push_back(vlc_plan_next_rows(2, seg, 2, k_ok, nullptr, 11, out));
  rc.push_back(vlc_plan_next_rows(2, seg, 2, k_up, nullptr, 64, out));
  rc.push_back(vlc_plan_budget_steps(-1, 3, nullptr));
  int64_t st = 0;
  rc.push_back(vlc_plan_budget_steps(10001, 3, &st));
  // device entry points: argument checks only
  rc.push_back(vlc_gather_rows(p, 4, 8, i32, 2, p, 7, nullptr));
  rc.push_back(vlc_gather_rows(p, 4, 3, i32, 2, p, VLC_BF16, nullptr));          // 6-byte rows
  rc.push_back(vlc_gather_rows(nullptr, 4, 8, i32, 2, p, VLC_BF16, nullptr));
  rc.push_back(vlc_gather_rows(p, 4, 8, i32, 0, p, VLC_BF16, nullptr));          // no rows: OK
  rc.push_back(vlc_gather_rows(buf + 4, 4, 8, i32, 2, p, VLC_BF16, nullptr));    // misaligned
  rc.push_back(vlc_rope_shift_kv(p, p, p, p, i32, i32, i32, 2, 4, 96, 1e6, VLC_BF16, nullptr));
  rc.push_back(vlc_rope_shift_kv(p, p, p, p, i32, i32, i32, -2, 4, 128, 1e6, VLC_BF16, nullptr));
  rc.push_back(vlc_rope_shift_kv(p, p, p, p, i32, i32, nullptr, 2, 4, 128, 1e6, VLC_BF16, nullptr));
  rc.push_back(vlc_rope_shift_kv(p, p, p, p, i32, i32, i32, 2, 4, 128, -1.0, VLC_BF16, nullptr));
  rc.push_back(vlc_rope_shift_kv_layers(nullptr, 3, 10, 4, 128, 1e6, VLC_BF16, nullptr));
  rc.push_back(vlc_rope_shift_kv_layers((const vlc_shift_job*)(buf + 4), 3, 10, 4, 128, 1e6, VLC_BF16, nullptr));
  rc.push_back(vlc_scatter_kv(p, p, i32, 5, p, p, 4, 4, 128, VLC_BF16, nullptr));   // more rows than the cache
  rc.push_back(vlc_scatter_kv(p, nullptr, i32, 2, p, p, 4, 4, 128, VLC_BF16, nullptr));
  rc.push_back(vlc_sparse_q_attention(p, p, p, i32, i32, 2, 7, 2, 128, 0.1f, p, VLC_BF16, nullptr));  // Hq % Hkv
  rc.push_back(vlc_sparse_q_attention(p, p, p, i32, nullptr, 2, 4, 2, 128, 0.1f, p, VLC_BF16, nullptr));
  rc.push_back(vlc_sparse_q_attention(p, p, p, i32, i32, 0, 4, 2, 128, 0.1f, p, VLC_BF16, nullptr));
  vlc_layer_shape sh = {256, 4, 2, 128, 512, VLC_BF16, 1e-6f, 1e4, 0, 0, 0, 0, 0};
  vlc_layer_shape sh_bad = sh;
  sh_bad.Hkv = 3;
  rc.push_back((int)(vlc_layer_workspace_bytes(&sh_bad, 10) == 0));
  rc.push_back((int)(vlc_layer_workspace_bytes(&sh, 10) > 0));
  rc.push_back((int)(vlc_layer_workspace_bytes(&sh, -1) == 0));
  int64_t offs[VLC_WS_FIELDS];
  rc.push_back(vlc_layer_workspace_layout(&sh, 10, offs));
  rc.push_back(vlc_layer_workspace_layout(&sh, 10, nullptr));
  vlc_layer_weights w = {p, p, nullptr, p, p, p, p, nullptr, nullptr, nullptr};
  vlc_layer_plan plan = {};
  plan.n_in = 4;
  plan.n = 8;   // more rows than the layer above kept
  rc.push_back(vlc_layer_forward(&sh, &w, &plan, p, buf + 256, p, p, p, 4096, nullptr));
  plan.n = 2;   // NULL index arrays
  rc.push_back(vlc_layer_forward(&sh, &w, &plan, p, buf + 256, p, p, p, 4096, nullptr));
  rc.push_back(vlc_layer_forward(&sh, nullptr, &plan, p, buf + 256, p, p, p, 4096, nullptr));
  plan.map = plan.slot = plan.pos = plan.row_kv_start = plan.row_kv_len = i32;
  rc.push_back(vlc_layer_forward(&sh, &w, &plan, p, p, p, p, p, 4096, nullptr));              // h_out aliases h_in
  rc.push_back(vlc_layer_forward(&sh, &w, &plan, p, buf + 256, p, p, p, 16, nullptr));         // workspace too small
  rc.push_back(vlc_layer_forward_timed(&sh, &w, &plan, p, buf + 256, p, p, p, 4096, nullptr, nullptr));
  rc.push_back(vlc_layer_forward_chained(&sh, &w, &plan, p, buf + 256, p, p, p, 4096, nullptr, 2, nullptr, nullptr, nullptr));
  rc.push_back(vlc_first_token(p, i32, 2, 100, 512, 1e-6f, p, p, (float*)p, i32, p, 4096, VLC_F32, nullptr));
  rc.push_back(vlc_first_token(p, i32, 2, 256, 512, 1e-6f, p, p, (float*)p, i32, p, 16, VLC_F32, nullptr));
  rc.push_back(vlc_first_token_noalloc(p, i32, 129, 3584, 152064, 1e-6f, p, p, (float*)p, i32, VLC_BF16, nullptr));
  rc.push_back(vlc_first_token_noalloc(p, i32, 0, 3584, 152064, 1e-6f, p, p, (float*)p, i32, VLC_BF16, nullptr));
  rc.push_back(vlc_mean_squared_error((const float*)p, (const float*)p, 0, (double*)p, p, 8192, nullptr));
  rc.push_back(vlc_mean_squared_error((const float*)p, (const float*)p, 5, (double*)p, p, 8, nullptr));
  double fl = 0;
  rc.push_back(vlc_probe_mfma_bf16(nullptr, 0, nullptr, 0, 10, 1, &fl, nullptr));
  rc.push_back(vlc_probe_mfma_bf16(p, 4096, (float*)p, 1024, 10, 3, &fl, nullptr));
  printf("errors");
  for (int v : rc) printf(" %d", v);
  printf("\n%s\n", vlc_last_error());
  return 0;
}

int main(int argc, char** argv) {
  if (argc >= 3 && argv[1][0] == 'p') return planner(argv[2]);
  if (argc >= 2 && argv[1][0] == 'e') return errors();
  fprintf(stderr, "usage: host_check planner <file> | errors\n");
  return 2;
}
