// Driver of the host-side code of libddit_hot for a CPU-only build with AddressSanitizer and
// UndefinedBehaviorSanitizer on the host code (tests/test_host_sanitizers.py builds and runs it).
// It reads commands from a text file, calls the library's host-only entry points and the validation
// paths of the GPU entry points (which return before any HIP call), and prints what they returned;
// the test compares the printout with the oracle (scheduler, allocator) and with the ordinary build
// of the library (sizes, statuses).  No GPU is needed or touched.
#include <cinttypes>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <string>
#include <vector>

#include "../include/ddit_hot.h"

static ddit_shape make_shape(const long long *v) {
  ddit_shape s;
  memset(&s, 0, sizeof(s));
  s.struct_size = sizeof(s);
  s.flags = (uint32_t)v[0];
  s.B = (int)v[1]; s.T = (int)v[2]; s.Hp = (int)v[3]; s.Wp = (int)v[4]; s.D = (int)v[5]; s.H = (int)v[6];
  s.dh = (int)v[7]; s.M = (int)v[8]; s.Ly = (int)v[9]; s.n_blocks = (int)v[10];
  s.ln_eps = 1e-6f;
  return s;
}

static bool read_ll(FILE *f, long long *out, int n) {
  for (int i = 0; i < n; ++i)
    if (fscanf(f, "%lld", &out[i]) != 1) return false;
  return true;
}

static int do_sched(FILE *f) {
  long long h[7];
  if (!read_ll(f, h, 7)) return 1;
  const int n_gpus = (int)h[0], n_steps = (int)h[1], R = (int)h[2], K = (int)h[3], vae_gpus = (int)h[4];
  const bool has_vae = h[5] != 0;
  const long long max_events = h[6];
  std::vector<int64_t> step((size_t)R * K), vae(R);
  std::vector<int32_t> opt(R);
  long long v;
  for (auto &x : step) { if (!read_ll(f, &v, 1)) return 1; x = v; }
  for (auto &x : opt) { if (!read_ll(f, &v, 1)) return 1; x = (int32_t)v; }
  if (has_vae) for (auto &x : vae) { if (!read_ll(f, &v, 1)) return 1; x = v; }
  if (!read_ll(f, &v, 1)) return 1;
  const int n = (int)v;
  std::vector<ddit_sched_request> rq(n > 0 ? n : 1);
  for (int i = 0; i < n; ++i) {
    long long ar[2];
    if (!read_ll(f, ar, 2)) return 1;
    rq[i].arrival_us = ar[0]; rq[i].resolution = (int32_t)ar[1]; rq[i].reserved = 0;
  }
  ddit_sched_config c;
  memset(&c, 0, sizeof(c));
  c.struct_size = sizeof(c); c.n_gpus = n_gpus; c.n_steps = n_steps; c.n_resolutions = R; c.n_dop = K; c.vae_gpus = vae_gpus;
  c.step_us = step.data(); c.opt_dop = opt.data(); c.vae_us = has_vae ? vae.data() : nullptr;
  // the event array has exactly max_events entries: a write past it is what the sanitizer is here to catch
  std::vector<ddit_sched_record> rec(n > 0 ? n : 1);
  std::vector<ddit_sched_event> ev((size_t)(max_events > 0 ? max_events : 0));
  int64_t n_ev = 0;
  ddit_sched_totals tot;
  const int rc = ddit_sched_simulate(&c, rq.data(), n, rec.data(), max_events > 0 ? ev.data() : nullptr, max_events, &n_ev, &tot);
  printf("sched rc %d\n", rc);
  if (rc != 0) { printf("error %s\n", ddit_last_error()); return 0; }
  for (int i = 0; i < n; ++i)
    printf("rec %" PRId64 " %" PRId64 " %" PRId64 " %d %d %d %" PRId64 "\n", rec[i].start_us, rec[i].dit_end_us, rec[i].end_us,
           rec[i].first_dop, rec[i].final_dop, rec[i].promotions, rec[i].starvation);
  const int64_t shown = n_ev < max_events ? n_ev : max_events;
  for (int64_t i = 0; i < shown; ++i)
    printf("ev %" PRId64 " %d %d %d %d\n", ev[i].time_us, ev[i].kind, ev[i].request, ev[i].gpu_start, ev[i].gpu_count);
  printf("tot %" PRId64 " %" PRId64 " %" PRId64 "\n", tot.occupancy_gpu_us, tot.makespan_us, n_ev);
  return 0;
}

static int do_buddy(FILE *f) {
  long long h[2];
  if (!read_ll(f, h, 2)) return 1;
  void *pool = nullptr;
  int rc = ddit_buddy_create((int32_t)h[0], &pool);
  printf("buddy create %d\n", rc);
  if (rc != 0) return 0;
  for (long long i = 0; i < h[1]; ++i) {
    char op[8];
    if (fscanf(f, "%7s", op) != 1) return 1;
    if (op[0] == 'a') {
      long long s;
      if (!read_ll(f, &s, 1)) return 1;
      int32_t start = -2;
      rc = ddit_buddy_alloc(pool, (int32_t)s, &start);
      printf("a %d %d\n", rc, start);
    } else if (op[0] == 'r') {
      long long a[2];
      if (!read_ll(f, a, 2)) return 1;
      printf("r %d\n", ddit_buddy_release(pool, (int32_t)a[0], (int32_t)a[1]));
    } else {
      int32_t fr = -1;
      rc = ddit_buddy_free_gpus(pool, &fr);
      printf("f %d %d\n", rc, fr);
    }
  }
  printf("buddy destroy %d\n", ddit_buddy_destroy(pool));
  return 0;
}

static int do_dop(FILE *f) {
  long long h[3];
  if (!read_ll(f, h, 3)) return 1;
  std::vector<int64_t> row((size_t)h[0]);
  long long v;
  for (auto &x : row) { if (!read_ll(f, &v, 1)) return 1; x = v; }
  int32_t out = -1;
  const int rc = ddit_optimal_dop(row.data(), (int32_t)h[0], h[1], h[2], &out);
  printf("dop %d %d\n", rc, out);
  return 0;
}

// sizes and tap regions of a shape, and the statuses of every GPU entry point's validation path on it
static int do_shape(FILE *f) {
  long long v[11];
  if (!read_ll(f, v, 11)) return 1;
  ddit_shape s = make_shape(v);
  size_t bytes = 0, kv = 0;
  int rc = ddit_workspace_bytes(&s, &bytes);
  printf("shape ws %d %zu\n", rc, rc == 0 ? bytes : (size_t)0);
  const int rk = ddit_cross_kv_bytes(&s, &kv);
  printf("shape kv %d %zu\n", rk, rk == 0 ? kv : (size_t)0);
  if (s.flags & DDIT_FLAG_TAPS) {
    for (int layer = 0; layer < 2; ++layer)
      for (int t = 0; t < DDIT_TAP_COUNT; ++t) {
        size_t off = 0, nb = 0;
        const int rt = ddit_tap_region(&s, layer, t, &off, &nb);
        printf("tap %d %d %d %zu %zu\n", layer, t, rt, rt == 0 ? off : (size_t)0, rt == 0 ? nb : (size_t)0);
      }
  }
  ddit_io_weights io;
  memset(&io, 0, sizeof(io));
  io.struct_size = sizeof(io); io.C_in = 4; io.C_out = 4; io.C_text = 64;
  size_t iob = 0;
  const int ri = ddit_io_workspace_bytes(&s, &io, &iob);
  printf("shape io %d %zu\n", ri, ri == 0 ? iob : (size_t)0);
  // validation paths: a host buffer stands in for device memory, nothing is launched because every call below
  // is refused (NULL weights, workspace too small, misaligned pointer, bad valid length)
  alignas(256) static unsigned char buf[4096];
  int32_t bad_len[64];
  for (int i = 0; i < 64; ++i) bad_len[i] = 0;
  ddit_block_weights bw;
  memset(&bw, 0, sizeof(bw));
  ddit_step_weights sw;
  memset(&sw, 0, sizeof(sw));
  float ts[64] = {0};
  printf("v block_null %d\n", ddit_stdit_block_fwd(&s, nullptr, buf, buf, nullptr, (const float *)buf, buf, buf, sizeof(buf), nullptr));
  printf("v block_ws %d\n", ddit_stdit_block_fwd(&s, &bw, buf, buf, nullptr, (const float *)buf, buf, buf, 16, nullptr));
  printf("v block_static_null %d\n", ddit_stdit_block_fwd_static(&s, nullptr, buf, buf, nullptr, (const float *)buf, buf, nullptr));
  printf("v step_null %d\n", ddit_denoise_step(&s, nullptr, buf, buf, nullptr, ts, nullptr, buf, buf, sizeof(buf), nullptr));
  printf("v step_ws %d\n", ddit_denoise_step(&s, &sw, buf, buf, nullptr, ts, nullptr, buf, nullptr, 0, nullptr));
  printf("v step_misaligned %d\n", ddit_denoise_step(&s, &sw, buf + 2, buf, nullptr, ts, nullptr, buf, buf, sizeof(buf), nullptr));
  printf("v attn_null %d\n", ddit_attn_fwd(DDIT_ATTN_SPATIAL, &s, nullptr, buf, buf, 8, 8, nullptr, buf, 8, nullptr, nullptr, 0, nullptr));
  printf("v attn_ld %d\n", ddit_attn_fwd(DDIT_ATTN_CROSS, &s, buf, buf, buf, 8, 8, nullptr, buf, 8, nullptr, nullptr, 0, nullptr));
  printf("v attn_len %d\n", ddit_attn_fwd(DDIT_ATTN_CROSS, &s, buf, buf, buf, 1 << 20, 1 << 20, bad_len, buf, 1 << 20, nullptr, nullptr, 0, nullptr));
  printf("v attn_kind %d\n", ddit_attn_fwd((ddit_attn_kind)3, &s, buf, buf, buf, 1 << 20, 1 << 20, nullptr, buf, 1 << 20, nullptr, nullptr, 0, nullptr));
  printf("v kv_null %d\n", ddit_cross_kv_precompute(&s, nullptr, buf, buf, nullptr));
  printf("v sample_steps %d\n", ddit_sample(&s, &sw, &io, (float *)buf, buf, nullptr, nullptr, nullptr, nullptr, 1.0f, 0, 0, 0, (float *)buf, buf, sizeof(buf), nullptr));
  printf("v eps_ws %d\n", ddit_eps_theta(&s, &sw, &io, (const float *)buf, buf, nullptr, nullptr, ts, (float *)buf, buf, 16, nullptr));
  return 0;
}

static int do_linear(FILE *f) {
  long long v[5];
  if (!read_ll(f, v, 5)) return 1;   // epilogue N n k compute_units
  const int nt = ddit_linear_tile_count();
  std::vector<float> us((size_t)nt);
  int32_t tile = -1;
  const int rc = ddit_linear_tile_choice((int)v[0], v[1], (int32_t)v[2], (int32_t)v[3], (int32_t)v[4], &tile, us.data());
  printf("tile %d %d", rc, tile);
  for (int t = 0; t < nt; ++t) printf(" %.4f", us[t]);
  printf("\n");
  // the linear's own validation: refused before any launch
  alignas(16) static unsigned char buf[64];
  printf("v linear_null %d\n", ddit_linear_fwd((int)v[0], nullptr, 8, buf, nullptr, 8, 8, 8, buf, 8, nullptr, nullptr, nullptr, -1, 1, nullptr));
  printf("v linear_dims %d\n", ddit_linear_fwd(0, buf, 8, buf, nullptr, 8, 12, 8, buf, 16, nullptr, nullptr, nullptr, -1, 1, nullptr));
  printf("v linear_align %d\n", ddit_linear_fwd(0, buf + 2, 8, buf, nullptr, 8, 8, 8, buf, 8, nullptr, nullptr, nullptr, -1, 1, nullptr));
  printf("v linear_zero_rows %d\n", ddit_linear_fwd(0, buf, 8, buf, nullptr, 0, 8, 8, buf, 8, nullptr, nullptr, nullptr, -1, 1, nullptr));
  return 0;
}

int main(int argc, char **argv) {
  if (argc != 2) { fprintf(stderr, "usage: %s commands.txt\n", argv[0]); return 2; }
  FILE *f = fopen(argv[1], "r");
  if (!f) { perror("open"); return 2; }
  printf("abi %u tiles %d\n", ddit_abi_version(), ddit_linear_tile_count());
  char cmd[16];
  int bad = 0;
  while (!bad && fscanf(f, "%15s", cmd) == 1) {
    if (!strcmp(cmd, "SCHED")) bad = do_sched(f);
    else if (!strcmp(cmd, "BUDDY")) bad = do_buddy(f);
    else if (!strcmp(cmd, "DOP")) bad = do_dop(f);
    else if (!strcmp(cmd, "SHAPE")) bad = do_shape(f);
    else if (!strcmp(cmd, "LINEAR")) bad = do_linear(f);
    else bad = 1;
  }
  fclose(f);
  if (bad) { fprintf(stderr, "malformed command file near '%s'\n", cmd); return 2; }
  printf("done\n");
  return 0;
}
