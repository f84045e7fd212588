/*
 * A plain C client of include/dfx.h: no Python, no PyTorch, device memory from hipMalloc.
 * Two checks through the C ABI alone, with int32 data whose sums are exact in any order:
 *   1. the circular wait of Sec. 2.3 / Sec. 6.1 (two all-reduces issued in opposite orders on
 *      two vranks) completes, with the right sums;
 *   2. an 8-vrank all-reduce with a ragged length (several channels, a sub-vector tail), a
 *      reduce-scatter with the direct steps and a broadcast, submitted in descending rank order, as rings
 *      and chains through the connectors' FIFOs;
 *   3. the library's defaults (fold steps at this size): a small 8-vrank all-reduce two hundred times inside a
 *      resident daemon, values checked after the last one; prints the best host-to-host time.
 * Expected values are the definitions written out (element-wise wraparound sums, copies).
 * Exit status 0 = all good; anything else names the failing step on stderr.
 */
#define _POSIX_C_SOURCE 200809L   /* clock_gettime under -std=c11 */
#include <hip/hip_runtime_api.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>
#include <time.h>

#include "dfx.h"

#define CHECK_HIP(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { fprintf(stderr, "%s: %s\n", #x, hipGetErrorString(e_)); return 2; } } while (0)
#define CHECK_DFX(x) do { int s_ = (x); if (s_ != DFX_OK) { fprintf(stderr, "%s: %s (%d)\n", #x, dfx_strerror(s_), s_); return 3; } } while (0)

static uint32_t rng_state = 12345u;
static int32_t next_value(void) {   /* xorshift32, values in [-2^20, 2^20) */
  rng_state ^= rng_state << 13; rng_state ^= rng_state >> 17; rng_state ^= rng_state << 5;
  return (int32_t)(rng_state & 0x1fffffu) - (1 << 20);
}

/* host copies of R send buffers of n elements each, and their device twins */
typedef struct { int R; size_t n; int32_t** host; int32_t** dev; } bufs;

static int bufs_make(bufs* b, int R, size_t n, int fill_random) {
  b->R = R; b->n = n;
  b->host = (int32_t**)calloc((size_t)R, sizeof(int32_t*));
  b->dev = (int32_t**)calloc((size_t)R, sizeof(int32_t*));
  for (int r = 0; r < R; ++r) {
    b->host[r] = (int32_t*)malloc(n * sizeof(int32_t));
    for (size_t i = 0; i < n; ++i) b->host[r][i] = fill_random ? next_value() : -7;
    CHECK_HIP(hipMalloc((void**)&b->dev[r], n * sizeof(int32_t)));
    CHECK_HIP(hipMemcpy(b->dev[r], b->host[r], n * sizeof(int32_t), hipMemcpyHostToDevice));
  }
  return 0;
}

static int bufs_fetch(bufs* b) {
  for (int r = 0; r < b->R; ++r) CHECK_HIP(hipMemcpy(b->host[r], b->dev[r], b->n * sizeof(int32_t), hipMemcpyDeviceToHost));
  return 0;
}

static void bufs_free(bufs* b) {
  for (int r = 0; r < b->R; ++r) { free(b->host[r]); (void)hipFree(b->dev[r]); }
  free(b->host); free(b->dev);
}

static int circular_wait(void) {
  const int R = 2; const size_t n = 1024;
  bufs sa, sb, ra, rb;
  if (bufs_make(&sa, R, n, 1) || bufs_make(&sb, R, n, 1) || bufs_make(&ra, R, n, 0) || bufs_make(&rb, R, n, 0)) return 2;
  dfx_ctx* ctx = NULL;
  CHECK_DFX(dfx_init(&ctx, R, NULL, NULL));
  CHECK_DFX(dfx_prepare(ctx, 0, DFX_ALLREDUCE, n, DFX_I32, DFX_SUM, 0, 0));
  CHECK_DFX(dfx_prepare(ctx, 1, DFX_ALLREDUCE, n, DFX_I32, DFX_SUM, 0, 0));
  /* rank 0: A then B; rank 1: B then A */
  CHECK_DFX(dfx_submit(ctx, 0, 0, sa.dev[0], ra.dev[0]));
  CHECK_DFX(dfx_submit(ctx, 0, 1, sb.dev[0], rb.dev[0]));
  CHECK_DFX(dfx_submit(ctx, 1, 1, sb.dev[1], rb.dev[1]));
  CHECK_DFX(dfx_submit(ctx, 1, 0, sa.dev[1], ra.dev[1]));
  CHECK_DFX(dfx_wait(ctx, 0, 0, 10000000000ull));
  CHECK_DFX(dfx_wait_all(ctx, 10000000000ull));
  CHECK_DFX(dfx_finalize(ctx));
  if (bufs_fetch(&ra) || bufs_fetch(&rb)) return 2;
  for (int r = 0; r < R; ++r)
    for (size_t i = 0; i < n; ++i) {
      const int32_t wa = (int32_t)((uint32_t)sa.host[0][i] + (uint32_t)sa.host[1][i]);
      const int32_t wb = (int32_t)((uint32_t)sb.host[0][i] + (uint32_t)sb.host[1][i]);
      if (ra.host[r][i] != wa || rb.host[r][i] != wb) { fprintf(stderr, "circular wait: wrong value at rank %d element %zu\n", r, i); return 4; }
    }
  bufs_free(&sa); bufs_free(&sb); bufs_free(&ra); bufs_free(&rb);
  return 0;
}

static int eight_ranks(void) {
  const int R = 8; const size_t n = 300007, blk = 65536;   /* blk * 4 bytes is a 16-byte multiple: direct reduce-scatter */
  const int root = 5;
  bufs s, r_ar, s_rs, r_rs, r_bc;
  if (bufs_make(&s, R, n, 1) || bufs_make(&r_ar, R, n, 0) || bufs_make(&s_rs, R, blk * R, 1) || bufs_make(&r_rs, R, blk, 0) || bufs_make(&r_bc, R, n, 0)) return 2;
  dfx_config cfg;
  memset(&cfg, 0, sizeof(cfg));
  CHECK_DFX(dfx_config_default(&cfg));
  cfg.direct_min_bytes = 0;   /* direct steps at every size */
  cfg.fold_max_bytes = 0;     /* rings and chains through the FIFOs */
  dfx_ctx* ctx = NULL;
  CHECK_DFX(dfx_init(&ctx, R, &cfg, NULL));
  CHECK_DFX(dfx_prepare(ctx, 0, DFX_ALLREDUCE, n, DFX_I32, DFX_SUM, 0, 0));
  CHECK_DFX(dfx_prepare(ctx, 1, DFX_REDUCESCATTER, blk, DFX_I32, DFX_SUM, 0, 0));
  CHECK_DFX(dfx_prepare(ctx, 2, DFX_BROADCAST, n, DFX_I32, DFX_SUM, root, 0));
  for (int r = R - 1; r >= 0; --r) {
    const int order[3] = {(r + 0) % 3, (r + 1) % 3, (r + 2) % 3};   /* every rank its own order */
    for (int k = 0; k < 3; ++k) {
      const int id = order[k];
      const void* sp = id == 1 ? (const void*)s_rs.dev[r] : (const void*)s.dev[r];
      void* rp = id == 0 ? (void*)r_ar.dev[r] : id == 1 ? (void*)r_rs.dev[r] : (void*)r_bc.dev[r];
      CHECK_DFX(dfx_submit(ctx, r, id, sp, rp));
    }
  }
  CHECK_DFX(dfx_wait_all(ctx, 20000000000ull));
  dfx_cqe cq[8];
  if (dfx_poll(ctx, 0, cq, 8) != 0) { fprintf(stderr, "completions left over after dfx_wait_all\n"); return 4; }
  dfx_stats_t st;
  CHECK_DFX(dfx_stats(ctx, 3, &st));
  if (st.cqe_posted != 3) { fprintf(stderr, "vrank 3 posted %llu completions, not 3\n", (unsigned long long)st.cqe_posted); return 4; }
  CHECK_DFX(dfx_finalize(ctx));
  if (bufs_fetch(&r_ar) || bufs_fetch(&r_rs) || bufs_fetch(&r_bc)) return 2;
  for (size_t i = 0; i < n; ++i) {
    uint32_t w = 0;
    for (int q = 0; q < R; ++q) w += (uint32_t)s.host[q][i];
    for (int r = 0; r < R; ++r) {
      if (r_ar.host[r][i] != (int32_t)w) { fprintf(stderr, "all-reduce: wrong value at rank %d element %zu\n", r, i); return 4; }
      if (r_bc.host[r][i] != s.host[root][i]) { fprintf(stderr, "broadcast: wrong value at rank %d element %zu\n", r, i); return 4; }
    }
  }
  for (int r = 0; r < R; ++r)
    for (size_t i = 0; i < blk; ++i) {
      uint32_t w = 0;
      for (int q = 0; q < R; ++q) w += (uint32_t)s_rs.host[q][(size_t)r * blk + i];
      if (r_rs.host[r][i] != (int32_t)w) { fprintf(stderr, "reduce-scatter: wrong value at rank %d element %zu\n", r, i); return 4; }
    }
  bufs_free(&s); bufs_free(&r_ar); bufs_free(&s_rs); bufs_free(&r_rs); bufs_free(&r_bc);
  return 0;
}

static double now_us(void) {
  struct timespec t;
  clock_gettime(CLOCK_MONOTONIC, &t);
  return (double)t.tv_sec * 1e6 + (double)t.tv_nsec * 1e-3;
}

static int small_allreduce_latency(void) {
  const int R = 8; const size_t n = 2048;   /* 8 KiB per rank */
  bufs s, d;
  if (bufs_make(&s, R, n, 1) || bufs_make(&d, R, n, 0)) return 2;
  dfx_config cfg;
  memset(&cfg, 0, sizeof(cfg));
  CHECK_DFX(dfx_config_default(&cfg));
  cfg.quit_idle_us = 0;       /* the daemon stays resident between the invocations */
  dfx_ctx* ctx = NULL;
  CHECK_DFX(dfx_init(&ctx, R, &cfg, NULL));
  CHECK_DFX(dfx_prepare(ctx, 0, DFX_ALLREDUCE, n, DFX_I32, DFX_SUM, 0, 0));
  const void* sp[8]; void* rp[8];
  for (int r = 0; r < R; ++r) { sp[r] = s.dev[r]; rp[r] = d.dev[r]; }
  double best = 1e30;
  for (int it = 0; it < 200; ++it) {
    const double t0 = now_us();
    CHECK_DFX(dfx_submit_all(ctx, 0, sp, rp, 10000000000ull));
    CHECK_DFX(dfx_wait_all(ctx, 10000000000ull));
    const double dt = now_us() - t0;
    if (dt < best) best = dt;
  }
  CHECK_DFX(dfx_finalize(ctx));
  if (bufs_fetch(&d)) return 2;
  for (size_t i = 0; i < n; ++i) {
    uint32_t w = 0;
    for (int q = 0; q < R; ++q) w += (uint32_t)s.host[q][i];
    for (int r = 0; r < R; ++r)
      if (d.host[r][i] != (int32_t)w) { fprintf(stderr, "small all-reduce: wrong value at rank %d element %zu\n", r, i); return 4; }
  }
  printf("small all-reduce ok: 8 KiB x 8 vranks, best of 200 host-to-host %.1f us\n", best);
  bufs_free(&s); bufs_free(&d);
  return 0;
}

int main(void) {
  int rc = circular_wait();
  if (rc) return rc;
  printf("circular wait ok\n"); fflush(stdout);
  rc = eight_ranks();
  if (rc) return rc;
  printf("eight ranks ok\n"); fflush(stdout);
  rc = small_allreduce_latency();
  if (rc) return rc;
  return 0;
}
