/* Drives the host-only paths of the C ABI (argument and state checks, workspace layout, the partitioner)
 * in a build whose host code is compiled with -fsanitize=address,undefined.  Touches no device: every
 * call either fails in validation or does host bookkeeping.  Exit status 0 and the line "sanitize ok"
 * mean that every status was the documented one and the sanitizers reported nothing. */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "lp.h"
#include "lp_measure.h"

static int failures = 0;
#define EXPECT(cond)                                                     \
  do {                                                                   \
    if (!(cond)) {                                                       \
      fprintf(stderr, "line %d: %s\n", __LINE__, #cond);                 \
      ++failures;                                                        \
    }                                                                    \
  } while (0)

static lp_layer_desc linear(int in, int out, int act, int delay) {
  lp_layer_desc d;
  memset(&d, 0, sizeof d);
  d.kind = LP_LINEAR; d.in = in; d.out = out; d.act = act; d.delay = delay;
  return d;
}
static lp_layer_desc conv(int in, int out, int H, int W, int pool, int delay) {
  lp_layer_desc d;
  memset(&d, 0, sizeof d);
  d.kind = LP_CONV3X3; d.in = in; d.out = out; d.H = H; d.W = W; d.act = LP_ACT_RELU; d.pool = pool; d.delay = delay;
  return d;
}

static uint64_t rng_state = 0x9e3779b97f4a7c15ull;
static double uniform(double lo, double hi) {
  rng_state = rng_state * 6364136223846793005ull + 1442695040888963407ull;
  return lo + (hi - lo) * (double)(rng_state >> 11) / 9007199254740992.0;
}

static void create_and_state_errors(void) {
  lp_layer_desc mlp[4] = {linear(784, 256, LP_ACT_RELU, 6), linear(256, 128, LP_ACT_RELU, 4), linear(128, 64, LP_ACT_RELU, 2),
                          linear(64, 10, LP_ACT_IDENTITY, 0)};
  lp_ctx* c = NULL;
  EXPECT(lp_create(NULL, 4, 32, LP_F32, LP_LOSS_SOFTMAX_CE, 0.01f, &c) == LP_ERR_NULL);
  EXPECT(lp_create(mlp, 4, 32, LP_F32, LP_LOSS_SOFTMAX_CE, 0.01f, NULL) == LP_ERR_NULL);
  EXPECT(lp_create(mlp, 0, 32, LP_F32, LP_LOSS_SOFTMAX_CE, 0.01f, &c) == LP_ERR_SHAPE);
  EXPECT(lp_create(mlp, 4, 0, LP_F32, LP_LOSS_SOFTMAX_CE, 0.01f, &c) == LP_ERR_SHAPE);
  EXPECT(lp_create(mlp, 4, 32, 7, LP_LOSS_SOFTMAX_CE, 0.01f, &c) == LP_ERR_DTYPE);
  EXPECT(lp_create(mlp, 4, 32, LP_F32, 9, 0.01f, &c) == LP_ERR_DTYPE);
  lp_layer_desc bad[4];
  memcpy(bad, mlp, sizeof bad); bad[1].in = 255;
  EXPECT(lp_create(bad, 4, 32, LP_F32, LP_LOSS_SOFTMAX_CE, 0.01f, &c) == LP_ERR_LAYER);
  memcpy(bad, mlp, sizeof bad); bad[2].delay = -1;
  EXPECT(lp_create(bad, 4, 32, LP_F32, LP_LOSS_SOFTMAX_CE, 0.01f, &c) == LP_ERR_DELAY);
  memcpy(bad, mlp, sizeof bad); bad[3].act = LP_ACT_RELU;
  EXPECT(lp_create(bad, 4, 32, LP_F32, LP_LOSS_SOFTMAX_CE, 0.01f, &c) == LP_ERR_DTYPE);
  EXPECT(strstr(lp_last_error(NULL), "layer 4") != NULL);
  lp_layer_desc big = linear(32768, 32768, LP_ACT_IDENTITY, 0);
  EXPECT(lp_create(&big, 1, 8, LP_BF16, LP_LOSS_MSE, 0.01f, &c) == LP_ERR_SHAPE);
  EXPECT(c == NULL);

  EXPECT(lp_create(mlp, 4, 32, LP_F32, LP_LOSS_SOFTMAX_CE, 0.01f, &c) == LP_OK && c != NULL);
  size_t bytes = 0;
  EXPECT(lp_workspace_bytes(c, &bytes) == LP_OK && bytes > 0 && bytes % 256 == 0);
  EXPECT(lp_workspace_bytes(NULL, &bytes) == LP_ERR_NULL);
  void* fake = (void*)(uintptr_t)0x10000;   /* never dereferenced */
  EXPECT(lp_forward(c, 1, fake, fake, fake, NULL) == LP_ERR_STATE);
  EXPECT(strstr(lp_last_error(c), "workspace") != NULL);
  EXPECT(lp_bind_workspace(c, NULL, bytes) == LP_ERR_NULL);
  EXPECT(lp_bind_workspace(c, (void*)(uintptr_t)0x10008, bytes) == LP_ERR_WORKSPACE);
  EXPECT(lp_bind_workspace(c, fake, 16) == LP_ERR_WORKSPACE);
  EXPECT(lp_bind_workspace(c, fake, bytes) == LP_OK);
  EXPECT(lp_forward(c, 1, fake, fake, fake, NULL) == LP_ERR_STATE);   /* weights never set */
  EXPECT(lp_forward(c, 0, fake, fake, fake, NULL) == LP_ERR_LAYER);
  EXPECT(lp_forward(c, 5, fake, fake, fake, NULL) == LP_ERR_LAYER);
  EXPECT(lp_forward(c, 1, NULL, fake, fake, NULL) == LP_ERR_NULL);
  EXPECT(lp_forward(c, 1, fake, NULL, NULL, NULL) == LP_ERR_NULL);
  EXPECT(lp_grad_act(c, 2, fake, fake, 10, 5, NULL) == LP_ERR_SHAPE);
  EXPECT(lp_grad_act(c, 2, fake, fake, 0, 257, NULL) == LP_ERR_SHAPE);
  EXPECT(lp_grad_weight(c, 1, NULL, fake, NULL, NULL) == LP_ERR_NULL);
  EXPECT(lp_update(c, 1, NULL, NULL) == LP_ERR_STATE);
  EXPECT(lp_loss_grad(c, NULL, fake, fake, NULL, NULL) == LP_ERR_NULL);
  EXPECT(lp_act_grad(c, 1, NULL, fake, fake, NULL) == LP_ERR_NULL);
  EXPECT(lp_cast(c, NULL, fake, 8, NULL) == LP_ERR_NULL);
  EXPECT(lp_cast(c, (const float*)(uintptr_t)0x10004, fake, 8, NULL) == LP_ERR_SHAPE);
  EXPECT(lp_set_delta_split(c, 1, 8) == LP_ERR_LAYER);
  EXPECT(lp_set_delta_split(c, 2, 256) == LP_ERR_SHAPE);
  EXPECT(lp_set_delta_split(c, 2, 255) == LP_OK);
  void* streams[1] = {NULL};
  EXPECT(lp_step(c, fake, fake, NULL, NULL, streams, 1) == LP_ERR_STATE);
  EXPECT(lp_step(c, NULL, fake, NULL, NULL, streams, 1) == LP_ERR_NULL);
  EXPECT(lp_step(c, fake, fake, NULL, NULL, NULL, 0) == LP_ERR_NULL);
  void* p = NULL;
  size_t n = 0;
  EXPECT(lp_tensor(c, 1, 99, &p, &n) == LP_ERR_DTYPE);
  EXPECT(lp_tensor(c, 1, LP_T_MASTER_W, &p, &n) == LP_OK && n == (size_t)784 * 256 * 4);
  EXPECT(lp_tensor(c, 4, LP_T_DA, &p, &n) == LP_OK && p == NULL);
  long steps = -1;
  EXPECT(lp_step_index(c, &steps) == LP_OK && steps == 0);
  EXPECT(lp_advance(c) == LP_OK && lp_step_index(c, &steps) == LP_OK && steps == 1);
  EXPECT(lp_set_run_ahead(c, 1) == LP_ERR_STATE);
  EXPECT(lp_profile(c, 1) == LP_OK && lp_profile(c, 0) == LP_OK);
  EXPECT(lp_profile_read(c, 77, NULL, NULL, 0) == LP_ERR_DTYPE);
  EXPECT(lp_destroy(c) == LP_OK);
  EXPECT(lp_destroy(NULL) == LP_ERR_NULL);
  EXPECT(lp_probe_mfma(NULL, 0, 1, 1, 0, NULL) == LP_ERR_NULL);
  EXPECT(lp_probe_mfma((float*)fake, 511, 1, 1, 0, NULL) == LP_ERR_SHAPE);
}

static void layouts(void) {
  /* workspace layouts of every option, on a network with rings of different depth */
  lp_layer_desc net[5];
  for (int i = 0; i < 5; ++i) net[i] = linear(i == 0 ? 512 : 1024, i == 4 ? 1000 : 1024, i == 4 ? LP_ACT_IDENTITY : LP_ACT_GELU, 2 * (4 - i));
  lp_ctx* c = NULL;
  EXPECT(lp_create(net, 5, 256, LP_BF16, LP_LOSS_SOFTMAX_CE, 1e-3f, &c) == LP_OK);
  size_t n0 = 0, n1 = 0;
  EXPECT(lp_workspace_bytes(c, &n0) == LP_OK);
  EXPECT(lp_set_run_ahead(c, 1) == LP_OK && lp_workspace_bytes(c, &n1) == LP_OK && n1 > n0);
  EXPECT(lp_set_graphs(c, 1) == LP_ERR_STATE);
  EXPECT(lp_set_run_ahead(c, 0) == LP_OK && lp_workspace_bytes(c, &n1) == LP_OK && n1 == n0);
  EXPECT(lp_set_graphs(c, 1) == LP_OK && lp_workspace_bytes(c, &n1) == LP_OK && n1 > n0);
  EXPECT(lp_set_graphs(c, 0) == LP_OK);
  EXPECT(lp_set_factor_ring(c, 0, 1) == LP_OK && lp_workspace_bytes(c, &n1) == LP_OK && n1 < n0);
  EXPECT(lp_set_factor_ring(c, 9, 1) == LP_ERR_LAYER);
  /* retimed update: weight versions in place of gradients; one kind of delay element per layer */
  void* fake = (void*)(uintptr_t)0x10000;   /* never dereferenced */
  EXPECT(lp_set_retimed_update(c, 2, 1) == LP_ERR_LAYER);
  EXPECT(lp_set_factor_ring(c, 0, 0) == LP_OK && lp_workspace_bytes(c, &n1) == LP_OK && n1 == n0);
  EXPECT(lp_set_retimed_update(c, 0, 1) == LP_OK && lp_workspace_bytes(c, &n1) == LP_OK && n1 < n0);
  EXPECT(lp_set_factor_ring(c, 2, 1) == LP_ERR_LAYER);
  EXPECT(lp_set_retimed_update(c, 9, 1) == LP_ERR_LAYER && lp_set_retimed_update(NULL, 0, 1) == LP_ERR_NULL);
  EXPECT(lp_set_graphs(c, 1) == LP_OK && lp_set_graphs(c, 0) == LP_OK);
  EXPECT(lp_bind_workspace(c, fake, (size_t)1 << 40) == LP_OK);
  EXPECT(lp_set_retimed_update(c, 0, 0) == LP_ERR_STATE);
  {
    void* p0 = NULL; void* p1 = NULL; size_t nb = 0;
    EXPECT(lp_tensor(c, 1, LP_T_WORK_W, &p0, &nb) == LP_OK && p0 != NULL && nb == (size_t)512 * 1024 * 2);
    EXPECT(lp_tensor(c, 4, LP_T_WORK_W, &p1, &nb) == LP_OK && p1 != NULL);
    void* g = fake;
    EXPECT(lp_tensor(c, 1, LP_T_G_LAST, &g, &nb) == LP_OK && g == NULL);
    /* eight steps on: step 9 of layer 1 (d = 8) still reads version 0, layer 4 (d = 2, four slots) version 6 in slot 2; step 10 of layer 1 reads version 1 */
    for (int i = 0; i < 8; ++i) EXPECT(lp_advance(c) == LP_OK);
    void* q0 = NULL; void* q1 = NULL;
    EXPECT(lp_tensor(c, 1, LP_T_WORK_W, &q0, &nb) == LP_OK && q0 == p0);
    EXPECT(lp_tensor(c, 4, LP_T_WORK_W, &q1, &nb) == LP_OK && q1 != p1);
    EXPECT(lp_advance(c) == LP_OK && lp_tensor(c, 1, LP_T_WORK_W, &q0, &nb) == LP_OK && q0 != p0);
    EXPECT(lp_update(c, 1, NULL, NULL) == LP_ERR_STATE);
  }
  long a = -1, b = -1, e = -1;
  EXPECT(lp_graph_stats(c, &a, &b, &e) == LP_OK && a == 0 && b == 0 && e == 0);
  EXPECT(lp_destroy(c) == LP_OK);

  lp_layer_desc cnn[3] = {conv(3, 16, 8, 8, 0, 4), conv(16, 16, 8, 8, 2, 2), linear(4 * 4 * 16, 10, LP_ACT_IDENTITY, 0)};
  EXPECT(lp_create(cnn, 3, 4, LP_BF16, LP_LOSS_SOFTMAX_CE, 1e-3f, &c) == LP_OK);
  EXPECT(lp_set_factor_ring(c, 1, 1) == LP_ERR_LAYER);
  EXPECT(lp_destroy(c) == LP_OK);
  cnn[1].H = 7;
  EXPECT(lp_create(cnn, 3, 4, LP_BF16, LP_LOSS_SOFTMAX_CE, 1e-3f, &c) != LP_OK);
  cnn[1].H = 8;
  EXPECT(lp_create(cnn, 3, 4, LP_F32, LP_LOSS_SOFTMAX_CE, 1e-3f, &c) == LP_ERR_DTYPE);
}

static void partitions(void) {
  double fix[16], flex[16], frac[16], load[9], tp;
  int st[16], rest[16];
  for (int trial = 0; trial < 2000; ++trial) {
    const int L = 1 + (int)uniform(0, 15.99), np = 1 + (int)uniform(0, 8.99);
    double total = 0.0, sum = 0.0;
    for (int l = 0; l < L; ++l) {
      fix[l] = trial % 7 == 0 ? 0.0 : uniform(0.1, 5.0);
      flex[l] = trial % 5 == 0 ? 0.0 : uniform(0.0, 20.0);
      total += fix[l] + flex[l];
    }
    EXPECT(lp_partition(fix, flex, L, np, 1.05, st, rest, frac, load, &tp) == LP_OK);
    for (int s = 0; s < np; ++s) sum += load[s];
    EXPECT(sum <= total * (1 + 1e-9) + 1e-12 && sum >= total * (1 - 1e-9) - 1e-12);
    for (int l = 0; l < L; ++l) EXPECT(st[l] >= 0 && st[l] < np && frac[l] >= 0.0 && frac[l] <= 1.0 && rest[l] >= st[l]);
  }
  EXPECT(lp_partition(NULL, flex, 1, 1, 1.05, st, rest, frac, load, &tp) == LP_ERR_NULL);
  EXPECT(lp_partition(fix, flex, 0, 1, 1.05, st, rest, frac, load, &tp) == LP_ERR_SHAPE);
  EXPECT(lp_partition(fix, flex, 1, 0, 1.05, st, rest, frac, load, &tp) == LP_ERR_SHAPE);
  EXPECT(lp_partition(fix, flex, 1, 1, 1.0, st, rest, frac, load, &tp) == LP_ERR_SHAPE);
  fix[0] = -1.0;
  EXPECT(lp_partition(fix, flex, 1, 1, 1.05, st, rest, frac, load, NULL) == LP_ERR_SHAPE);
}

int main(void) {
  create_and_state_errors();
  layouts();
  partitions();
  if (failures) {
    fprintf(stderr, "%d expectation(s) failed\n", failures);
    return 1;
  }
  puts("sanitize ok");
  return 0;
}
