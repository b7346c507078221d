/* Plain C99 client of include/normtest.h, built and run by tests/test_library_host.py: the header must compile
 * as C, the host-only entry points must be callable without a GPU, and the struct layouts printed here are
 * compared with the ctypes mirror in the Python binding. */
#include <stddef.h>
#include <stdio.h>
#include <string.h>

#include "normtest.h"

#define FIELD(T, f) printf("field " #T " " #f " %zu %zu\n", offsetof(T, f), sizeof(((T*)0)->f))

int main(void) {
  printf("size nt_hyper %zu\n", sizeof(nt_hyper));
  FIELD(nt_hyper, lr); FIELD(nt_hyper, beta1); FIELD(nt_hyper, beta2); FIELD(nt_hyper, eps);
  FIELD(nt_hyper, weight_decay); FIELD(nt_hyper, eta); FIELD(nt_hyper, step); FIELD(nt_hyper, b_k);
  FIELD(nt_hyper, b_max); FIELD(nt_hyper, round_to); FIELD(nt_hyper, ddof); FIELD(nt_hyper, flags);
  printf("size nt_shard_info %zu\n", sizeof(nt_shard_info));
  FIELD(nt_shard_info, shard_id); FIELD(nt_shard_info, num_shards); FIELD(nt_shard_info, shard_offset);
  FIELD(nt_shard_info, d_global);
  printf("size nt_result %zu\n", sizeof(nt_result));
  FIELD(nt_result, A); FIELD(nt_result, B); FIELD(nt_result, C); FIELD(nt_result, A_lo); FIELD(nt_result, B_lo);
  FIELD(nt_result, C_lo); FIELD(nt_result, gbar_sq); FIELD(nt_result, var_l1); FIELD(nt_result, T);
  FIELD(nt_result, clip_coef); FIELD(nt_result, next_b); FIELD(nt_result, coord_fail); FIELD(nt_result, pass);
  FIELD(nt_result, status); FIELD(nt_result, coord_max_ratio);
  printf("size nt_layer_stats %zu\n", sizeof(nt_layer_stats));
  FIELD(nt_layer_stats, A); FIELD(nt_layer_stats, B); FIELD(nt_layer_stats, C); FIELD(nt_layer_stats, gbar_sq);
  FIELD(nt_layer_stats, var_l1); FIELD(nt_layer_stats, T); FIELD(nt_layer_stats, n);
  FIELD(nt_layer_stats, coord_fail); FIELD(nt_layer_stats, pass); FIELD(nt_layer_stats, status);
  FIELD(nt_layer_stats, coord_max_ratio);
  printf("enum NT_F32 %d\nenum NT_BF16 %d\n", (int)NT_F32, (int)NT_BF16);
  printf("enum NT_DO_STATS %u\nenum NT_DO_ADAMW %u\nenum NT_PARTIAL %u\nenum NT_WRITE_GBAR %u\nenum NT_COORD_TEST %u\n"
         "enum NT_ONE_PASS %u\n",
         NT_DO_STATS, NT_DO_ADAMW, NT_PARTIAL, NT_WRITE_GBAR, NT_COORD_TEST, NT_ONE_PASS);
  printf("enum NT_STATUS_NONFINITE %u\nenum NT_STATUS_ZERO_GRAD_NORM %u\nenum NT_STATUS_CLAMPED %u\n"
         "enum NT_STATUS_PARTIAL_ONLY %u\nenum NT_STATUS_T_SATURATED %u\nenum NT_STATUS_NO_STATS %u\n"
         "enum NT_STATUS_BAD_RANGE %u\n",
         NT_STATUS_NONFINITE, NT_STATUS_ZERO_GRAD_NORM, NT_STATUS_CLAMPED, NT_STATUS_PARTIAL_ONLY,
         NT_STATUS_T_SATURATED, NT_STATUS_NO_STATS, NT_STATUS_BAD_RANGE);
  printf("enum NT_OK %d\nenum NT_ERR_BAD_ARG %d\nenum NT_ERR_UNSUPPORTED %d\nenum NT_ERR_WORKSPACE_TOO_SMALL %d\n"
         "enum NT_ERR_TOO_LARGE %d\nenum NT_ERR_HIP_BASE %d\n",
         NT_OK, NT_ERR_BAD_ARG, NT_ERR_UNSUPPORTED, NT_ERR_WORKSPACE_TOO_SMALL, NT_ERR_TOO_LARGE, NT_ERR_HIP_BASE);

  /* host-only calls: two shards of the hand example g_1=(1,2), g_2=(3,6) split per coordinate
   * (coordinate 1: A=10, B=16, C=2; coordinate 2: A=40, B=64, C=8), eta=0.5, ddof=1: T = 10/(0.25*20) = 2 */
  {
    nt_result parts[2], out;
    nt_hyper h;
    int64_t micro = 0, accum = 0, glob = 0;
    memset(parts, 0, sizeof(parts));
    memset(&h, 0, sizeof(h));
    parts[0].A = 10; parts[0].B = 16; parts[0].C = 2; parts[0].coord_fail = -1; parts[0].status = NT_STATUS_PARTIAL_ONLY;
    parts[1].A = 40; parts[1].B = 64; parts[1].C = 8; parts[1].coord_fail = -1; parts[1].status = NT_STATUS_PARTIAL_ONLY;
    h.eta = 0.5; h.b_k = 1; h.b_max = 0; h.round_to = 2; h.ddof = 1;
    if (normtest_combine(parts, 2, 2, &h, &out) != NT_OK) return 2;
    printf("combine %.17g %.17g %.17g %.17g %d %lld\n", out.A, out.B, out.C, out.T, (int)out.pass, (long long)out.next_b);
    if (normtest_resplit(8192, 4, 16, 8, &micro, &accum, &glob) != NT_OK) return 3;
    printf("resplit %lld %lld %lld\n", (long long)micro, (long long)accum, (long long)glob);
    printf("clip %.17g\n", normtest_clip_coef(4.0, 1.0));
    printf("workspace %zu tile %lld\n", normtest_workspace_bytes(8, 1000000), (long long)normtest_tile_coords(8));
    printf("workspace_for %zu %zu %zu\n", normtest_workspace_bytes_for(NT_BF16, 64, 1000000, NT_DO_STATS | NT_DO_ADAMW),
           normtest_workspace_bytes_for(NT_F32, 64, 1000000, NT_DO_STATS | NT_DO_ADAMW),
           normtest_workspace_bytes(64, 1000000));
    printf("static_max %lld\n", (long long)normtest_static_max_coords(8));
    printf("strerror %s\n", normtest_strerror(NT_ERR_WORKSPACE_TOO_SMALL));
    if (normtest_layer_stats(NULL, 0, NT_BF16, 8, 100, 100, NULL, 1, NULL, NULL, NULL) != NT_ERR_BAD_ARG) return 4;
  }
  return 0;
}
