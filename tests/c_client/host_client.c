/* A plain C99 client of the library: proves that the header is valid C (no C++ needed), that the
 * struct layouts the compiler derives match the ones the tests assume, and that the host-only
 * entry points can be called without a GPU.  Prints key=value lines for the test to read. */
#include <stddef.h>
#include <stdio.h>
#include <string.h>
#include "supergen_tile.h"

int main(void) {
  sg_problem p;
  size_t ws = 0;
  int32_t dy = -1, dx = -1;
  int st;
  memset(&p, 0, sizeof p);
  p.T = 3; p.H = 16; p.W = 16;
  p.tile_h = 10; p.tile_w = 10; p.stride_h = 6; p.stride_w = 6;
  p.n_tile_rows = 2; p.n_tile_cols = 2;
  p.heads = 2; p.head_dim = 64;
  p.dtype = SG_F32;
  p.scale = 0.125f;
  p.grid_stride_token = 64;
  p.grid_stride_head = (int64_t)3 * 16 * 16 * 64;
  printf("version=%s\n", sg_version());
  printf("sizeof_problem=%zu\n", sizeof(sg_problem));
  printf("offset_stride_token=%zu\n", offsetof(sg_problem, grid_stride_token));
  printf("offset_shift_h=%zu\n", offsetof(sg_problem, shift_h));
  printf("sizeof_step_io=%zu\n", sizeof(sg_step_io));
  printf("sizeof_gain_state=%zu\n", sizeof(sg_gain_state));
  printf("sizeof_gain_step_io=%zu\n", sizeof(sg_gain_step_io));
  printf("sizeof_region_control=%zu\n", sizeof(sg_region_control));
  printf("sizeof_scheduler_update=%zu\n", sizeof(sg_scheduler_update));
  printf("validate=%d\n", sg_problem_validate(&p));
  p.stride_w = 11;
  printf("validate_gap=%d\n", sg_problem_validate(&p));
  p.stride_w = 6;
  st = sg_workspace_bytes(20, &ws);
  printf("workspace_status=%d\nworkspace_bytes=%zu\n", st, ws);
  printf("null_attention=%d\n", sg_tile_attention(&p, NULL, NULL, NULL, 0, 0, NULL, NULL));
  printf("null_blend=%d\n", sg_tile_blend(&p, NULL, NULL, NULL));
  printf("null_step=%d\n", sg_denoise_step_tiled(&p, NULL, NULL));
  st = sg_shift_schedule(&p, 5, 4, 2, &dy, &dx);   /* step 5, loop step 4, every 2nd step: 2 moves of 10 / 4 */
  printf("shift_status=%d\nshift_h=%d\nshift_w=%d\n", st, (int)dy, (int)dx);
  printf("status_string=%s\n", sg_status_string(SG_ERR_INVALID_ARG));
  return 0;
}
