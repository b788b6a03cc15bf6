/* A plain C99 caller of the device-side entry points: no C++ and no Python in the process.  It reads a problem
 * and its canvas tensors from a file, runs tile attention on every tile, the blend, and the same step through
 * sg_denoise_step_tiled, and writes the results to a second file; the test that starts it compares them with the
 * oracle and with what the Python binding gets from the same inputs.
 *
 *   gpu_client IN OUT
 *   IN : int32 T H W tile_h tile_w stride_h stride_w n_tile_rows n_tile_cols heads head_dim dtype shift_h shift_w,
 *        float scale, then q, k, v as [heads][T][H][W][head_dim] in the problem's element type
 *   OUT: every tile's packed attention output (row-major over tiles), the blended canvas, and the canvas the step
 *        call produced
 */
#include <stdio.h>
#include <stdlib.h>
#include <string.h>
#include <hip/hip_runtime_api.h>
#include "supergen_tile.h"

#define HIP_OK(call)                                                                      \
  do {                                                                                    \
    hipError_t e_ = (call);                                                               \
    if (e_ != hipSuccess) {                                                               \
      fprintf(stderr, "%s failed: %s\n", #call, hipGetErrorString(e_));                   \
      return 2;                                                                           \
    }                                                                                     \
  } while (0)
#define SG_OK_OR_DIE(call)                                                                                \
  do {                                                                                                    \
    int s_ = (call);                                                                                      \
    if (s_ != SG_OK) {                                                                                    \
      fprintf(stderr, "%s returned %d (%s), hip error %d\n", #call, s_, sg_status_string(s_), sg_last_hip_error()); \
      return 3;                                                                                           \
    }                                                                                                     \
  } while (0)

int main(int argc, char** argv) {
  if (argc != 3) {
    fprintf(stderr, "usage: %s IN OUT\n", argv[0]);
    return 1;
  }
  FILE* in = fopen(argv[1], "rb");
  if (!in) {
    perror(argv[1]);
    return 1;
  }
  int32_t hdr[14];
  float scale;
  if (fread(hdr, sizeof(int32_t), 14, in) != 14 || fread(&scale, sizeof(float), 1, in) != 1) {
    fprintf(stderr, "short header\n");
    return 1;
  }
  sg_problem p;
  memset(&p, 0, sizeof p);
  p.T = hdr[0]; p.H = hdr[1]; p.W = hdr[2];
  p.tile_h = hdr[3]; p.tile_w = hdr[4];
  p.stride_h = hdr[5]; p.stride_w = hdr[6];
  p.n_tile_rows = hdr[7]; p.n_tile_cols = hdr[8];
  p.heads = hdr[9]; p.head_dim = hdr[10];
  p.dtype = hdr[11];
  p.shift_h = hdr[12]; p.shift_w = hdr[13];
  p.scale = scale;
  p.grid_stride_token = p.head_dim;
  p.grid_stride_head = (int64_t)p.T * p.H * p.W * p.head_dim;
  SG_OK_OR_DIE(sg_problem_validate(&p));

  const size_t esz = p.dtype == SG_F32 ? 4 : 2;
  const size_t canvas_bytes = (size_t)p.heads * p.T * p.H * p.W * p.head_dim * esz;
  const size_t tile_bytes = (size_t)p.heads * p.T * p.tile_h * p.tile_w * p.head_dim * esz;
  const int n_tiles = p.n_tile_rows * p.n_tile_cols;
  if (n_tiles > SG_MAX_TILES) return 1;

  void* host = malloc(canvas_bytes > tile_bytes ? canvas_bytes : tile_bytes);
  void *q, *k, *v, *canvas, *canvas_step;
  void* dev[3];
  for (int i = 0; i < 3; ++i) {
    if (fread(host, 1, canvas_bytes, in) != canvas_bytes) {
      fprintf(stderr, "short tensor %d\n", i);
      return 1;
    }
    HIP_OK(hipMalloc(&dev[i], canvas_bytes));
    HIP_OK(hipMemcpy(dev[i], host, canvas_bytes, hipMemcpyHostToDevice));
  }
  fclose(in);
  q = dev[0]; k = dev[1]; v = dev[2];
  HIP_OK(hipMalloc(&canvas, canvas_bytes));
  HIP_OK(hipMalloc(&canvas_step, canvas_bytes));

  void* tile_out[SG_MAX_TILES];
  void* tile_out_step[SG_MAX_TILES];
  for (int i = 0; i < n_tiles; ++i) {
    HIP_OK(hipMalloc(&tile_out[i], tile_bytes));
    HIP_OK(hipMalloc(&tile_out_step[i], tile_bytes));
  }

  hipStream_t stream;
  HIP_OK(hipStreamCreate(&stream));
  for (int r = 0; r < p.n_tile_rows; ++r)
    for (int c = 0; c < p.n_tile_cols; ++c)
      SG_OK_OR_DIE(sg_tile_attention(&p, q, k, v, r, c, tile_out[r * p.n_tile_cols + c], stream));
  SG_OK_OR_DIE(sg_tile_blend(&p, (const void* const*)tile_out, canvas, stream));

  sg_step_io io;
  memset(&io, 0, sizeof io);
  io.q = q; io.k = k; io.v = v;
  io.cache_out = tile_out_step;
  io.threshold = -1.0f;
  io.grid_out = canvas_step;
  SG_OK_OR_DIE(sg_denoise_step_tiled(&p, &io, stream));
  HIP_OK(hipStreamSynchronize(stream));

  FILE* out = fopen(argv[2], "wb");
  if (!out) {
    perror(argv[2]);
    return 1;
  }
  for (int i = 0; i < n_tiles; ++i) {
    HIP_OK(hipMemcpy(host, tile_out[i], tile_bytes, hipMemcpyDeviceToHost));
    fwrite(host, 1, tile_bytes, out);
  }
  HIP_OK(hipMemcpy(host, canvas, canvas_bytes, hipMemcpyDeviceToHost));
  fwrite(host, 1, canvas_bytes, out);
  HIP_OK(hipMemcpy(host, canvas_step, canvas_bytes, hipMemcpyDeviceToHost));
  fwrite(host, 1, canvas_bytes, out);
  if (fclose(out) != 0) return 1;

  for (int i = 0; i < n_tiles; ++i) {
    HIP_OK(hipFree(tile_out[i]));
    HIP_OK(hipFree(tile_out_step[i]));
  }
  HIP_OK(hipFree(q)); HIP_OK(hipFree(k)); HIP_OK(hipFree(v));
  HIP_OK(hipFree(canvas)); HIP_OK(hipFree(canvas_step));
  HIP_OK(hipStreamDestroy(stream));
  free(host);
  printf("gpu_client: %d tiles, library %s\n", n_tiles, sg_version());
  return 0;
}
