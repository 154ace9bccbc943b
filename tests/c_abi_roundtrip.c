/* A plain C program that drives libsprnn through its C ABI with nothing but the HIP runtime for device memory:
 * a cyclic-shift permutation matrix with weights 1.0, zero input and a non-negative h_0 must rotate h_0 bit for bit
 * (h_t[i] = h_0[(i + t) mod H]).  Built and run by tests/test_c_abi_gpu.py.  Exit code 0 = pass. */
#include <hip/hip_runtime_api.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "sprnn.h"

#define CHECK_HIP(call) do { hipError_t e_ = (call); if (e_ != hipSuccess) { fprintf(stderr, "%s: %s\n", #call, hipGetErrorString(e_)); return 2; } } while (0)
#define CHECK_RC(call) do { int rc_ = (call); if (rc_ != SPRNN_OK) { fprintf(stderr, "%s: %s\n", #call, sprnn_status_string(rc_)); return 3; } } while (0)

int main(void) {
  enum { H = 300, B = 4, T = 7 };
  int32_t row_ptr[H + 1], col[H];
  uint16_t val[H];
  for (int i = 0; i < H; ++i) { row_ptr[i] = i; col[i] = (i + 1) % H; val[i] = 0x3C00; /* 1.0 in binary16 */ }
  row_ptr[H] = H;

  static float h0[B][H], x[T][B][H], out[T][B][H];
  for (int b = 0; b < B; ++b)
    for (int i = 0; i < H; ++i) h0[b][i] = (float)((i * 7 + b * 13) % 101) * 0.25f;
  memset(x, 0, sizeof(x));

  float *d_x = NULL, *d_h0 = NULL, *d_out = NULL;
  CHECK_HIP(hipMalloc((void**)&d_x, sizeof(x)));
  CHECK_HIP(hipMalloc((void**)&d_h0, sizeof(h0)));
  CHECK_HIP(hipMalloc((void**)&d_out, sizeof(out)));
  CHECK_HIP(hipMemcpy(d_x, x, sizeof(x), hipMemcpyHostToDevice));
  CHECK_HIP(hipMemcpy(d_h0, h0, sizeof(h0), hipMemcpyHostToDevice));

  /* Default options: ordinary launches, so this program can run beside the test runner that starts it (which may
   * itself have used the library on this device; nothing of it runs meanwhile). */
  sprnn_options_t opt;
  memset(&opt, 0, sizeof(opt));
  sprnn_handle_t handle = NULL;
  CHECK_RC(sprnn_create_ex(&handle, H, B, SPRNN_ACT_RELU, row_ptr, col, val, 0, &opt));
  sprnn_info_t info;
  CHECK_RC(sprnn_get_info(handle, &info));
  CHECK_RC(sprnn_forward(handle, T, d_x, d_h0, d_out, NULL));
  CHECK_RC(sprnn_check(handle));
  CHECK_HIP(hipMemcpy(out, d_out, sizeof(out), hipMemcpyDeviceToHost));

  long bad = 0;
  for (int t = 0; t < T; ++t)
    for (int b = 0; b < B; ++b)
      for (int i = 0; i < H; ++i)
        if (memcmp(&out[t][b][i], &h0[b][(i + t + 1) % H], sizeof(float)) != 0) ++bad;
  /* The library orders its persistent launches on a device whatever streams they go to.  Streams that come and go:
   * a launch on a stream of its own, the stream destroyed, then a launch on another new stream and one on the
   * default stream; every result must again be the rotation. */
  for (int round = 0; round < 3; ++round) {
    hipStream_t s = NULL;
    if (round < 2) CHECK_HIP(hipStreamCreateWithFlags(&s, hipStreamNonBlocking));
    CHECK_HIP(hipMemset(d_out, 0xFF, sizeof(out)));
    CHECK_HIP(hipDeviceSynchronize());
    CHECK_RC(sprnn_forward(handle, T, d_x, d_h0, d_out, s));
    CHECK_HIP(hipStreamSynchronize(s));
    CHECK_RC(sprnn_check(handle));
    CHECK_HIP(hipMemcpy(out, d_out, sizeof(out), hipMemcpyDeviceToHost));
    for (int t = 0; t < T; ++t)
      for (int b = 0; b < B; ++b)
        for (int i = 0; i < H; ++i)
          if (memcmp(&out[t][b][i], &h0[b][(i + t + 1) % H], sizeof(float)) != 0) ++bad;
    if (s) CHECK_HIP(hipStreamDestroy(s));
  }
  /* wrong call for the cell, and a NULL output: clean refusals */
  if (sprnn_forward_lstm(handle, T, d_x, NULL, NULL, d_out, d_out, NULL) != SPRNN_ERR_UNSUPPORTED) ++bad;
  if (sprnn_forward(handle, T, d_x, d_h0, NULL, NULL) != SPRNN_ERR_INVALID) ++bad;
  CHECK_RC(sprnn_destroy(handle));
  CHECK_HIP(hipFree(d_x)); CHECK_HIP(hipFree(d_h0)); CHECK_HIP(hipFree(d_out));
  printf("grid %d block %d nnz %lld: %ld mismatches\n", info.grid, info.block, (long long)info.nnz, bad);
  return bad ? 1 : 0;
}
