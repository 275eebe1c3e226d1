/* A plain C consumer of the C ABI in include/vla.h: no Python, no PyTorch.  Reads q, k, v from a raw file,
 * runs vla_forward on GPU 0 through the HIP runtime's C interface and writes o, S_T, A_T to a raw file.
 * Test infrastructure (tests/test_c_abi_gpu.py drives it and compares the result with the oracle).
 *
 * usage: c_abi_client IN OUT B H T d io_dtype mode
 *   IN : q, k, v, each B*H*T*d elements of the I/O type (float32 or raw bfloat16 bit patterns)
 *   OUT: o (B*H*T*d elements of the I/O type), then S_T and A_T (B*H*d*d float32 each)
 */
#include <hip/hip_runtime_api.h>
#include <stdio.h>
#include <stdlib.h>

#include "../include/vla.h"

#define CHECK_HIP(call)                                                              \
  do {                                                                               \
    hipError_t e_ = (call);                                                          \
    if (e_ != hipSuccess) {                                                          \
      fprintf(stderr, "%s failed: %s\n", #call, hipGetErrorString(e_));              \
      return 2;                                                                      \
    }                                                                                \
  } while (0)

int main(int argc, char** argv) {
  if (argc != 9) {
    fprintf(stderr, "usage: %s IN OUT B H T d io_dtype mode\n", argv[0]);
    return 1;
  }
  const int B = atoi(argv[3]), H = atoi(argv[4]), T = atoi(argv[5]), d = atoi(argv[6]);
  const int io = atoi(argv[7]), mode = atoi(argv[8]);
  const size_t esz = io == VLA_BF16 ? 2 : 4;
  const size_t n_io = (size_t)B * H * T * d, n_state = (size_t)B * H * d * d;

  void* host_in = malloc(3 * n_io * esz);
  void* host_out = malloc(n_io * esz + 2 * n_state * sizeof(float));
  if (!host_in || !host_out) return 1;
  FILE* f = fopen(argv[1], "rb");
  if (!f || fread(host_in, esz, 3 * n_io, f) != 3 * n_io) {
    fprintf(stderr, "cannot read %s\n", argv[1]);
    return 1;
  }
  fclose(f);

  vla_opts opts;
  vla_default_opts(&opts);
  opts.mode = mode;
  const size_t ws_bytes = vla_forward_workspace_bytes(B, H, T, d, d, io, &opts);

  char *dq, *dk, *dv, *dout, *ws = NULL;
  float *dS, *dA;
  hipStream_t stream;
  CHECK_HIP(hipSetDevice(0));
  CHECK_HIP(hipStreamCreate(&stream));
  CHECK_HIP(hipMalloc((void**)&dq, n_io * esz));
  CHECK_HIP(hipMalloc((void**)&dk, n_io * esz));
  CHECK_HIP(hipMalloc((void**)&dv, n_io * esz));
  CHECK_HIP(hipMalloc((void**)&dout, n_io * esz));
  CHECK_HIP(hipMalloc((void**)&dS, n_state * sizeof(float)));
  CHECK_HIP(hipMalloc((void**)&dA, n_state * sizeof(float)));
  if (ws_bytes) CHECK_HIP(hipMalloc((void**)&ws, ws_bytes));
  CHECK_HIP(hipMemcpy(dq, host_in, n_io * esz, hipMemcpyHostToDevice));
  CHECK_HIP(hipMemcpy(dk, (char*)host_in + n_io * esz, n_io * esz, hipMemcpyHostToDevice));
  CHECK_HIP(hipMemcpy(dv, (char*)host_in + 2 * n_io * esz, n_io * esz, hipMemcpyHostToDevice));

  const int rc = vla_forward(dq, dk, dv, NULL, NULL, dout, dS, dA, B, H, T, d, d, io, &opts, ws, ws_bytes,
                             (void*)stream);
  if (rc != VLA_OK) {
    fprintf(stderr, "vla_forward: %s\n", vla_status_string(rc));
    return 3;
  }
  CHECK_HIP(hipStreamSynchronize(stream));
  CHECK_HIP(hipMemcpy(host_out, dout, n_io * esz, hipMemcpyDeviceToHost));
  CHECK_HIP(hipMemcpy((char*)host_out + n_io * esz, dS, n_state * sizeof(float), hipMemcpyDeviceToHost));
  CHECK_HIP(hipMemcpy((char*)host_out + n_io * esz + n_state * sizeof(float), dA, n_state * sizeof(float),
                      hipMemcpyDeviceToHost));
  f = fopen(argv[2], "wb");
  if (!f || fwrite(host_out, 1, n_io * esz + 2 * n_state * sizeof(float), f) !=
                n_io * esz + 2 * n_state * sizeof(float)) {
    fprintf(stderr, "cannot write %s\n", argv[2]);
    return 1;
  }
  fclose(f);
  printf("libvla %d: mode %d resolved to %d, workspace %zu bytes\n", vla_version(), mode,
         vla_resolve_mode(B, H, T, d, d, io, &opts), ws_bytes);
  return 0;
}
