// plain copy kernel of known size: calibration for FETCH_SIZE / WRITE_SIZE counters
#include <hip/hip_runtime.h>
#include <cstdio>
__global__ void copy_kernel(const uint4* __restrict__ s, uint4* __restrict__ d, size_t n) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) d[i] = s[i];
}
int main() {
  const size_t bytes = 1ull << 30;  // 1 GiB read + 1 GiB written
  uint4 *s, *d;
  if (hipMalloc(&s, bytes) != hipSuccess || hipMalloc(&d, bytes) != hipSuccess) return 1;
  (void)hipMemset(s, 1, bytes);
  (void)hipMemset(d, 0, bytes);
  const size_t n = bytes / 16;
  for (int r = 0; r < 3; ++r) copy_kernel<<<(unsigned)((n + 255) / 256), 256>>>(s, d, n);
  (void)hipDeviceSynchronize();
  printf("copied %zu bytes x3\n", bytes);
  return 0;
}
