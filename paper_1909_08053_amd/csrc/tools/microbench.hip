// On-box ceilings for the roofline discussion: bf16 MFMA issue rate, LDS read bandwidth, HBM copy bandwidth.
// Stand-alone program (no library code): hipcc --offload-arch=gfx950 -O3 microbench.hip -o mlm_microbench
#include <hip/hip_runtime.h>
#include <stdio.h>
typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float floatx16;
#define CK(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { printf("HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__); return 1; } } while (0)

// NACC independent accumulators per wave, back-to-back v_mfma_f32_32x32x16_bf16
template <int NACC>
__global__ __launch_bounds__(256) void k_mfma(float* out, int iters) {
  floatx16 acc[NACC];
  for (int i = 0; i < NACC; ++i)
    for (int e = 0; e < 16; ++e) acc[i][e] = 0.f;
  bf16x8 a, b;
  for (int e = 0; e < 8; ++e) { a[e] = (__bf16)(float)(threadIdx.x + e); b[e] = (__bf16)(float)e; }
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int i = 0; i < NACC; ++i) acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[i], 0, 0, 0);
  }
  float s = 0.f;
  for (int i = 0; i < NACC; ++i)
    for (int e = 0; e < 16; ++e) s += acc[i][e];
  out[blockIdx.x * blockDim.x + threadIdx.x] = s;
}

// 16-byte LDS reads, rows of `stride` bf16 elements, lanes 0..31 on consecutive rows (the GEMM's operand read pattern)
__global__ __launch_bounds__(256) void k_lds(float* out, int iters, int stride) {
  extern __shared__ __attribute__((aligned(16))) unsigned char raw[];
  __bf16* s = (__bf16*)raw;
  for (int i = threadIdx.x; i < 256 * 80; i += 256) s[i] = (__bf16)1.0f;
  __syncthreads();
  const int lane = threadIdx.x & 63, l32 = lane & 31, lh = lane >> 5, wave = threadIdx.x >> 6;
  float4 acc = make_float4(0, 0, 0, 0);
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const float4 v = *(const float4*)(s + ((wave * 32 + l32 + 32 * (j & 1)) % 256) * stride + (j >> 1) * 16 + lh * 8);
      acc.x += v.x; acc.y += v.y; acc.z += v.z; acc.w += v.w;
    }
  }
  out[blockIdx.x * blockDim.x + threadIdx.x] = acc.x + acc.y + acc.z + acc.w;
}

__global__ __launch_bounds__(256) void k_copy(const float4* __restrict__ in, float4* __restrict__ o, size_t n) {
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i < n) o[i] = in[i];
}

int main() {
  float* out;
  CK(hipMalloc(&out, 1 << 24));
  hipEvent_t e0, e1;
  CK(hipEventCreate(&e0));
  CK(hipEventCreate(&e1));
  float ms;
  const int iters = 4000;
  k_mfma<8><<<256, 256>>>(out, 100);
  CK(hipDeviceSynchronize());
  CK(hipEventRecord(e0));
  k_mfma<8><<<256, 256>>>(out, iters * 8);
  CK(hipEventRecord(e1));
  CK(hipDeviceSynchronize());
  CK(hipEventElapsedTime(&ms, e0, e1));
  printf("mfma_f32_32x32x16_bf16, 1 wave per SIMD (256 blocks x 4 waves): %.1f TFLOP/s\n",
         256.0 * 4 * iters * 8 * 8 * 32 * 32 * 16 * 2 / ms / 1e9);
  CK(hipEventRecord(e0));
  k_mfma<4><<<2048, 256>>>(out, iters);
  CK(hipEventRecord(e1));
  CK(hipDeviceSynchronize());
  CK(hipEventElapsedTime(&ms, e0, e1));
  printf("mfma_f32_32x32x16_bf16, 2048 blocks x 4 waves: %.1f TFLOP/s\n", 2048.0 * 4 * iters * 4 * 32 * 32 * 16 * 2 / ms / 1e9);
  CK(hipFuncSetAttribute((const void*)k_lds, hipFuncAttributeMaxDynamicSharedMemorySize, 65536));
  for (int stride : {72, 64}) {
    const int li = 20000;
    k_lds<<<256, 256, 256 * 80 * 2>>>(out, 10, stride);
    CK(hipDeviceSynchronize());
    CK(hipEventRecord(e0));
    k_lds<<<256, 256, 256 * 80 * 2>>>(out, li, stride);
    CK(hipEventRecord(e1));
    CK(hipDeviceSynchronize());
    CK(hipEventElapsedTime(&ms, e0, e1));
    const double bytes = 256.0 * 256 * li * 8 * 16;
    printf("LDS 16-byte reads, row stride %d elements: %.1f TB/s chip-wide = %.0f B/clk/CU at 2.4 GHz\n", stride,
           bytes / ms / 1e9, bytes / 256 / (ms * 1e-3 * 2.4e9));
  }
  const size_t n = (size_t)1 << 26;   // 1 GiB in, 1 GiB out
  float4 *src, *dst;
  CK(hipMalloc(&src, n * 16));
  CK(hipMalloc(&dst, n * 16));
  CK(hipMemset(src, 1, n * 16));
  k_copy<<<(unsigned)(n / 256), 256>>>(src, dst, n);
  CK(hipDeviceSynchronize());
  CK(hipEventRecord(e0));
  for (int r = 0; r < 5; ++r) k_copy<<<(unsigned)(n / 256), 256>>>(src, dst, n);
  CK(hipEventRecord(e1));
  CK(hipDeviceSynchronize());
  CK(hipEventElapsedTime(&ms, e0, e1));
  printf("HBM copy 1 GiB -> 1 GiB: %.2f TB/s (read + write)\n", 5.0 * 2 * n * 16 / ms / 1e9);
  return 0;
}
