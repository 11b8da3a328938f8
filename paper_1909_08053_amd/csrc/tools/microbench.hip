// On-box ceilings for the roofline discussion: bf16 MFMA issue rate on constant and on normally distributed operands,
// the same with the GEMM main loop's LDS fragment reads and with its HBM -> LDS copies added, LDS read bandwidth, HBM
// copy bandwidth.  Stand-alone program (no library code, not part of the library build):
//   hipcc --offload-arch=gfx950 -O3 -Xclang -target-feature -Xclang -packed-fp32-ops microbench.hip -o mlm_microbench
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdio.h>
typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float floatx16;
#define CK(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { printf("HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__); return 1; } } while (0)

// NACC independent accumulators per wave, back-to-back v_mfma_f32_32x32x16_bf16, loop-constant small-integer operands
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

// ---- the GEMM main loop's three streams, one at a time --------------------------------------------------------
// Workgroup = 8 waves (two per SIMD), each with the 128 x 64 wave tile of the library's 256 x 256 GEMM: per 16-deep
// half slice a wave issues 8 MFMAs on 4 + 2 operand fragments.  LEVEL 0: the fragments are a register-resident set of
// normally distributed bf16 values (activations ~ N(0, 1), weights ~ N(0, 0.02^2)) that rotates every half slice, so
// every MFMA sees operands that differ from its predecessor's -- the matrix pipe alone on real data, no memory
// traffic.  LEVEL 1: the fragments are read from a 128-KB LDS ring of such values with the library's k-contiguous
// addressing (six 16-byte reads per lane and half slice, one after each MFMA).  LEVEL 2: additionally every wave
// re-arms the ring with four 1-KB HBM -> LDS copies per slice (32 KB per slice and workgroup, from a 64-MB buffer),
// (the stage whose operands were just pulled into registers gets the slice four ahead, so three slices of copies are
// in flight) and meets the other waves at one barrier per slice, as the GEMM does.  WINDOW = slices of 32 KB a
// workgroup cycles through: 1024 (32 MB per workgroup, 64 MB in all: served by the memory-side cache) or 16 with all
// workgroups on the same 512 KB (served by the L2s).
typedef __attribute__((address_space(3))) void lds_void_t;
__device__ __forceinline__ void dma16(const void* g, uint32_t lds_addr) {
  asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, off" ::"s"(lds_addr), "v"(g) : "memory");
}
template <int N> __device__ __forceinline__ void wait_vmcnt() {
  __builtin_amdgcn_s_waitcnt((N & 15) | (7 << 4) | (15 << 8) | ((N >> 4) << 14));
}
__device__ __forceinline__ uint32_t hash32(uint32_t x) {
  x ^= x >> 16; x *= 0x7feb352du; x ^= x >> 15; x *= 0x846ca68bu; x ^= x >> 16;
  return x;
}
__device__ __forceinline__ float gauss(uint32_t i) {           // Box-Muller on two hashed uniforms
  const float u1 = (hash32(2 * i + 1) >> 8) * (1.0f / 16777216.0f) + 1e-7f;
  const float u2 = (hash32(2 * i + 2) >> 8) * (1.0f / 16777216.0f);
  return sqrtf(-2.0f * __logf(u1)) * __cosf(6.2831853f * u2);
}
__global__ void k_fill_gauss(__bf16* p, size_t n, float sigma) {
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = sigma == 0.0f ? (__bf16)1.0f : (__bf16)(sigma * gauss((uint32_t)i));   // sigma 0: the constant 1
}

// Wave-tile shapes: NW waves as 2 x NW/2, each TM x TN MFMA tiles of 32 x 32; block tile 64 TM x 16 NW TN.
//   8 waves, 4 x 2: the library's 256 x 256 tile with two waves per SIMD (6 fragment reads per 8 MFMAs, 32 KB per slice)
//   4 waves, 4 x 4: 256 x 256 with one wave per SIMD (8 reads per 16 MFMAs)
// (a 256 x 384 tile -- 4 waves of 4 x 6, 0.83 x the copy bytes per flop -- needs 384 accumulator registers per lane;
// the compiler spills several hundred of them, so that shape is not measured)
template <int LEVEL, int WINDOW, int NW, int TM, int TN, bool CONSTANT>
__global__ __launch_bounds__(NW * 64) void k_loop(float* out, const __bf16* __restrict__ src, int slices) {
  constexpr int WN = NW / 2, BM = 64 * TM, BN = 32 * WN * TN, NT = NW * 64;
  constexpr int STAGE = (BM + BN) * 64, RING = 4 * STAGE, NC = STAGE / 1024 / NW, NMF = TM * TN;
  static_assert(STAGE % (1024 * NW) == 0 && NMF > TM + TN, "shape");
  extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm0 = (wave / WN) * (32 * TM), wn0 = (wave % WN) * (32 * TN), l32 = lane & 31, lh = lane >> 5;
  // ring: A's two pair buffers ([BM rows][64 k]) then B's ([BN rows][64 k]), filled with N(0,1) / N(0, 0.02^2) values
  for (int i = tid; i < RING / 2; i += NT)
    ((__bf16*)lds)[i] = CONSTANT ? (__bf16)1.0f : (__bf16)((i < 2 * BM * 64 ? 1.0f : 0.02f) * gauss(blockIdx.x * 131072u + i));
  __syncthreads();
  floatx16 acc[TN][TM];
  for (int i = 0; i < TN; ++i)
    for (int j = 0; j < TM; ++j)
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;
  constexpr int R = LEVEL == 0 ? 4 : 1;      // LEVEL 0: rotating register sets
  bf16x8 ra[R][TM], rb[R][TN];
  if (LEVEL == 0) {
    for (int r = 0; r < R; ++r) {
      for (int j = 0; j < TM; ++j)
        for (int e = 0; e < 8; ++e) ra[r][j][e] = CONSTANT ? (__bf16)1.0f : (__bf16)gauss(((blockIdx.x * NT + tid) * 128 + (r * TM + j) * 8 + e) * 2654435761u);
      for (int i = 0; i < TN; ++i)
        for (int e = 0; e < 8; ++e) rb[r][i][e] = CONSTANT ? (__bf16)1.0f : (__bf16)(0.02f * gauss(((blockIdx.x * NT + tid) * 128 + 64 + (r * TN + i) * 8 + e) * 40503u));
    }
  }
  const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned char*)lds;
  // this lane's 16 bytes of each of the wave's NC 1-KB copies of a slice
  constexpr size_t slice_elems = STAGE / 2;
  const __bf16* gsrc = src + (WINDOW == 1024 ? (size_t)blockIdx.x * 977 % 512 : 0) * slice_elems + (size_t)(wave * NC) * 512 + lane * 8;
  auto frag = [&](const unsigned char* ring, int rows, int stage, int r0, int ks) {
    const int row = r0 + l32;
    const int u = (stage & 1) * 4 + ks * 2 + lh;
    const int sw = (((row >> 1) & 1) << 2) | ((row >> 2) & 3);
    return *reinterpret_cast<const bf16x8*>(ring + (stage >> 1) * (rows * 128) + row * 128 + ((u ^ sw) << 4));
  };
  const unsigned char* ringA = lds;
  const unsigned char* ringB = lds + 4 * BM * 64;
  bf16x8 fa[TM], fb[TN];
  if (LEVEL >= 1) {
    for (int j = 0; j < TM; ++j) fa[j] = frag(ringA, BM, 0, wm0 + j * 32, 0);
    for (int i = 0; i < TN; ++i) fb[i] = frag(ringB, BN, 0, wn0 + i * 32, 0);
  }
  for (int kt2 = 0; kt2 < slices; kt2 += 2)
#pragma unroll
  for (int par = 0; par < 2; ++par) {
    const int kt = kt2 + par;
    const int stage = kt & 3;
#pragma unroll
    for (int half = 0; half < 2; ++half) {
      bf16x8 na[TM], nb[TN];
#pragma unroll
      for (int idx = 0; idx < NMF; ++idx) {
        if (LEVEL == 0) {
          const int r = (2 * par + half) % R;          // compile-time: the slice loop is unrolled by two
          acc[idx / TM][idx % TM] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(rb[r][idx / TM], ra[r][idx % TM], acc[idx / TM][idx % TM], 0, 0, 0);
        } else {
          acc[idx / TM][idx % TM] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[idx / TM], fa[idx % TM], acc[idx / TM][idx % TM], 0, 0, 0);
          __builtin_amdgcn_sched_barrier(0);
          if (idx >= 1 && idx <= TM + TN) {            // one fragment read after each MFMA but the first
            const int q = idx - 1;
            const int nst = half == 0 ? stage : ((kt + 1) & 3), nks = half == 0 ? 1 : 0;
            if (q < TM) na[q] = frag(ringA, BM, nst, wm0 + q * 32, nks);
            else nb[q - TM] = frag(ringB, BN, nst, wn0 + (q - TM) * 32, nks);
          }
          if (LEVEL == 2 && half == 1) {
            // re-arm this slice's stage (its operands are all in registers by now), copies spread over the MFMAs
#pragma unroll
            for (int c = 0; c < NC; ++c) {
              if ((c * NMF) / NC != idx) continue;
              const size_t sl = (size_t)(kt & (WINDOW / 2 - 1));
              dma16(gsrc + sl * slice_elems + c * 512, lds0 + stage * STAGE + (wave * NC + c) * 1024);
            }
          }
          __builtin_amdgcn_sched_barrier(0);
        }
      }
      if (LEVEL >= 1) {
#pragma unroll
        for (int j = 0; j < TM; ++j) fa[j] = na[j];
#pragma unroll
        for (int i = 0; i < TN; ++i) fb[i] = nb[i];
        if (half == 0) {
          if (LEVEL == 2) wait_vmcnt<2 * NC>();        // the copies issued three slices ago (for the next slice) have landed
          __builtin_amdgcn_s_waitcnt(0xC07F);
          __builtin_amdgcn_s_barrier();
        }
      }
    }
  }
  if (LEVEL == 2) wait_vmcnt<0>();
  float s = 0.f;
  for (int i = 0; i < TN; ++i)
    for (int j = 0; j < TM; ++j)
      for (int e = 0; e < 16; ++e) s += acc[i][j][e];
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

typedef __attribute__((__vector_size__(4 * sizeof(float)))) float floatx4;
// The same ladder with v_mfma_f32_16x16x32_bf16 (the shape the library's 8-wave GEMM loop uses): one MFMA spans the
// slice's 32 k, a wave holds the NA + NB fragments of one slice and replaces each by the next slice's right after its
// last MFMA (B fragment outer, A fragment inner); hand-over after MFMA HO of the slice, re-arm copies after it.
// NW = 8: 2 x 4 waves of 128 x 64 (NA = 8, NB = 4); NW = 4: 2 x 2 waves of 128 x 128 (NA = 8, NB = 8)
template <int LEVEL, int WINDOW, bool CONSTANT, int NW, int HO>
__global__ __launch_bounds__(NW * 64) void k_loop16(float* out, const __bf16* __restrict__ src, int slices) {
  constexpr int BM = 256, BN = 256, NT = NW * 64, NA = 8, NB = NW == 8 ? 4 : 8, WN = NW / 2;
  constexpr int STAGE = (BM + BN) * 64, RING = 4 * STAGE, NC = STAGE / 1024 / NW;
  extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm0 = (wave / WN) * 128, wn0 = (wave % WN) * (16 * NB), l16 = lane & 15, lg = lane >> 4;
  for (int i = tid; i < RING / 2; i += NT)
    ((__bf16*)lds)[i] = CONSTANT ? (__bf16)1.0f : (__bf16)((i < 2 * BM * 64 ? 1.0f : 0.02f) * gauss(blockIdx.x * 131072u + i));
  __syncthreads();
  floatx4 acc[NB][NA];
  for (int i = 0; i < NB; ++i) for (int j = 0; j < NA; ++j) for (int e = 0; e < 4; ++e) acc[i][j][e] = 0.f;
  constexpr int R = LEVEL == 0 ? 2 : 1;
  bf16x8 ra[R][NA], rb[R][NB];
  if (LEVEL == 0) {
    for (int r = 0; r < R; ++r) {
      for (int j = 0; j < NA; ++j)
        for (int e = 0; e < 8; ++e) ra[r][j][e] = CONSTANT ? (__bf16)1.0f : (__bf16)gauss(((blockIdx.x * NT + tid) * 128 + (r * NA + j) * 8 + e) * 2654435761u);
      for (int i = 0; i < NB; ++i)
        for (int e = 0; e < 8; ++e) rb[r][i][e] = CONSTANT ? (__bf16)1.0f : (__bf16)(0.02f * gauss(((blockIdx.x * NT + tid) * 128 + 64 + (r * NB + i) * 8 + e) * 40503u));
    }
  }
  const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned char*)lds;
  constexpr size_t slice_elems = STAGE / 2;
  const __bf16* gsrc = src + (WINDOW == 1024 ? (size_t)blockIdx.x * 977 % 512 : 0) * slice_elems + (size_t)(wave * NC) * 512 + lane * 8;
  auto frag = [&](const unsigned char* ring, int rows, int stage, int r0) {
    const int row = r0 + l16;
    const int u = (stage & 1) * 4 + lg;
    const int sw = (((row >> 1) & 1) << 2) | ((row >> 2) & 3);
    return *reinterpret_cast<const bf16x8*>(ring + (stage >> 1) * (rows * 128) + row * 128 + ((u ^ sw) << 4));
  };
  const unsigned char* ringA = lds;
  const unsigned char* ringB = lds + 4 * BM * 64;
  bf16x8 fa[NA], fb[NB];
  if (LEVEL >= 1) {
    for (int j = 0; j < NA; ++j) fa[j] = frag(ringA, BM, 0, wm0 + j * 16);
    for (int i = 0; i < NB; ++i) fb[i] = frag(ringB, BN, 0, wn0 + i * 16);
  }
  constexpr int NMF = NA * NB;
  for (int kt2 = 0; kt2 < slices; kt2 += 2)
#pragma unroll
  for (int par = 0; par < 2; ++par) {
    const int kt = kt2 + par;
    const int stage = kt & 3, nst = (kt + 1) & 3;
#pragma unroll
    for (int i = 0; i < NB; ++i) {
#pragma unroll
      for (int j = 0; j < NA; ++j) {
        if (LEVEL == 0) {
          acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(rb[par % R][i], ra[par % R][j], acc[i][j], 0, 0, 0);
        } else {
          acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fb[i], fa[j], acc[i][j], 0, 0, 0);
          __builtin_amdgcn_sched_barrier(0);
          if (i == NB - 1) fa[j] = frag(ringA, BM, nst, wm0 + j * 16);          // last use of fa[j] in this slice
          if (j == NA - 1) fb[i] = frag(ringB, BN, nst, wn0 + i * 16);          // last use of fb[i]
          if (LEVEL == 2 && i >= 1) {
#pragma unroll
            for (int c = 0; c < NC; ++c) {
              if ((c * ((NB - 1) * NA)) / NC != (i - 1) * NA + j) continue;
              const size_t sl = (size_t)(kt & (WINDOW / 2 - 1));
              dma16(gsrc + sl * slice_elems + c * 512, lds0 + stage * STAGE + (wave * NC + c) * 1024);
            }
          }
          __builtin_amdgcn_sched_barrier(0);
          if (i == 0 && j == HO) {
            // hand-over, placed before the first read of the next slice (the reload of fb[0] after MFMA (0, NA - 1))
            if (LEVEL == 2) wait_vmcnt<2 * NC>();
            __builtin_amdgcn_s_waitcnt(0xC07F);
            __builtin_amdgcn_s_barrier();
          }
        }
      }
    }
  }
  if (LEVEL == 2) wait_vmcnt<0>();
  float s = 0.f;
  for (int i = 0; i < NB; ++i) for (int j = 0; j < NA; ++j) for (int e = 0; e < 4; ++e) s += acc[i][j][e];
  out[blockIdx.x * blockDim.x + threadIdx.x] = s;
}
template <int LEVEL, int WINDOW, bool CONSTANT>
static int run_loop16(const char* what, float* out, const __bf16* src) {
  constexpr int RING = 4 * 512 * 64;
  hipEvent_t e0, e1;
  CK(hipEventCreate(&e0));
  CK(hipEventCreate(&e1));
  auto kern = k_loop16<LEVEL, WINDOW, CONSTANT, 8, 6>;
  CK(hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, RING));
  const int slices = 20000;
  kern<<<256, 512, RING>>>(out, src, 2000);
  CK(hipDeviceSynchronize());
  float best = 1e30f, sum = 0.f;
  for (int rep = 0; rep < 5; ++rep) {
    float ms;
    CK(hipEventRecord(e0));
    kern<<<256, 512, RING>>>(out, src, slices);
    CK(hipEventRecord(e1));
    CK(hipDeviceSynchronize());
    CK(hipEventElapsedTime(&ms, e0, e1));
    best = ms < best ? ms : best;
    sum += ms;
  }
  const double flops = 256.0 * slices * 2.0 * 256 * 256 * 32;
  printf("%-58s %7.1f TFLOP/s mean of 5, %7.1f best\n", what, flops * 5 / sum / 1e9, flops / best / 1e9);
  return 0;
}
template <bool CONSTANT>
static int run_shape16(const char* title, float* out, const __bf16* src) {
  printf("%s:\n", title);
  if (run_loop16<0, 16, CONSTANT>("  MFMA only (operand sets rotating in registers)", out, src)) return 1;
  if (run_loop16<1, 16, CONSTANT>("  + fragments read from LDS, one barrier per slice", out, src)) return 1;
  if (run_loop16<2, 16, CONSTANT>("  + slices copied to LDS by global_load_lds, from the L2s", out, src)) return 1;
  if (run_loop16<2, 1024, CONSTANT>("  + same copies, from the memory-side cache (64 MB)", out, src)) return 1;
  return 0;
}
template <int LEVEL, int WINDOW, int NW, int TM, int TN, bool CONSTANT>
static int run_loop(const char* what, float* out, const __bf16* src) {
  constexpr int RING = 4 * (64 * TM + 16 * NW * TN) * 64;
  hipEvent_t e0, e1;
  CK(hipEventCreate(&e0));
  CK(hipEventCreate(&e1));
  auto kern = k_loop<LEVEL, WINDOW, NW, TM, TN, CONSTANT>;
  CK(hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, RING));
  const int slices = 20000;                   // 2 x 10^4 slices of 32: 10-20 ms per launch
  kern<<<256, NW * 64, RING>>>(out, src, 2000);
  CK(hipDeviceSynchronize());
  float best = 1e30f, sum = 0.f;
  for (int rep = 0; rep < 5; ++rep) {
    float ms;
    CK(hipEventRecord(e0));
    kern<<<256, NW * 64, RING>>>(out, src, slices);
    CK(hipEventRecord(e1));
    CK(hipDeviceSynchronize());
    CK(hipEventElapsedTime(&ms, e0, e1));
    best = ms < best ? ms : best;
    sum += ms;
  }
  const double flops = 256.0 * NW * slices * 2.0 * TM * TN * 32 * 32 * 16 * 2;
  printf("%-58s %7.1f TFLOP/s mean of 5, %7.1f best\n", what, flops * 5 / sum / 1e9, flops / best / 1e9);
  return 0;
}

template <int NW, int TM, int TN, bool CONSTANT>
static int run_shape(const char* name, float* out, const __bf16* src) {
  printf("%s, %s:\n", name, CONSTANT ? "every operand element = 1 (no switching activity in the data paths)" : "operands N(0,1) x N(0,0.02)");
  if (run_loop<0, 1024, NW, TM, TN, CONSTANT>("  MFMA only (operand sets rotating in registers)", out, src)) return 1;
  if (run_loop<1, 1024, NW, TM, TN, CONSTANT>("  + fragments read from LDS, one barrier per slice", out, src)) return 1;
  if (run_loop<2, 16, NW, TM, TN, CONSTANT>("  + slices copied to LDS by global_load_lds, from the L2s", out, src)) return 1;
  if (run_loop<2, 1024, NW, TM, TN, CONSTANT>("  + same copies, from the memory-side cache (64 MB)", out, src)) return 1;
  return 0;
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
  printf("mfma_f32_32x32x16_bf16, constant operands, 1 wave per SIMD (256 blocks x 4 waves): %.1f TFLOP/s\n",
         256.0 * 4 * iters * 8 * 8 * 32 * 32 * 16 * 2 / ms / 1e9);
  CK(hipEventRecord(e0));
  k_mfma<4><<<2048, 256>>>(out, iters);
  CK(hipEventRecord(e1));
  CK(hipDeviceSynchronize());
  CK(hipEventElapsedTime(&ms, e0, e1));
  printf("mfma_f32_32x32x16_bf16, constant operands, 2048 blocks x 4 waves: %.1f TFLOP/s\n", 2048.0 * 4 * iters * 4 * 32 * 32 * 16 * 2 / ms / 1e9);

  // normally distributed operands: matrix pipe alone, + LDS fragment reads, + HBM -> LDS copies
  const size_t src_elems = (size_t)32 << 20;      // 64 MB of N(0, 1) bf16
  __bf16* src;
  CK(hipMalloc(&src, src_elems * 2));
  k_fill_gauss<<<(unsigned)(src_elems / 256), 256>>>(src, src_elems, 1.0f);
  CK(hipDeviceSynchronize());
  if (run_shape<8, 4, 2, false>("8 waves of 128 x 64 (256 x 256 tile, 6 fragment reads per 8 MFMAs, 32 KB per slice)", out, src)) return 1;
  if (run_shape<4, 4, 4, false>("4 waves of 128 x 128 (256 x 256 tile, 8 reads per 16 MFMAs, 32 KB per slice)", out, src)) return 1;
  if (run_shape16<false>("8 waves of 128 x 64 with mfma_f32_16x16x32_bf16 (12 fragment reads per 32 MFMAs, 32 KB per slice), operands N(0,1) x N(0,0.02)", out, src)) return 1;
  // the same instruction streams on constant data: what the schedule allows when no bit toggles (the gap to the
  // figures above is clock lost to switching power, not to issue slots, LDS or copy bandwidth)
  k_fill_gauss<<<(unsigned)(src_elems / 256), 256>>>(src, src_elems, 0.0f);
  CK(hipDeviceSynchronize());
  if (run_shape<8, 4, 2, true>("8 waves of 128 x 64", out, src)) return 1;
  if (run_shape16<true>("8 waves of 128 x 64 with mfma_f32_16x16x32_bf16, every operand element = 1", out, src)) return 1;

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
  float4 *csrc, *dst;
  CK(hipMalloc(&csrc, n * 16));
  CK(hipMalloc(&dst, n * 16));
  CK(hipMemset(csrc, 1, n * 16));
  k_copy<<<(unsigned)(n / 256), 256>>>(csrc, dst, n);
  CK(hipDeviceSynchronize());
  CK(hipEventRecord(e0));
  for (int r = 0; r < 5; ++r) k_copy<<<(unsigned)(n / 256), 256>>>(csrc, dst, n);
  CK(hipEventRecord(e1));
  CK(hipDeviceSynchronize());
  CK(hipEventElapsedTime(&ms, e0, e1));
  printf("HBM copy 1 GiB -> 1 GiB: %.2f TB/s (read + write)\n", 5.0 * 2 * n * 16 / ms / 1e9);
  return 0;
}
