// Stand-alone measurement of what bounds the scoring sweeps on gfx950: how the matrix pipe and the
// vector pipe share a SIMD, and what clock the part sustains meanwhile.  Not part of the library; it
// backs the figures quoted for the sweep kernels with numbers anyone can re-measure.
//
//   part A  one "tile" of the second scoring pass as the sweep kernel issues it -- 8 operand reads
//           from LDS, 8 dependent v_mfma_f32_32x32x16_bf16 (32 rows x 32 keys x 128), then for the
//           16 results of a lane (fma, v_exp_f32, fma) with the per-row constants read from LDS --
//           run as MFMA part only, vector part only, and both, 16 waves per work-group on all CUs,
//           with random bf16 operand bits; two orderings of the same work (in-wave software pipeline
//           over 16x16x32 sub-tiles; half the waves one phase late).
//   part B  issue cost of single vector instructions, alone and next to a chain of MFMAs.
//   part C  the tile of part A rebuilt step by step toward the sweep kernel's loop: a barrier per unit of
//           four tiles; the rows staged global -> registers -> LDS into a double buffer; the key
//           operands reloaded from global memory every fifth unit; the per-row table staged per unit.
// The shader clock is read with s_memtime against the 100 MHz s_memrealtime counter.
#include <hip/hip_runtime.h>

#include <cstdio>
#include <cstdlib>

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
#define CHECK(x)                                                                  \
  do {                                                                            \
    hipError_t e_ = (x);                                                          \
    if (e_ != hipSuccess) {                                                       \
      printf("HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__);       \
      exit(1);                                                                    \
    }                                                                             \
  } while (0)

constexpr int kQRow = 272;      // bytes of a staged query row in LDS (256 + 16 pad), as in the sweep kernel
__device__ inline unsigned rnd_bf16x2(unsigned i) {      // two bf16 values in [1, 2) with random sign and mantissa
  unsigned h = i * 2654435761u;
  h ^= h >> 15; h *= 2246822519u; h ^= h >> 13;
  return 0x3F803F80u | (h & 0x807F807Fu);
}
__device__ __forceinline__ bf16x8 bf(u32x4 v) { return __builtin_bit_cast(bf16x8, v); }
__device__ __forceinline__ float ex2(float x) { return __builtin_amdgcn_exp2f(x); }

// MODE 0: MFMA part and vector part, tile after tile (the sweep kernel's order)
//      1: MFMA part only     2: vector part only
//      3: 16x16x32 sub-tiles, the 4 MFMAs of sub-tile s+1 interleaved with the vector work on sub-tile s
//      4: as 0, but the waves with (wave >> 2) & 1 run one phase late (vector work of tile t-1, then MFMAs of tile t)
template <int MODE>
__global__ __launch_bounds__(1024) void k_tile(float* out, int units, float c, long long* clk) {
  __shared__ __align__(16) unsigned char q[128 * kQRow];
  __shared__ __align__(16) float2 cst[128];
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, l32 = lane & 31, half = lane >> 5, l16 = lane & 15,
            quad = lane >> 4;
  for (int i = tid; i < 128 * kQRow / 4; i += 1024) ((unsigned*)q)[i] = rnd_bf16x2(i);
  for (int i = tid; i < 128; i += 1024) cst[i] = make_float2(-3.0f - 0.01f * i, 1.0f / (1.0f + i));
  __syncthreads();
  u32x4 kf[8];
  for (int kk = 0; kk < 8; ++kk)
    for (int j = 0; j < 4; ++j) kf[kk][j] = rnd_bf16x2(tid * 64 + kk * 4 + j + 12345);
  double col64 = 0.0;
  float cs0 = 0.f, cs1 = 0.f;
  long long c0 = 0, w0 = 0;
  if (tid == 0) { c0 = clock64(); w0 = wall_clock64(); }
  f32x16 acc;
#pragma unroll
  for (int e = 0; e < 16; ++e) acc[e] = 0.01f * e;
  auto mfma_part = [&](int rt) {
    u32x4 qv[8];
#pragma unroll
    for (int kk = 0; kk < 8; ++kk) qv[kk] = *(const u32x4*)(&q[(rt * 32 + l32) * kQRow + half * 16 + kk * 32]);
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[e] = 0.f;
#pragma unroll
    for (int kk = 0; kk < 8; ++kk) acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bf(qv[kk]), bf(kf[kk]), acc, 0, 0, 0);
  };
  auto vector_part = [&](int rt) {
    float a0 = 0.f, a1 = 0.f;
#pragma unroll
    for (int e = 0; e < 16; e += 2) {
      const int row0 = rt * 32 + 8 * (e >> 2) + 4 * half + (e & 3);
      const f32x4 cv = *(const f32x4*)(&cst[row0]);
      a0 = fmaf(ex2(fmaf(acc[e], c, cv[0])), cv[1], a0);
      a1 = fmaf(ex2(fmaf(acc[e + 1], c, cv[2])), cv[3], a1);
    }
    col64 += (double)(a0 + a1);
  };
  auto pin = [&]() {
    asm volatile("" : "+v"(col64), "+v"(cs0) : : "memory");
    __builtin_amdgcn_sched_barrier(0);
  };
  if (MODE == 0 || MODE == 1 || MODE == 2) {
    for (int u = 0; u < units; ++u) {
#pragma unroll
      for (int rt = 0; rt < 4; ++rt) {
        if (MODE != 2) mfma_part(rt);
        if (MODE == 1) cs0 += acc[3];
        if (MODE != 1) vector_part(rt);
        if (MODE == 2) acc[rt] += 1e-9f;
        pin();
      }
    }
  }
  if (MODE == 3) {
    f32x4 accA = {0, 0, 0, 0}, accB = {0, 0, 0, 0};
    auto rdq = [&](int rg, int kk) { return *(const u32x4*)(&q[(rg * 16 + l16) * kQRow + quad * 16 + kk * 64]); };
    auto elem = [&](const f32x4& a, const f32x4& cv0, const f32x4& cv1, int e) {
      const float nr = e == 0 ? cv0[0] : e == 1 ? cv0[2] : e == 2 ? cv1[0] : cv1[2];
      const float w = e == 0 ? cv0[1] : e == 1 ? cv0[3] : e == 2 ? cv1[1] : cv1[3];
      const float x = fmaf(a[e], c, nr);
      if (e & 1) cs1 = fmaf(ex2(x), w, cs1); else cs0 = fmaf(ex2(x), w, cs0);
    };
    u32x4 qa[4], qb[4];
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) qa[kk] = rdq(0, kk);
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) accA = __builtin_amdgcn_mfma_f32_16x16x32_bf16(bf(qa[kk]), bf(kf[kk]), accA, 0, 0, 0);
    for (int u = 0; u < units; ++u) {
#pragma unroll
      for (int s = 0; s < 16; ++s) {      // 16 sub-tiles of 16 rows x 16 keys per unit of 128 rows and 32 keys
        const int sn = (s + 1) & 15, rg = s >> 1, rgn = sn >> 1, kgn = sn & 1;
        f32x4& cur = (s & 1) ? accB : accA;
        f32x4& nxt = (s & 1) ? accA : accB;
        u32x4* qn = (rgn & 1) ? qb : qa;
        if (kgn == 0) {
#pragma unroll
          for (int kk = 0; kk < 4; ++kk) qn[kk] = rdq(rgn, kk);
        }
        const f32x4 cv0 = *(const f32x4*)(&cst[rg * 16 + 4 * quad]);
        const f32x4 cv1 = *(const f32x4*)(&cst[rg * 16 + 4 * quad + 2]);
#pragma unroll
        for (int e = 0; e < 4; ++e) nxt[e] = 0.f;
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
          nxt = __builtin_amdgcn_mfma_f32_16x16x32_bf16(bf(qn[kk]), bf(kf[kgn * 4 + kk]), nxt, 0, 0, 0);
          elem(cur, cv0, cv1, kk);
          __builtin_amdgcn_sched_barrier(0);
        }
        if ((s & 3) == 3) { col64 += (double)(cs0 + cs1); cs0 = 0.f; cs1 = 0.f; }
      }
    }
    cs0 += accA[0] + accB[0];
  }
  if (MODE == 4) {
    if (((wave >> 2) & 1) == 0) {
      for (int u = 0; u < units; ++u) {
#pragma unroll
        for (int rt = 0; rt < 4; ++rt) { mfma_part(rt); pin(); vector_part(rt); pin(); }
      }
    } else {
      for (int u = 0; u < units; ++u) {
#pragma unroll
        for (int rt = 0; rt < 4; ++rt) { vector_part((rt + 3) & 3); pin(); mfma_part(rt); pin(); }
      }
      vector_part(3);
    }
  }
  if (tid == 0 && blockIdx.x == 0) { clk[0] = clock64() - c0; clk[1] = wall_clock64() - w0; }
  out[blockIdx.x * 1024 + tid] = (float)col64 + cs0 + cs1;
}

enum { OP_FMA, OP_ADD, OP_EXP, OP_MAX, OP_CVT, OP_XOR, OP_FMA64, OP_LDS };
static const char* kOpNames[] = {"v_fma_f32", "v_add_f32", "v_exp_f32", "v_max_f32", "v_cvt_f32_i32", "v_xor_b32",
                                 "v_fma_f64", "ds_read_b128"};
template <int OP>
__device__ __forceinline__ void vop(float& t, float a, float b, double& d, u32x4& l, const unsigned char* lds) {
  if (OP == OP_FMA) asm volatile("v_fma_f32 %0, %0, %1, %2" : "+v"(t) : "v"(a), "v"(b));
  if (OP == OP_ADD) asm volatile("v_add_f32 %0, %0, %1" : "+v"(t) : "v"(b));
  if (OP == OP_EXP) asm volatile("v_exp_f32 %0, %0" : "+v"(t));
  if (OP == OP_MAX) asm volatile("v_max_f32 %0, %0, %1" : "+v"(t) : "v"(b));
  if (OP == OP_CVT) asm volatile("v_cvt_f32_i32 %0, %0" : "+v"(t));
  if (OP == OP_XOR) asm volatile("v_xor_b32 %0, %0, %1" : "+v"(t) : "v"(b));
  if (OP == OP_FMA64) asm volatile("v_fma_f64 %0, %0, %0, %0" : "+v"(d));
  if (OP == OP_LDS) asm volatile("ds_read_b128 %0, %1" : "=v"(l) : "v"((unsigned)(size_t)lds));
}
// 16 slices per iteration: one MFMA of a dependent chain (two accumulators in turn) and NV instructions of one kind
// on private registers
template <int OP, int NV, bool MF>
__global__ __launch_bounds__(1024) void k_issue(float* out, long long* clk, int iters) {
  __shared__ __align__(16) unsigned char lds[1024 * 16];
  const int tid = threadIdx.x;
  for (int i = tid; i < 4096; i += 1024) ((unsigned*)lds)[i] = rnd_bf16x2(i);
  __syncthreads();
  u32x4 kf[8], qv[8];
  for (int kk = 0; kk < 8; ++kk)
    for (int j = 0; j < 4; ++j) {
      kf[kk][j] = rnd_bf16x2(tid * 64 + kk * 4 + j);
      qv[kk][j] = rnd_bf16x2(tid * 64 + kk * 4 + j + 77777);
    }
  f32x16 accA, accB;
  for (int e = 0; e < 16; ++e) { accA[e] = 0.f; accB[e] = 0.f; }
  float t[12];
  for (int i = 0; i < 12; ++i) t[i] = tid * 0.001f + i * 0.01f;
  double d = tid;
  u32x4 l = {0, 0, 0, 0};
  const float a = 0.999f, b = 0.001f;
  const unsigned char* lp = lds + (tid & 63) * 16;
  long long c0 = 0, w0 = 0;
  if (tid == 0) { c0 = clock64(); w0 = wall_clock64(); }
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int sl = 0; sl < 16; ++sl) {
      if (MF) {
        if (sl < 8) accA = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bf(kf[sl & 7]), bf(qv[sl & 7]), accA, 0, 0, 0);
        else accB = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bf(kf[sl & 7]), bf(qv[sl & 7]), accB, 0, 0, 0);
      }
#pragma unroll
      for (int i = 0; i < NV; ++i) vop<OP>(t[i % 12], a, b, d, l, lp);
      __builtin_amdgcn_sched_barrier(0);
    }
    if (MF) { accA[0] *= 0.0f; accB[0] *= 0.0f; }
  }
  if (tid == 0 && blockIdx.x == 0) { clk[0] = clock64() - c0; clk[1] = wall_clock64() - w0; }
  float s = 0;
  for (int e = 0; e < 16; ++e) s += accA[e] + accB[e];
  for (int i = 0; i < 12; ++i) s += t[i];
  out[blockIdx.x * 1024 + tid] = s + (float)d + __builtin_bit_cast(float, l[0]);
}

// part C.  LEVEL 0: free-running tiles (one row buffer).  1: + barrier per unit.  2: + rows staged (global ->
// registers at the top of a unit, registers -> LDS at its end, double buffer).  3: + key operands reloaded
// every 5 units (a work-group's 128 KB).  4: + the per-row table staged per unit.
template <int LEVEL>
__global__ __launch_bounds__(1024) void k_morph(float* out, int units, float c, long long* clk, const u32x4* __restrict__ gq,
                                                const u32x4* __restrict__ gk, const float2* __restrict__ gc) {
  __shared__ __align__(16) unsigned char q[2][128 * kQRow];
  __shared__ __align__(16) float2 cst[2][128];
  const int tid = threadIdx.x, lane = tid & 63, l32 = lane & 31, half = lane >> 5;
  for (int b = 0; b < 2; ++b) {
    for (int i = tid; i < 128 * kQRow / 4; i += 1024) ((unsigned*)q[b])[i] = rnd_bf16x2(i + b * 7777);
    for (int i = tid; i < 128; i += 1024) cst[b][i] = make_float2(-3.0f - 0.01f * i, 1.0f / (1.0f + i));
  }
  __syncthreads();
  u32x4 kf[8];
  for (int kk = 0; kk < 8; ++kk)
    for (int j = 0; j < 4; ++j) kf[kk][j] = rnd_bf16x2(tid * 64 + kk * 4 + j + 12345);
  double col64 = 0.0;
  long long c0 = 0, w0 = 0;
  if (tid == 0) { c0 = clock64(); w0 = wall_clock64(); }
  f32x16 acc;
  const int my_row = tid / 16, my_col = tid % 16;      // staging: 128 rows x 16 pieces, rows r and r + 64 per thread
  u32x4 pre0 = {0, 0, 0, 0}, pre1 = {0, 0, 0, 0};
  float2 pre_c = make_float2(0.f, 0.f);
  for (int u = 0; u < units; ++u) {
    const int buf = LEVEL >= 2 ? (u & 1) : 0;
    if (LEVEL >= 2) {      // every work-group streams the same 40 units of 32 KB, as the sweeps stream one window
      const u32x4* src = gq + (size_t)((u + 1) % 40) * 2048;
      pre0 = src[my_row * 16 + my_col];
      pre1 = src[(my_row + 64) * 16 + my_col];
    }
    if (LEVEL >= 4) pre_c = gc[((u + 1) % 40) * 128 + (tid & 127)];
#pragma unroll
    for (int rt = 0; rt < 4; ++rt) {
      u32x4 qv[8];
#pragma unroll
      for (int kk = 0; kk < 8; ++kk) qv[kk] = *(const u32x4*)(&q[buf][(rt * 32 + l32) * kQRow + half * 16 + kk * 32]);
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[e] = 0.f;
#pragma unroll
      for (int kk = 0; kk < 8; ++kk) acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bf(qv[kk]), bf(kf[kk]), acc, 0, 0, 0);
      if (LEVEL >= 3 && rt == 3 && (u % 5) == 4) {
        const u32x4* ks = gk + ((size_t)blockIdx.x * 1024 + tid) * 64 + (size_t)((u / 5) % 8) * 8;
#pragma unroll
        for (int kk = 0; kk < 8; ++kk) kf[kk] = ks[kk];
      }
      float a0 = 0.f, a1 = 0.f;
#pragma unroll
      for (int e = 0; e < 16; e += 2) {
        const int row0 = rt * 32 + 8 * (e >> 2) + 4 * half + (e & 3);
        const f32x4 cv = *(const f32x4*)(&cst[LEVEL >= 4 ? buf : 0][row0]);
        a0 = fmaf(ex2(fmaf(acc[e], c, cv[0])), cv[1], a0);
        a1 = fmaf(ex2(fmaf(acc[e + 1], c, cv[2])), cv[3], a1);
      }
      col64 += (double)(a0 + a1);
      asm volatile("" : "+v"(col64) : : "memory");
      __builtin_amdgcn_sched_barrier(0);
    }
    if (LEVEL >= 2) {
      *(u32x4*)(&q[buf ^ 1][my_row * kQRow + my_col * 16]) = pre0;
      *(u32x4*)(&q[buf ^ 1][(my_row + 64) * kQRow + my_col * 16]) = pre1;
    }
    if (LEVEL >= 4 && tid < 128) cst[buf ^ 1][tid] = pre_c;
    if (LEVEL >= 1) __syncthreads();
  }
  if (tid == 0 && blockIdx.x == 0) { clk[0] = clock64() - c0; clk[1] = wall_clock64() - w0; }
  out[blockIdx.x * 1024 + tid] = (float)col64;
}
__global__ void k_fill_bits(unsigned* p, size_t n, unsigned salt) {
  for (size_t i = blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256) p[i] = rnd_bf16x2((unsigned)i + salt);
}
__global__ void k_fill_table(float2* p, int n) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i < n) p[i] = make_float2(-3.0f - 0.01f * (i & 127), 1.0f / (1.0f + (i & 127)));
}

static float* g_out;
static long long* g_clk;
template <class F>
static float time_ms(F f, int reps) {
  hipEvent_t a, b;
  CHECK(hipEventCreate(&a));
  CHECK(hipEventCreate(&b));
  f();
  CHECK(hipDeviceSynchronize());
  CHECK(hipEventRecord(a));
  for (int i = 0; i < reps; ++i) f();
  CHECK(hipEventRecord(b));
  CHECK(hipEventSynchronize(b));
  float ms;
  CHECK(hipEventElapsedTime(&ms, a, b));
  return ms / reps;
}
static double ghz_of_last_run() {
  long long h[2];
  CHECK(hipMemcpy(h, g_clk, sizeof(h), hipMemcpyDeviceToHost));
  return (double)h[0] / ((double)h[1] / 100e6) / 1e9;
}
template <int MODE>
static void run_tile(const char* name, int units) {
  const float ms = time_ms([&] { hipLaunchKernelGGL((k_tile<MODE>), dim3(256), dim3(1024), 0, 0, g_out, units, 0.1275f, g_clk); }, 5);
  const double ghz = ghz_of_last_run();
  const double tiles = (double)units * 4 * 4;      // 32x32 tiles per SIMD (4 waves per SIMD)
  printf("| %-66s | %7.1f | %6.1f | %5.0f | %4.2f |\n", name, ms * 1e3, ms * 1e6 / tiles, ms * 1e6 / tiles * ghz, ghz);
  fflush(stdout);
}
template <int OP, int NV>
static void run_issue(int iters) {
  auto one = [&](auto kern, double& ns, double& ghz) {
    const float ms = time_ms([&] { hipLaunchKernelGGL(kern, dim3(256), dim3(1024), 0, 0, g_out, g_clk, iters); }, 3);
    ghz = ghz_of_last_run();
    ns = ms * 1e6 / ((double)iters * 16 * 4);      // per slice and SIMD
  };
  double nm, gm, nv, gv, nb, gb;
  one(k_issue<OP, 0, true>, nm, gm);
  one(k_issue<OP, NV, false>, nv, gv);
  one(k_issue<OP, NV, true>, nb, gb);
  printf("| %-14s x %2d | %5.1f ns  %5.1f cyc  %4.2f GHz | %5.1f ns  %5.1f cyc (%4.2f each)  %4.2f GHz | %5.1f ns  %5.1f cyc  %4.2f GHz |\n",
         kOpNames[OP], NV, nm, nm * gm, gm, nv, nv * gv, nv * gv / NV, gv, nb, nb * gb, gb);
  fflush(stdout);
}

static u32x4 *g_rows, *g_keys;
static float2* g_table;
template <int LEVEL>
static void run_morph(const char* name, int units) {
  const float ms = time_ms([&] {
    hipLaunchKernelGGL((k_morph<LEVEL>), dim3(256), dim3(1024), 0, 0, g_out, units, 0.1275f, g_clk, g_rows, g_keys, g_table);
  }, 5);
  const double ghz = ghz_of_last_run();
  const double tiles = (double)units * 4 * 4;
  printf("| %-66s | %7.1f | %6.1f | %5.0f | %4.2f |\n", name, ms * 1e3, ms * 1e6 / tiles, ms * 1e6 / tiles * ghz, ghz);
  fflush(stdout);
}

int main() {
  CHECK(hipMalloc(&g_out, 256 * 1024 * 4));
  CHECK(hipMalloc(&g_clk, 64));
  const int units = 160;
  printf("part A: one tile of 32 rows x 32 keys x 128 per wave, 16 waves per work-group, 256 work-groups, random bf16 bits\n");
  printf("| %-66s | us      | ns/tile | cycles/tile | GHz |\n|---|---|---|---|---|\n", "order of the work (time and cycles per tile and SIMD)");
  for (int rep = 0; rep < 2; ++rep) {
    run_tile<1>("MFMA part only (8 operand reads, 8 x 32x32x16)", units);
    run_tile<2>("vector part only (16 x (fma, exp, fma), constants from LDS)", units);
    run_tile<0>("both, tile after tile", units);
    run_tile<3>("both, 16x16x32 sub-tiles software-pipelined inside the wave", units);
    run_tile<4>("both, half of the waves one phase late", units);
  }
  printf("\npart B: per slice and SIMD, 4 waves per SIMD: one MFMA alone | the vector instructions alone | both\n");
  printf("| instructions per MFMA | MFMA alone | vector alone | both |\n|---|---|---|---|\n");
  const int iters = 2000;
  run_issue<OP_FMA, 12>(iters);
  run_issue<OP_ADD, 12>(iters);
  run_issue<OP_XOR, 12>(iters);
  run_issue<OP_MAX, 12>(iters);
  run_issue<OP_CVT, 12>(iters);
  run_issue<OP_EXP, 6>(iters);
  run_issue<OP_EXP, 12>(iters);
  run_issue<OP_FMA64, 6>(iters);
  run_issue<OP_LDS, 6>(iters);

  const size_t n_rows = 40 * 2048, n_keys = (size_t)256 * 1024 * 64;      // 16-byte pieces: 1.25 MB of rows, 256 MB of keys
  CHECK(hipMalloc(&g_rows, n_rows * 16));
  CHECK(hipMalloc(&g_keys, n_keys * 16));
  CHECK(hipMalloc(&g_table, 40 * 128 * sizeof(float2)));
  hipLaunchKernelGGL(k_fill_bits, dim3(1024), dim3(256), 0, 0, (unsigned*)g_rows, n_rows * 4, 1u);
  hipLaunchKernelGGL(k_fill_bits, dim3(4096), dim3(256), 0, 0, (unsigned*)g_keys, n_keys * 4, 99u);
  hipLaunchKernelGGL(k_fill_table, dim3(20), dim3(256), 0, 0, g_table, 40 * 128);
  CHECK(hipDeviceSynchronize());
  printf("\npart C: the tile of part A (both pipes) rebuilt toward the sweep kernel's loop, 160 units of 4 tiles per wave\n");
  printf("| %-66s | us      | ns/tile | cycles/tile | GHz |\n|---|---|---|---|---|\n", "what the loop does besides the tiles");
  for (int rep = 0; rep < 2; ++rep) {
    run_morph<0>("nothing (free-running tiles)", units);
    run_morph<1>("+ a barrier per unit of four tiles", units);
    run_morph<2>("+ rows staged global -> registers -> LDS, double buffer", units);
    run_morph<3>("+ key operands reloaded every fifth unit (128 KB per work-group)", units);
    run_morph<4>("+ per-row table staged per unit", units);
  }
  return 0;
}
