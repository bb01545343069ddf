// Stand-alone measurement of what bounds the attention kernel on this chip: the
// rate of dense bf16 MFMA work under the chip's power limit as a function of the
// operand data, and the rate of a loop with the attention kernel's instruction mix
// per 64-key tile (MFMAs, LDS operand reads, exp2 / convert / row-sum vector work)
// without global loads and barriers - as the kernel has it (32 query columns per wave,
// 8 waves) and with 64 columns per wave (4 waves).  Not part of the library; prints a
// table, then a probe of whether a wave's vector work overlaps its own MFMAs.
// Build-time switches for ablations of the mix loop: see MIX_NO_* below.
//
//   hipcc --offload-arch=gfx950 -O3 -o ceiling_bench ceiling_bench.hip && ./ceiling_bench
#include <hip/hip_runtime.h>
#include <math.h>
#include <stdio.h>
#include <stdlib.h>
#include <vector>

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;
typedef const __attribute__((address_space(3))) unsigned char* lds_cptr;

#define CK(x)                                                                      \
  do {                                                                             \
    hipError_t e_ = (x);                                                           \
    if (e_ != hipSuccess) {                                                        \
      printf("HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__);        \
      exit(1);                                                                     \
    }                                                                              \
  } while (0)

constexpr int kBlocks = 256, kThreads = 512;

// 8 MFMAs per iteration and wave, four independent accumulators, operands in registers.
__global__ __launch_bounds__(512) void mfma_only(const u32x4* data, float* out, int iters, long long* clk) {
  const int tid = blockIdx.x * kThreads + threadIdx.x;
  union { u32x4 u; bf16x8 v; } a[8], b[8];
  for (int j = 0; j < 8; ++j) {
    a[j].u = data[(size_t)tid * 16 + j];
    b[j].u = data[(size_t)tid * 16 + 8 + j];
  }
  f32x16 o0 = {0}, o1 = {0}, o2 = {0}, o3 = {0};
  const long long t0 = clock64(), w0 = wall_clock64();
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int j = 0; j < 8; j += 4) {
      o0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[j].v, b[j].v, o0, 0, 0, 0);
      o1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[j + 1].v, b[j + 1].v, o1, 0, 0, 0);
      o2 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[j + 2].v, b[j + 2].v, o2, 0, 0, 0);
      o3 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[j + 3].v, b[j + 3].v, o3, 0, 0, 0);
    }
  }
  const long long t1 = clock64(), w1 = wall_clock64();
  float s = 0.f;
  for (int j = 0; j < 16; ++j) s += o0[j] + o1[j] + o2[j] + o3[j];
  out[tid] = s;
  if (blockIdx.x == 0 && threadIdx.x == 0) clk[0] = t1 - t0, clk[1] = w1 - w0;
}

// Ablations of the 32-column mix loop, chosen at build time (timing only; each keeps
// every MFMA): -DMIX_NO_K_READS / -DMIX_NO_V_READS reuse the fragment registers instead
// of reading LDS, -DMIX_NO_EXP replaces exp2 by the identity.
#ifdef MIX_NO_K_READS
#define LDKX(i, h) ka[i]
#else
#define LDKX(i, h) LDK(i, h)
#endif
#ifdef MIX_NO_V_READS
#define LDVX(i) vf[(i) & 3]
#else
#define LDVX(i) LDV(i)
#endif
#ifdef MIX_NO_EXP
#define EXPF(x) (x)
#else
#define EXPF(x) __builtin_amdgcn_exp2f(x)
#endif

// One iteration = one 64-key tile of a 256-row workgroup tile at D = 128, as the
// attention kernel runs it: two 32-key units per wave, each with 8 MFMAs of S^T
// (K fragments from LDS), 8 MFMAs of O^T (transposed V reads from LDS) and the
// exp2 / bf16 / row-sum work on 16 scores, interleaved step by step.
__global__ __launch_bounds__(512) void attention_mix(const unsigned short* rnd, float* out, int iters, long long* clk,
                                                     float c, float mc) {
  __shared__ __attribute__((aligned(1024))) unsigned char lds[65536];
  const int lane = threadIdx.x & 63, l32 = lane & 31, hi = lane >> 5;
  for (int i = threadIdx.x; i < 65536 / 2; i += kThreads) ((unsigned short*)lds)[i] = rnd[(size_t)blockIdx.x * 32768 + i];
  // the loop below reads LDS through offsets the compiler cannot trace back to `lds`:
  // without this it would drop the stores above as dead
  asm volatile("" ::"r"(&lds[0]) : "memory");
  __syncthreads();
  uint32_t kb_[8], vb_[4];
  for (int kk = 0; kk < 8; ++kk) {
    kb_[kk] = l32 * 256 + (((kk * 2 + hi) ^ (l32 & 15)) * 16);
    asm volatile("" : "+v"(kb_[kk]));
  }
  {
    const int j = lane & 15, half16 = (lane >> 4) & 1, vrow = 4 * hi + (j >> 2);
    for (int db = 0; db < 4; ++db) {
      const int lg = db * 4 + 2 * half16 + ((j & 3) >> 1);
      vb_[db] = 32768 + vrow * 256 + ((lg ^ ((vrow & 3) << 2)) * 16) + (j & 1) * 8;
      asm volatile("" : "+v"(vb_[db]));
    }
  }
  union { unsigned short u[8]; bf16x8 v; } ua, ub;
  for (int j = 0; j < 8; ++j) {
    ua.u[j] = rnd[(size_t)(blockIdx.x * kThreads + threadIdx.x) * 16 + j];
    ub.u[j] = rnd[(size_t)(blockIdx.x * kThreads + threadIdx.x) * 16 + 8 + j];
  }
  const bf16x8 a = ua.v, b = ub.v;
  bf16x8 ka[8] = {a, a, a, a, a, a, a, a}, vf[4] = {a, a, a, a};
  f32x16 s0 = {0}, s1 = {0}, o0 = {0}, o1 = {0}, o2 = {0}, o3 = {0};
  union { bf16x2 h[8]; bf16x8 v[2]; } pf[2];
  for (int j = 0; j < 8; ++j) pf[0].h[j] = pf[1].h[j] = bf16x2{(__bf16)1.0f, (__bf16)0.5f};
  const bf16x2 ones2 = {(__bf16)1.0f, (__bf16)1.0f};
  float rs0 = 0.f, rs1 = 0.f;
  __syncthreads();
  const long long t0 = clock64(), w0 = wall_clock64();
#define LDK(i, half) \
  (*(const __attribute__((address_space(3))) bf16x8*)((lds_cptr)(uintptr_t)kb_[(i) & 7] + (half) * 8192 + ((it & 1) * 16384)))
#define LDV(i)                                                                                              \
  ({                                                                                                        \
    lds_cptr vp = (lds_cptr)(uintptr_t)vb_[(i) & 3] + (((i) >> 2) & 1) * 4096;                               \
    union { struct { s16x4 x, y; } h; bf16x8 v; } cat;                                                       \
    cat.h.x = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3)))*)(vp));       \
    cat.h.y = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3)))*)(vp + 2048)); \
    cat.v;                                                                                                   \
  })
#define PVMF(i, PN)                                                                                                       \
  do {                                                                                                                    \
    if (((i) & 3) == 0) o0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[(i) & 3], pf[PN].v[(i) / 4], o0, 0, 0, 0);         \
    if (((i) & 3) == 1) o1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[(i) & 3], pf[PN].v[(i) / 4], o1, 0, 0, 0);         \
    if (((i) & 3) == 2) o2 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[(i) & 3], pf[PN].v[(i) / 4], o2, 0, 0, 0);         \
    if (((i) & 3) == 3) o3 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[(i) & 3], pf[PN].v[(i) / 4], o3, 0, 0, 0);         \
  } while (0)
#define EXPP(i, SC, PC)                                                                  \
  do {                                                                                   \
    float x0 = SC[2 * (i)], x1 = SC[2 * (i) + 1];                                        \
    asm volatile("" : "+v"(x0), "+v"(x1));                                               \
    const float p0 = EXPF(__builtin_fmaf(x0, c, -mc));                                   \
    const float p1 = EXPF(__builtin_fmaf(x1, c, -mc));                                   \
    bf16x2 pk;                                                                           \
    pk[0] = (__bf16)p0;                                                                  \
    pk[1] = (__bf16)p1;                                                                  \
    if ((i) & 1) {                                                                       \
      rs1 = __builtin_amdgcn_fdot2_f32_bf16(pk, ones2, rs1, false);                      \
      asm volatile("" : "+v"(pk), "+v"(rs1));                                            \
    } else {                                                                             \
      rs0 = __builtin_amdgcn_fdot2_f32_bf16(pk, ones2, rs0, false);                      \
      asm volatile("" : "+v"(pk), "+v"(rs0));                                            \
    }                                                                                    \
    pf[PC].h[i] = pk;                                                                    \
  } while (0)
#define UNIT(SN, SC, PC, PN, HALF)                                          \
  do {                                                                      \
    _Pragma("unroll") for (int r = 0; r < 16; ++r) SN[r] = 0.f;             \
    _Pragma("unroll") for (int i = 0; i < 8; ++i) {                         \
      SN = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka[i], b, SN, 0, 0, 0);  \
      ka[i] = LDKX(i, HALF);                                                \
      PVMF(i, PN);                                                          \
      vf[i & 3] = LDVX(i + 4);                                              \
      EXPP(i, SC, PC);                                                      \
      __builtin_amdgcn_sched_barrier(0);                                    \
    }                                                                       \
  } while (0)
  for (int it = 0; it < iters; ++it) {
    UNIT(s1, s0, 0, 1, 0);
    UNIT(s0, s1, 1, 0, 1);
  }
  const long long t1 = clock64(), w1 = wall_clock64();
  float s = rs0 + rs1;
  for (int j = 0; j < 16; ++j) s += s0[j] + s1[j] + o0[j] + o1[j] + o2[j] + o3[j];
  out[blockIdx.x * kThreads + threadIdx.x] = s;
  if (blockIdx.x == 0 && threadIdx.x == 0) clk[0] = t1 - t0, clk[1] = w1 - w0;
}

#undef LDK
#undef LDV
#undef PVMF
#undef EXPP
#undef UNIT
// The same tile with 64 query columns per wave (4 waves per workgroup, one per SIMD):
// every fragment read from LDS feeds two MFMAs, the accumulators spill over into the
// AGPR half of the register file.  Instruction order not tuned.
__global__ __launch_bounds__(256) void attention_mix64(const unsigned short* rnd, float* out, int iters, long long* clk,
                                                     float c, float mc) {
  __shared__ __attribute__((aligned(1024))) unsigned char lds[65536];
  const int lane = threadIdx.x & 63, l32 = lane & 31, hi = lane >> 5;
  for (int i = threadIdx.x; i < 65536 / 2; i += 256) ((unsigned short*)lds)[i] = rnd[(size_t)blockIdx.x * 32768 + i];
  // the loop below reads LDS through offsets the compiler cannot trace back to `lds`:
  // without this it would drop the stores above as dead
  asm volatile("" ::"r"(&lds[0]) : "memory");
  __syncthreads();
  uint32_t kb_[8], vb_[4];
  for (int kk = 0; kk < 8; ++kk) {
    kb_[kk] = l32 * 256 + (((kk * 2 + hi) ^ (l32 & 15)) * 16);
    asm volatile("" : "+v"(kb_[kk]));
  }
  {
    const int j = lane & 15, half16 = (lane >> 4) & 1, vrow = 4 * hi + (j >> 2);
    for (int db = 0; db < 4; ++db) {
      const int lg = db * 4 + 2 * half16 + ((j & 3) >> 1);
      vb_[db] = 32768 + vrow * 256 + ((lg ^ ((vrow & 3) << 2)) * 16) + (j & 1) * 8;
      asm volatile("" : "+v"(vb_[db]));
    }
  }
  union { unsigned short u[8]; bf16x8 v; } ua, ub;
  for (int j = 0; j < 8; ++j) {
    ua.u[j] = rnd[(size_t)(blockIdx.x * kThreads + threadIdx.x) * 16 + j];
    ub.u[j] = rnd[(size_t)(blockIdx.x * kThreads + threadIdx.x) * 16 + 8 + j];
  }
  const bf16x8 a = ua.v, b = ub.v;
  bf16x8 b2 = ub.v; asm volatile("" : "+v"(b2));
  bf16x8 ka[8] = {a, a, a, a, a, a, a, a}, vf[4] = {a, a, a, a};
  f32x16 s0 = {0}, s1 = {0}, o0 = {0}, o1 = {0}, o2 = {0}, o3 = {0};
  f32x16 t0_ = {0}, t1_ = {0}, q0 = {0}, q1 = {0}, q2 = {0}, q3 = {0};
  union { bf16x2 h[8]; bf16x8 v[2]; } pf[2], pg[2];
  for (int j = 0; j < 8; ++j) pf[0].h[j] = pf[1].h[j] = pg[0].h[j] = pg[1].h[j] = bf16x2{(__bf16)1.0f, (__bf16)0.5f};
  const bf16x2 ones2 = {(__bf16)1.0f, (__bf16)1.0f};
  float rs0 = 0.f, rs1 = 0.f, rt0 = 0.f, rt1 = 0.f;
  __syncthreads();
  const long long tt0 = clock64(), w0 = wall_clock64();
#define LDK(i, half) \
  (*(const __attribute__((address_space(3))) bf16x8*)((lds_cptr)(uintptr_t)kb_[(i) & 7] + (half) * 8192 + ((it & 1) * 16384)))
#define LDV(i)                                                                                              \
  ({                                                                                                        \
    lds_cptr vp = (lds_cptr)(uintptr_t)vb_[(i) & 3] + (((i) >> 2) & 1) * 4096;                               \
    union { struct { s16x4 x, y; } h; bf16x8 v; } cat;                                                       \
    cat.h.x = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3)))*)(vp));       \
    cat.h.y = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3)))*)(vp + 2048)); \
    cat.v;                                                                                                   \
  })
#define PVMF(i, PN)                                                                                                       \
  do {                                                                                                                    \
    if (((i) & 3) == 0) o0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[(i) & 3], pf[PN].v[(i) / 4], o0, 0, 0, 0);         \
    if (((i) & 3) == 1) o1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[(i) & 3], pf[PN].v[(i) / 4], o1, 0, 0, 0);         \
    if (((i) & 3) == 2) o2 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[(i) & 3], pf[PN].v[(i) / 4], o2, 0, 0, 0);         \
    if (((i) & 3) == 3) o3 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[(i) & 3], pf[PN].v[(i) / 4], o3, 0, 0, 0);         \
  } while (0)
#define PVMG(i, PN)                                                                                                       \
  do {                                                                                                                    \
    if (((i) & 3) == 0) q0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[(i) & 3], pg[PN].v[(i) / 4], q0, 0, 0, 0);         \
    if (((i) & 3) == 1) q1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[(i) & 3], pg[PN].v[(i) / 4], q1, 0, 0, 0);         \
    if (((i) & 3) == 2) q2 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[(i) & 3], pg[PN].v[(i) / 4], q2, 0, 0, 0);         \
    if (((i) & 3) == 3) q3 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[(i) & 3], pg[PN].v[(i) / 4], q3, 0, 0, 0);         \
  } while (0)
#define EXPQ(i, SC, PC)                                                                  \
  do {                                                                                   \
    float x0 = SC[2 * (i)], x1 = SC[2 * (i) + 1];                                        \
    asm volatile("" : "+v"(x0), "+v"(x1));                                               \
    const float p0 = __builtin_amdgcn_exp2f(__builtin_fmaf(x0, c, -mc));                 \
    const float p1 = __builtin_amdgcn_exp2f(__builtin_fmaf(x1, c, -mc));                 \
    bf16x2 pk;                                                                           \
    pk[0] = (__bf16)p0;                                                                  \
    pk[1] = (__bf16)p1;                                                                  \
    if ((i) & 1) {                                                                       \
      rt1 = __builtin_amdgcn_fdot2_f32_bf16(pk, ones2, rt1, false);                      \
      asm volatile("" : "+v"(pk), "+v"(rt1));                                            \
    } else {                                                                             \
      rt0 = __builtin_amdgcn_fdot2_f32_bf16(pk, ones2, rt0, false);                      \
      asm volatile("" : "+v"(pk), "+v"(rt0));                                            \
    }                                                                                    \
    pg[PC].h[i] = pk;                                                                    \
  } while (0)
#define EXPP(i, SC, PC)                                                                  \
  do {                                                                                   \
    float x0 = SC[2 * (i)], x1 = SC[2 * (i) + 1];                                        \
    asm volatile("" : "+v"(x0), "+v"(x1));                                               \
    const float p0 = __builtin_amdgcn_exp2f(__builtin_fmaf(x0, c, -mc));                 \
    const float p1 = __builtin_amdgcn_exp2f(__builtin_fmaf(x1, c, -mc));                 \
    bf16x2 pk;                                                                           \
    pk[0] = (__bf16)p0;                                                                  \
    pk[1] = (__bf16)p1;                                                                  \
    if ((i) & 1) {                                                                       \
      rs1 = __builtin_amdgcn_fdot2_f32_bf16(pk, ones2, rs1, false);                      \
      asm volatile("" : "+v"(pk), "+v"(rs1));                                            \
    } else {                                                                             \
      rs0 = __builtin_amdgcn_fdot2_f32_bf16(pk, ones2, rs0, false);                      \
      asm volatile("" : "+v"(pk), "+v"(rs0));                                            \
    }                                                                                    \
    pf[PC].h[i] = pk;                                                                    \
  } while (0)
#define UNIT(SN, SC, TN, TC, PC, PN, HALF)                                  \
  do {                                                                      \
    _Pragma("unroll") for (int r = 0; r < 16; ++r) SN[r] = 0.f, TN[r] = 0.f; \
    _Pragma("unroll") for (int i = 0; i < 8; ++i) {                         \
      SN = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka[i], b, SN, 0, 0, 0);  \
      TN = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka[i], b2, TN, 0, 0, 0); \
      ka[i] = LDK(i, HALF);                                                 \
      EXPP(i, SC, PC);                                                      \
      PVMF(i, PN);                                                          \
      PVMG(i, PN);                                                          \
      vf[i & 3] = LDV(i + 4);                                               \
      EXPQ(i, TC, PC);                                                      \
      __builtin_amdgcn_sched_barrier(0);                                    \
    }                                                                       \
  } while (0)
  for (int it = 0; it < iters; ++it) {
    UNIT(s1, s0, t1_, t0_, 0, 1, 0);
    UNIT(s0, s1, t0_, t1_, 1, 0, 1);
  }
  const long long tt1 = clock64(), w1 = wall_clock64();
  float s = rs0 + rs1 + rt0 + rt1;
  for (int j = 0; j < 16; ++j) s += s0[j] + s1[j] + o0[j] + o1[j] + o2[j] + o3[j] + t0_[j] + t1_[j] + q0[j] + q1[j] + q2[j] + q3[j];
  out[blockIdx.x * kThreads + threadIdx.x] = s;
  if (blockIdx.x == 0 && threadIdx.x == 0) clk[0] = tt1 - tt0, clk[1] = w1 - w0;
}

// Does a wave's vector work hide under its own MFMAs?  A loop of { MFMA ; NV independent
// v_fma_f32 } on alternating accumulators, with one and with two waves per SIMD.
template <int NV>
__global__ void overlap_probe(float* out, int iters, long long* clk, float c) {
  bf16x8 a, b;
  for (int j = 0; j < 8; ++j) {
    a[j] = (__bf16)(float)((threadIdx.x + j) & 7);
    b[j] = (__bf16)(float)(j + 1);
  }
  f32x16 acc0 = {0}, acc1 = {0};
  float x[8];
  for (int j = 0; j < 8; ++j) x[j] = (float)(threadIdx.x + j);
  __syncthreads();
  const long long t0 = clock64();
  for (int it = 0; it < iters; ++it) {
    acc0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc0, 0, 0, 0);
#pragma unroll
    for (int v = 0; v < NV; ++v) {
      x[v % 8] = __builtin_fmaf(x[v % 8], c, 1.0f);
      asm volatile("" : "+v"(x[v % 8]));
    }
    acc1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc1, 0, 0, 0);
#pragma unroll
    for (int v = 0; v < NV; ++v) {
      x[(v + 4) % 8] = __builtin_fmaf(x[(v + 4) % 8], c, 1.0f);
      asm volatile("" : "+v"(x[(v + 4) % 8]));
    }
    __builtin_amdgcn_sched_barrier(0);
  }
  const long long t1 = clock64();
  float s = 0;
  for (int j = 0; j < 16; ++j) s += acc0[j] + acc1[j];
  for (int j = 0; j < 8; ++j) s += x[j];
  out[blockIdx.x * blockDim.x + threadIdx.x] = s;
  // the slowest wave of workgroup 0 (waves that share a SIMD do not get equal shares)
  if (blockIdx.x == 0 && (threadIdx.x & 63) == 0) atomicMax((unsigned long long*)clk, (unsigned long long)(t1 - t0));
}

template <int NV>
static void run_overlap_probe(float* out, long long* clk, int threads) {
  const int iters = 20000;
  for (int r = 0; r < 3; ++r) {
    CK(hipMemset(clk, 0, 8));
    hipLaunchKernelGGL(overlap_probe<NV>, dim3(kBlocks), dim3(threads), 0, 0, out, iters, clk, 0.999f);
  }
  CK(hipDeviceSynchronize());
  long long c;
  CK(hipMemcpy(&c, clk, 8, hipMemcpyDeviceToHost));
  // cycles one SIMD spends per MFMA slot: a wave's cycles per MFMA, divided by the waves that share the SIMD
  printf("%d wave(s) per SIMD, %2d v_fma per MFMA: %6.1f cycles per MFMA and SIMD\n", threads / 256, NV,
         (double)c / iters / 2 / (threads / 256));
  fflush(stdout);
}

static unsigned short to_bf16(float f) {
  union { float f; unsigned int u; } cv;
  cv.f = f;
  unsigned int u = cv.u;
  u += 0x7fff + ((u >> 16) & 1);
  return (unsigned short)(u >> 16);
}

int main() {
  const size_t n = (size_t)kBlocks * kThreads * 16 * 8;   // bf16 elements: 16 x 16 bytes per thread
  std::vector<unsigned short> h(n);
  unsigned short* d;
  float* out;
  long long* clk;
  CK(hipMalloc(&d, n * 2));
  CK(hipMalloc(&out, kBlocks * kThreads * 4));
  CK(hipMalloc(&clk, 16));
  hipEvent_t e0, e1;
  CK(hipEventCreate(&e0));
  CK(hipEventCreate(&e1));
  const char* names[] = {"all zero", "all one", "N(0,1)", "all one (again)"};
  printf("%-44s %10s %12s\n", "loop / operand data", "TFLOP/s", "clock GHz");
  for (int kind = 0; kind < 3; ++kind) {
    for (int mode = (kind == 0 ? 0 : 1); mode < (kind == 0 ? 3 : 4); ++mode) {
      srand(1234);
      for (size_t i = 0; i < n; ++i) {
        const float u1 = (rand() + 1.0f) / ((float)RAND_MAX + 2.0f), u2 = (rand() + 1.0f) / ((float)RAND_MAX + 2.0f);
        h[i] = mode == 0 ? 0 : (mode & 1) ? 0x3f80 : to_bf16(sqrtf(-2.f * logf(u1)) * cosf(6.2831853f * u2));
      }
      CK(hipMemcpy(d, h.data(), n * 2, hipMemcpyHostToDevice));
      const int iters = kind == 0 ? 20000 : 4000, warm = kind == 0 ? 40 : 80, reps = kind == 0 ? 20 : 40;
      // warm-up: the clock needs ~100 ms of load to settle
      for (int w = 0; w < warm + reps; ++w) {
        if (w == warm) CK(hipEventRecord(e0));
        if (kind == 0) hipLaunchKernelGGL(mfma_only, dim3(kBlocks), dim3(kThreads), 0, 0, (const u32x4*)d, out, iters, clk);
        else if (kind == 1) hipLaunchKernelGGL(attention_mix, dim3(kBlocks), dim3(kThreads), 0, 0, d, out, iters, clk, 0.127f, 3.0f);
        else hipLaunchKernelGGL(attention_mix64, dim3(kBlocks), dim3(256), 0, 0, d, out, iters, clk, 0.127f, 3.0f);
      }
      CK(hipEventRecord(e1));
      CK(hipDeviceSynchronize());
      float ms;
      CK(hipEventElapsedTime(&ms, e0, e1));
      long long c[2];
      CK(hipMemcpy(c, clk, 16, hipMemcpyDeviceToHost));
      // mfma_only: 8 MFMAs of 32768 flop per iteration and wave; attention_mix: a 256 x 64 x 128 tile, 4 flop per element
      const double flop = (double)reps * kBlocks * iters * (kind == 0 ? 8.0 * 8 * 32768.0 : 256.0 * 64 * 128 * 4);
      char label[96];
      snprintf(label, sizeof label, "%s, %s", kind == 0 ? "MFMA only" : kind == 1 ? "attention kernel's mix per tile" : "mix, 64 columns per wave", names[mode]);
      printf("%-44s %10.0f %12.2f\n", label, flop / (ms * 1e-3) / 1e12, (double)c[0] / ((double)c[1] * 10.0));
      fflush(stdout);
    }
  }
  printf("\nown-wave overlap of vector work with MFMAs\n");
  for (int threads : {256, 512}) {
    run_overlap_probe<0>(out, clk, threads);
    run_overlap_probe<4>(out, clk, threads);
    run_overlap_probe<8>(out, clk, threads);
    run_overlap_probe<16>(out, clk, threads);
  }
  return 0;
}
