// Model of one scoring pass of the one-workgroup-per-problem kernel at the size of the C4
// workload (192 prompt rows, d_k = 128, 150 key blocks of 32 per workgroup, 256 workgroups,
// every workgroup its own keys: 315 MB per pass), stripped of everything but the inner loop.
// It answers where the time of a pass goes:
//   A  the shipped operand scheme: 8 waves, a wave takes whole key blocks (keys straight from
//      memory into the A operands, one block ahead) and reads the prompt-row operand of every
//      matrix instruction from LDS
//   Q  the alternative that reads nothing from LDS in the loop: a wave keeps three of the six
//      row blocks in registers, waves w and w + 4 go over the same key blocks
//   P  pairs of waves on different SIMDs (2p, 2p + 1) share the key blocks p, p + 4, ...: three
//      row blocks each in registers, the key blocks go from memory into LDS slots of the pair
//      (row-contiguous global_load_lds, each wave its half, several blocks ahead) and both read
//      their operands from the slot; flags in LDS say "my half has landed" and "I have read it"
// each with the keys from memory, with every workgroup reading the same eight blocks (the
// loads hit in L2), and without loads.
//
//   hipcc --offload-arch=gfx950 -O3 -Xclang -target-feature -Xclang -packed-fp32-ops -o pass_model pass_model.hip && ./pass_model
#include <hip/hip_runtime.h>
#include <cstdio>
#include <cstdlib>
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
#define GLOBAL __attribute__((address_space(1)))
constexpr int D = 128, KS = D / 16, QS = D * 2 + 16, QB = 6;
#define MFMA(a, b, c) __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0)

// MODE 0: this workgroup's own keys; 1: the same eight blocks for everyone; 2: no loads
template <int MODE>
__device__ __forceinline__ void load_keys(const GLOBAL u32x4* K, int blk, int lane, bf16x8 (&kf)[KS]) {
  if (MODE == 2) { kf[0][0] = (__bf16)(float)blk; return; }
  if (MODE == 1) blk &= 7;
  const GLOBAL u32x4* rp = K + ((size_t)blk * 32 + (lane & 31)) * 16;
  const int h = lane >> 5;
#pragma unroll
  for (int s = 0; s < KS; ++s) kf[s] = __builtin_bit_cast(bf16x8, rp[2 * s + h]);
}
__device__ __forceinline__ void column_sums(const f32x16& a, float L, float sc, float (&u)[16]) {
#pragma unroll
  for (int v = 0; v < 16; ++v) u[v] += __builtin_amdgcn_exp2f(__builtin_fmaf(a[v], sc, -L));
}
__device__ __forceinline__ float fold(const float (&u)[16]) { float s = 0; for (int v = 0; v < 16; ++v) s += u[v]; return s; }

template <int MODE>
__global__ __launch_bounds__(512) void model_a(const char* Q, const char* Kall, float* out, int nblk) {
  extern __shared__ __align__(16) char smem[];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  for (int i = tid; i < QB * 32 * (D / 8); i += 512) {
    const int row = i / (D / 8), seg = i % (D / 8);
    *(u32x4*)(smem + row * QS + seg * 16) = ((const u32x4*)Q)[i];
  }
  __syncthreads();
  const GLOBAL u32x4* K = (const GLOBAL u32x4*)(Kall + (size_t)blockIdx.x * nblk * 32 * 256);
  const char* base = smem + (lane & 31) * QS + 16 * (lane >> 5);
  const float sc = 0.1275f;
  bf16x8 ka[KS], kb[KS];
  float tot = 0;
  auto process = [&](const bf16x8 (&kf)[KS]) {
    float u[16];
    for (int v = 0; v < 16; ++v) u[v] = 0;
    f32x16 acc[QB];
#pragma unroll
    for (int q = 0; q < QB + 2; q += 2) {   // row blocks in pairs, the vector work one pair behind
      if (q < QB) {
        const char* r0 = base + q * 32 * QS;
        const char* r1 = r0 + 32 * QS;
        f32x16 a0 = {0}, a1 = {0};
        bf16x8 c0 = *(const bf16x8*)r0, c1 = *(const bf16x8*)r1;
#pragma unroll
        for (int s = 0; s < KS; ++s) {
          bf16x8 n0 = c0, n1 = c1;
          if (s + 1 < KS) { n0 = *(const bf16x8*)(r0 + 32 * (s + 1)); n1 = *(const bf16x8*)(r1 + 32 * (s + 1)); }
          a0 = MFMA(kf[s], c0, a0); a1 = MFMA(kf[s], c1, a1);
          __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
          __builtin_amdgcn_sched_group_barrier(0x008, 2, 0);
          c0 = n0; c1 = n1;
        }
        acc[q] = a0; acc[q + 1] = a1;
      }
      if (q >= 2) { column_sums(acc[q - 2], 3.f + q, sc, u); column_sums(acc[q - 1], 4.f + q, sc, u); }
    }
    tot += fold(u);
  };
  int b = wave;
  if (b < nblk) load_keys<MODE>(K, b, lane, ka);
  while (b < nblk) {
    if (b + 8 < nblk) load_keys<MODE>(K, b + 8, lane, kb);
    process(ka); b += 8; if (b >= nblk) break;
    if (b + 8 < nblk) load_keys<MODE>(K, b + 8, lane, ka);
    process(kb); b += 8;
  }
  out[blockIdx.x * 512 + tid] = tot;
}

template <int MODE>
__global__ __launch_bounds__(512) void model_q(const char* Q, const char* Kall, float* out, int nblk) {
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int stream = wave & 3, half = wave >> 2;
  const GLOBAL u32x4* K = (const GLOBAL u32x4*)(Kall + (size_t)blockIdx.x * nblk * 32 * 256);
  const float sc = 0.1275f;
  bf16x8 qf[3][KS];
  {
    const GLOBAL u32x4* qp = (const GLOBAL u32x4*)Q;
#pragma unroll
    for (int q = 0; q < 3; ++q)
#pragma unroll
      for (int s = 0; s < KS; ++s)
        qf[q][s] = __builtin_bit_cast(bf16x8, qp[((size_t)(half * 3 + q) * 32 + (lane & 31)) * 16 + 2 * s + (lane >> 5)]);
  }
  bf16x8 ka[KS], kb[KS];
  float tot = 0;
  auto process = [&](const bf16x8 (&kf)[KS]) {
    float u[16];
    for (int v = 0; v < 16; ++v) u[v] = 0;
    f32x16 acc[3];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      if (q < 3) {
        f32x16 a0 = {0};
#pragma unroll
        for (int s = 0; s < KS; ++s) a0 = MFMA(kf[s], qf[q][s], a0);
        acc[q] = a0;
      }
      if (q >= 1) column_sums(acc[q - 1], 3.f + q, sc, u);
    }
    tot += fold(u);
  };
  int b = stream;
  if (b < nblk) load_keys<MODE>(K, b, lane, ka);
  while (b < nblk) {
    if (b + 4 < nblk) load_keys<MODE>(K, b + 4, lane, kb);
    process(ka); b += 4; if (b >= nblk) break;
    if (b + 4 < nblk) load_keys<MODE>(K, b + 4, lane, ka);
    process(kb); b += 4;
  }
  out[blockIdx.x * 512 + tid] = tot;
}

// P: waves 2p and 2p + 1 (on different SIMDs; partners on one SIMD are forced into the same
// phase and take 88 us) form a pair that shares the key blocks p, p + 4, ...: each keeps three of
// the six row blocks in registers; a key block goes from memory straight into an LDS slot of the
// pair (each wave requests its half with row-contiguous global_load_lds), DEPTH blocks ahead, and
// both read their A operands from the slot.  Flags in LDS tell the partner that a half has landed
// and that a slot has been read; every wait on a flag is bounded.
typedef __attribute__((address_space(3))) void lds_void;
template <int MODE, int DEPTH>
__global__ __launch_bounds__(512) void model_p(const char* Q, const char* Kall, float* out, int nblk) {
  extern __shared__ __align__(16) char smem[];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int pair = wave >> 1, half = wave & 1;   // partners on different SIMDs
  const GLOBAL char* K = (const GLOBAL char*)(Kall + (size_t)blockIdx.x * nblk * 32 * 256);
  char* slots = smem + (size_t)pair * DEPTH * 8192;
  volatile int* flags = (volatile int*)(smem + 4 * DEPTH * 8192);   // [pair][half][2][DEPTH]
  volatile int* landed_me = flags + ((pair * 2 + half) * 2 + 0) * DEPTH;
  volatile int* done_me = flags + ((pair * 2 + half) * 2 + 1) * DEPTH;
  volatile int* landed_other = flags + ((pair * 2 + (1 - half)) * 2 + 0) * DEPTH;
  volatile int* done_other = flags + ((pair * 2 + (1 - half)) * 2 + 1) * DEPTH;
  for (int i = tid; i < 4 * 2 * 2 * DEPTH; i += 512) flags[i] = 0;
  __syncthreads();
  const float sc = 0.1275f;
  bf16x8 qf[3][KS];
  {
    const GLOBAL u32x4* qp = (const GLOBAL u32x4*)Q;
#pragma unroll
    for (int q = 0; q < 3; ++q)
#pragma unroll
      for (int s = 0; s < KS; ++s)
        qf[q][s] = __builtin_bit_cast(bf16x8, qp[((size_t)(half * 3 + q) * 32 + (lane & 31)) * 16 + 2 * s + (lane >> 5)]);
  }
  const int n_i = pair < nblk ? (nblk - pair + 3) / 4 : 0;
  auto request = [&](int i) {
    int blk = pair + 4 * i;
    if (MODE == 1) blk &= 7;
    char* slot = slots + (i % DEPTH) * 8192;
#pragma unroll
    for (int jj = 0; jj < 4; ++jj) {
      const int j = 4 * half + jj;
      const int r = 4 * j + (lane >> 4);
      const int p = (lane & 15) ^ (r & 7);
      const GLOBAL char* src = K + ((size_t)blk * 32 + r) * 256 + p * 16;
      __builtin_amdgcn_global_load_lds((const GLOBAL void*)src, (lds_void*)(slot + j * 1024), 16, 0, 0);
    }
  };
  auto fetch = [&](int i, bf16x8 (&kf)[KS]) {
    const char* slot = slots + (i % DEPTH) * 8192;
    const int t = lane & 31, h = lane >> 5;
#pragma unroll
    for (int s2 = 0; s2 < KS; ++s2) kf[s2] = *(const bf16x8*)(slot + t * 256 + (((2 * s2 + h) ^ (t & 7)) * 16));
  };
  auto wait_for = [&](volatile int* f, int want) {
    int guard = 1 << 20;
    while (*f < want && --guard) __builtin_amdgcn_s_sleep(1);
  };
  float tot = 0;
  auto process = [&](const bf16x8 (&kf)[KS]) {
    float u[16];
    for (int v = 0; v < 16; ++v) u[v] = 0;
    f32x16 acc[3];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      if (q < 3) {
        f32x16 a0 = {0};
#pragma unroll
        for (int s = 0; s < KS; ++s) a0 = MFMA(kf[s], qf[q][s], a0);
        acc[q] = a0;
      }
      if (q >= 1) column_sums(acc[q - 1], 3.f + q, sc, u);
    }
    tot += fold(u);
  };
  if (MODE != 2)
    for (int i = 0; i < DEPTH && i < n_i; ++i) request(i);
  bf16x8 ka[KS];
  for (int i = 0; i < n_i; ++i) {
    const int s = i % DEPTH;
    if (MODE != 2) {
      // requests are served in order: my half of block i is in the slot when at most the
      // requests of the blocks after it are outstanding
      const int later = min(DEPTH - 1, n_i - 1 - i);
      if (later >= 3) asm volatile("s_waitcnt vmcnt(12)" ::: "memory");
      else if (later == 2) asm volatile("s_waitcnt vmcnt(8)" ::: "memory");
      else if (later == 1) asm volatile("s_waitcnt vmcnt(4)" ::: "memory");
      else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
      if (lane == 0) landed_me[s] = i + 1;
      wait_for(landed_other + s, i + 1);
    }
    fetch(i, ka);
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    if (MODE != 2) {
      if (lane == 0) done_me[s] = i + 1;
    }
    process(ka);
    if (MODE != 2 && i + DEPTH < n_i) {
      wait_for(done_other + s, i + 1);
      request(i + DEPTH);
    }
  }
  out[blockIdx.x * 512 + tid] = tot;
}

#define CK(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { printf("%s: %s\n", #x, hipGetErrorString(e_)); return 1; } } while (0)

int main() {
  const int nblk = 150, wgs = 256;
  char *Q, *K; float* out;
  CK(hipMalloc(&Q, QB * 32 * 256)); CK(hipMemset(Q, 0x3c, QB * 32 * 256));
  const size_t kbytes = (size_t)wgs * nblk * 32 * 256;
  CK(hipMalloc(&K, kbytes)); CK(hipMemset(K, 0x3c, kbytes));
  CK(hipMalloc(&out, wgs * 512 * 4));
  const size_t lds = QB * 32 * QS;
  CK(hipFuncSetAttribute((const void*)&model_a<0>, hipFuncAttributeMaxDynamicSharedMemorySize, 100 * 1024));
  CK(hipFuncSetAttribute((const void*)&model_a<1>, hipFuncAttributeMaxDynamicSharedMemorySize, 100 * 1024));
  CK(hipFuncSetAttribute((const void*)&model_a<2>, hipFuncAttributeMaxDynamicSharedMemorySize, 100 * 1024));
  hipEvent_t e0, e1; CK(hipEventCreate(&e0)); CK(hipEventCreate(&e1));
  constexpr int DP = 4;
  const size_t lds_p = 4 * DP * 8192 + 4 * 2 * 2 * DP * 4;
  CK(hipFuncSetAttribute((const void*)&model_p<0, DP>, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024));
  CK(hipFuncSetAttribute((const void*)&model_p<1, DP>, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024));
  CK(hipFuncSetAttribute((const void*)&model_p<2, DP>, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024));
  CK(hipFuncSetAttribute((const void*)&model_p<0, 2>, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024));
  const char* names[10] = {"A prompt rows from LDS", "A, keys from L2", "A, no key loads",
                          "Q three row blocks in registers", "Q, keys from L2", "Q, no key loads",
                          "P pairs, keys through LDS, depth 4", "P, keys from L2", "P, no key loads", "P depth 2"};
  auto launch = [&](int which) {
    switch (which) {
      case 0: hipLaunchKernelGGL(model_a<0>, dim3(wgs), dim3(512), lds, 0, Q, K, out, nblk); break;
      case 1: hipLaunchKernelGGL(model_a<1>, dim3(wgs), dim3(512), lds, 0, Q, K, out, nblk); break;
      case 2: hipLaunchKernelGGL(model_a<2>, dim3(wgs), dim3(512), lds, 0, Q, K, out, nblk); break;
      case 3: hipLaunchKernelGGL(model_q<0>, dim3(wgs), dim3(512), 0, 0, Q, K, out, nblk); break;
      case 4: hipLaunchKernelGGL(model_q<1>, dim3(wgs), dim3(512), 0, 0, Q, K, out, nblk); break;
      case 5: hipLaunchKernelGGL(model_q<2>, dim3(wgs), dim3(512), 0, 0, Q, K, out, nblk); break;
      case 6: hipLaunchKernelGGL((model_p<0, DP>), dim3(wgs), dim3(512), lds_p, 0, Q, K, out, nblk); break;
      case 7: hipLaunchKernelGGL((model_p<1, DP>), dim3(wgs), dim3(512), lds_p, 0, Q, K, out, nblk); break;
      case 8: hipLaunchKernelGGL((model_p<2, DP>), dim3(wgs), dim3(512), lds_p, 0, Q, K, out, nblk); break;
      default: hipLaunchKernelGGL((model_p<0, 2>), dim3(wgs), dim3(512), 4 * 2 * 8192 + 4 * 2 * 2 * 2 * 4, 0, Q, K, out, nblk); break;
    }
  };
  for (int rep = 0; rep < 3; ++rep)
    for (int which = 0; which < 10; ++which) {
      for (int i = 0; i < 3; ++i) launch(which);
      CK(hipEventRecord(e0));
      const int n = 40;
      for (int i = 0; i < n; ++i) launch(which);
      CK(hipEventRecord(e1)); CK(hipEventSynchronize(e1));
      float ms; CK(hipEventElapsedTime(&ms, e0, e1)); ms /= n;
      printf("%-34s: %6.1f us per pass of %d blocks (%5.1f ns per 32x32x128 tile per SIMD, %4.2f TB/s of keys)\n", names[which],
             ms * 1e3, nblk, ms * 1e6 / (nblk * QB / 4.0), kbytes / (ms * 1e-3) * 1e-12);
      fflush(stdout);
    }
  return hipGetLastError() == hipSuccess ? 0 : 1;
}
