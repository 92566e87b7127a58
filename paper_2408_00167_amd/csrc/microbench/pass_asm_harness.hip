// Check against a CPU reference and timing of the pass loops pass_asm.py writes (an experiment beside
// the compiled kernels; the library does not use them).  With an argument the check does not stop the run.
#include <hip/hip_runtime.h>
#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>
#include "pass_asm_gen.h"

#define CK(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { printf("HIP error %s at %s:%d\n", hipGetErrorString(e_), __FILE__, __LINE__); exit(1); } } while (0)
constexpr int QB = 6, R = QB * 32, Dh = 128, QS = Dh * 2 + 16;
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

// LDS: Q rows [R][QS], then negL [R] floats, then zbuf [8][QB][64] floats, then 8 progress words (FAIR=1)
__global__ __launch_bounds__(512) void k_pass(int mode, const char* Q, const float* negl, const char* Kc, const char* Kk,
                                                size_t kc_stride, size_t kk_stride, float* scores, size_t sc_stride,
                                                float* zout, int c, int m, float sc, int fake_nw, unsigned long long* tick) {
  extern __shared__ __align__(16) char smem[];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, t = lane & 31, h = lane >> 5;
  for (int i = tid; i < R * (Dh / 8); i += 512) {
    int row = i / (Dh / 8), seg = i % (Dh / 8);
    *(u32x4*)(smem + row * QS + seg * 16) = ((const u32x4*)Q)[i];
  }
  float* lneg = (float*)(smem + R * QS);
  float* zbuf = lneg + R;
  for (int i = tid; i < R; i += 512) lneg[i] = negl[i];
  unsigned* prog = (unsigned*)(zbuf + 8 * QB * 64);
  if (tid < 8) prog[tid] = 0;
  const unsigned paddr = (unsigned)(size_t)(prog) + 4 * wave;
  __syncthreads();
  const int nbc = c / 32, nbk = m / 32, nbtot = nbc + nbk;
  int nw = wave < nbtot ? (nbtot - wave + 7) / 8 : 0;
  if (fake_nw) nw = fake_nw;   // timing only: blocks past the end repeat the wave's first block
  const char* kc = Kc + blockIdx.x * kc_stride;
  const char* kk = Kk + blockIdx.x * kk_stride;
  float* sp = scores + blockIdx.x * sc_stride;
  const unsigned qaddr = (unsigned)(size_t)(smem) + t * QS + 16 * h;   // LDS byte address (low 32 bits of the generic address)
  const unsigned laddr = (unsigned)(size_t)(lneg) + 4 * t;
  const unsigned zaddr = (unsigned)(size_t)(zbuf) + (wave * QB * 64 + lane) * 4;
  const unsigned rowoff = t * 256 + 16 * h;
  const int v = t >> 1;
  const unsigned stoff = 4 * (8 * (v >> 2) + 4 * h + (v & 3));
  const unsigned long long t0 = wall_clock64();
  if (nw > 0) {
    if (mode == 2) pass2_asm_qb6(kc, kk, sp, c, nbc, nbtot, wave, nw, sc, qaddr, laddr, rowoff, stoff, paddr);
    else pass1_asm_qb6(kc, kk, nbc, nbtot, wave, nw, sc, qaddr, laddr, rowoff, zaddr, paddr);
  }
  const unsigned long long t1 = wall_clock64();
  if (tick && lane == 0) { tick[blockIdx.x * 8 + wave] = t1 - t0; }
  if (mode == 1) {
    __syncthreads();
    for (int i = tid; i < 8 * QB * 64; i += 256) zout[(size_t)blockIdx.x * 8 * QB * 64 + i] = nw > 0 || true ? zbuf[i] : 0.f;
  }
}

static unsigned short f2bf(float f) { unsigned u; memcpy(&u, &f, 4); u += 0x7fff + ((u >> 16) & 1); return u >> 16; }
static float bf2f(unsigned short b) { unsigned u = (unsigned)b << 16; float f; memcpy(&f, &u, 4); return f; }
static float rnd() { return (rand() / (float)RAND_MAX - 0.5f) * 3.4f; }

int main(int argc, char** argv) {
  const float sc = 1.4426950408889634f / sqrtf(128.f);
  // ---- correctness: one workgroup, c = 96 cache rows (3 blocks), m = 32 * 35 chunk rows
  for (int test = 0; test < 3; ++test) {
    const int c = test == 0 ? 0 : (test == 1 ? 96 : 64), m = test == 0 ? 32 * 37 : (test == 1 ? 32 * 35 : 32 * 2), N = c + m;
    std::vector<unsigned short> hQ(R * Dh), hKc((size_t)(c ? c : 32) * Dh), hKk((size_t)m * Dh);
    srand(7 + test);
    for (auto& x : hQ) x = f2bf(rnd());
    for (auto& x : hKc) x = f2bf(rnd());
    for (auto& x : hKk) x = f2bf(rnd());
    std::vector<double> S((size_t)R * N);
    for (int i = 0; i < R; ++i)
      for (int j = 0; j < N; ++j) {
        const unsigned short* kr = j < c ? &hKc[(size_t)j * Dh] : &hKk[(size_t)(j - c) * Dh];
        double a = 0;
        for (int d = 0; d < Dh; ++d) a += (double)bf2f(hQ[i * Dh + d]) * bf2f(kr[d]);
        S[(size_t)i * N + j] = a * (double)sc;
      }
    std::vector<float> negl(R), negmu(R);
    std::vector<double> lse(R), zref(R);
    for (int i = 0; i < R; ++i) {
      double mx = -1e300;
      for (int j = 0; j < N; ++j) mx = fmax(mx, S[(size_t)i * N + j]);
      double z = 0;
      for (int j = 0; j < N; ++j) z += exp2(S[(size_t)i * N + j] - mx);
      lse[i] = mx + log2(z);
      negl[i] = -(float)lse[i];
      negmu[i] = 0.f;   // pass 1 takes no reference
      zref[i] = 0;
      for (int j = 0; j < N; ++j) zref[i] += exp2(S[(size_t)i * N + j] + (double)negmu[i]);
    }
    char *dQ, *dKc, *dKk; float *dL, *dS, *dZ;
    CK(hipMalloc(&dQ, hQ.size() * 2)); CK(hipMalloc(&dKc, hKc.size() * 2)); CK(hipMalloc(&dKk, hKk.size() * 2));
    CK(hipMalloc(&dL, R * 4)); CK(hipMalloc(&dS, (N + 64) * 4)); CK(hipMalloc(&dZ, 8 * QB * 64 * 4));
    CK(hipMemcpy(dQ, hQ.data(), hQ.size() * 2, hipMemcpyHostToDevice));
    CK(hipMemcpy(dKc, hKc.data(), hKc.size() * 2, hipMemcpyHostToDevice));
    CK(hipMemcpy(dKk, hKk.data(), hKk.size() * 2, hipMemcpyHostToDevice));
    CK(hipMemset(dS, 0xff, (N + 64) * 4));
    const size_t lds = R * QS + R * 4 + 8 * QB * 64 * 4 + 32 ;
    CK(hipFuncSetAttribute((const void*)k_pass, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
    // pass 2
    CK(hipMemcpy(dL, negl.data(), R * 4, hipMemcpyHostToDevice));
    printf("test %d: c=%d m=%d: launching pass 2\n", test, c, m); fflush(stdout);
    hipLaunchKernelGGL(k_pass, dim3(1), dim3(512), lds, 0, 2, dQ, dL, dKc, dKk, (size_t)0, (size_t)0, dS, (size_t)0, dZ, c, m, sc, 0, (unsigned long long*)nullptr);
    CK(hipDeviceSynchronize());
    std::vector<float> hS(N + 64);
    CK(hipMemcpy(hS.data(), dS, (N + 64) * 4, hipMemcpyDeviceToHost));
    double worst = 0; int bad = 0;
    for (int j = 0; j < N; ++j) {
      double want = 0;
      for (int i = 0; i < R; ++i) want += exp2(S[(size_t)i * N + j] - lse[i]);
      double rel = fabs(hS[j] - want) / want;
      if (!(rel < 1e-4)) { if (bad < 5) printf("  key %d: got %g want %g\n", j, hS[j], want); ++bad; }
      if (rel > worst) worst = rel;
    }
    unsigned guard; memcpy(&guard, &hS[N], 4);
    printf("  pass 2: worst rel err %.3e, bad %d, guard %08x\n", worst, bad, guard);
    // pass 1
    CK(hipMemcpy(dL, negmu.data(), R * 4, hipMemcpyHostToDevice));
    printf("  launching pass 1\n"); fflush(stdout);
    hipLaunchKernelGGL(k_pass, dim3(1), dim3(512), lds, 0, 1, dQ, dL, dKc, dKk, (size_t)0, (size_t)0, dS, (size_t)0, dZ, c, m, sc, 0, (unsigned long long*)nullptr);
    CK(hipDeviceSynchronize());
    std::vector<float> hZ(8 * QB * 64);
    CK(hipMemcpy(hZ.data(), dZ, hZ.size() * 4, hipMemcpyDeviceToHost));
    worst = 0; bad = 0;
    const int nbtot = c / 32 + m / 32;
    for (int i = 0; i < R; ++i) {
      double got = 0;
      for (int w = 0; w < 8; ++w) if (w < nbtot) for (int h = 0; h < 2; ++h) got += hZ[(w * QB + i / 32) * 64 + h * 32 + (i % 32)];
      double rel = fabs(got - zref[i]) / zref[i];
      if (!(rel < 1e-4)) { if (bad < 5) printf("  row %d: got %g want %g\n", i, got, zref[i]); ++bad; }
      if (rel > worst) worst = rel;
    }
    printf("  pass 1: worst rel err %.3e, bad %d\n", worst, bad); fflush(stdout);
    hipFree(dQ); hipFree(dKc); hipFree(dKk); hipFree(dL); hipFree(dS); hipFree(dZ);
    if (bad && argc < 2) return 1;
  }
  // ---- timing: 256 workgroups, 149 blocks of chunk keys each, distinct keys (312 MB), several region strides
  {
    const int WG = 256, m = 149 * 32, c = 0;
    const size_t kbytes = (size_t)m * 256;
    const size_t strides[] = {kbytes, (size_t)1 << 25, ((size_t)1 << 25) + 4096 * 13, ((size_t)1 << 25) + 256 * 77, (size_t)1 << 26};
    char *dQ, *dK; float *dL, *dS, *dZ;
    CK(hipMalloc(&dQ, R * Dh * 2)); CK(hipMalloc(&dK, ((size_t)1 << 26) * WG + kbytes)); CK(hipMalloc(&dL, R * 4));
    CK(hipMemset(dK, 0x3c, ((size_t)1 << 26) * WG + kbytes));
    CK(hipMalloc(&dS, (size_t)WG * m * 4)); CK(hipMalloc(&dZ, (size_t)WG * 8 * QB * 64 * 4));
    std::vector<unsigned short> hQ(R * Dh);
    for (auto& x : hQ) x = f2bf(rnd());
    CK(hipMemcpy(dQ, hQ.data(), hQ.size() * 2, hipMemcpyHostToDevice));
    std::vector<float> negl(R, -12.f);
    CK(hipMemcpy(dL, negl.data(), R * 4, hipMemcpyHostToDevice));
    const size_t lds = R * QS + R * 4 + 8 * QB * 64 * 4 + 32 ;
    unsigned long long* dT; CK(hipMalloc(&dT, WG * 8 * 8));
    hipEvent_t e0, e1; CK(hipEventCreate(&e0)); CK(hipEventCreate(&e1));
    for (int mode = 1; mode <= 2; ++mode)
      for (size_t stride : strides) {
        for (int i = 0; i < 2; ++i)
          hipLaunchKernelGGL(k_pass, dim3(WG), dim3(512), lds, 0, mode, dQ, dL, dK, dK, stride, stride, dS, (size_t)m, dZ, c, m, sc, 0, dT);
        CK(hipEventRecord(e0));
        const int reps = 10;
        for (int i = 0; i < reps; ++i)
          hipLaunchKernelGGL(k_pass, dim3(WG), dim3(512), lds, 0, mode, dQ, dL, dK, dK, stride, stride, dS, (size_t)m, dZ, c, m, sc, 0, dT);
        CK(hipEventRecord(e1)); CK(hipEventSynchronize(e1));
        float ms; CK(hipEventElapsedTime(&ms, e0, e1));
        const double us = ms * 1e3 / reps;
        std::vector<unsigned long long> hT(WG * 8);
        CK(hipMemcpy(hT.data(), dT, WG * 8 * 8, hipMemcpyDeviceToHost));
        double avg = 0, mx = 0;
        for (int i = 0; i < WG * 8; ++i) { auto x = hT[i]; avg += x; if (x > mx) mx = x; }
        avg /= WG * 8;
        { double pw[8] = {0}; for (int i = 0; i < WG * 8; ++i) pw[i % 8] += hT[i]; printf("   per wave index (us):"); for (int w = 0; w < 8; ++w) printf(" %.1f", pw[w] / WG / 100.0); printf("\n"); }
        printf("pass %d, region stride %zu: %.1f us per launch; inside the loop call mean %.1f us, slowest wave %.1f us; %.2f TB/s of keys\n",
               mode, stride, us, avg / 100.0, mx / 100.0, WG * kbytes / us * 1e-6);
        fflush(stdout);
      }
  }
  return 0;
}
