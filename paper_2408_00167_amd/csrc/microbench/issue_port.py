"""Writes issue_port.hip: how the matrix instructions of one 32 keys x 32 prompt rows x 128
logit tile and the vector work on such a tile (per accumulator value: one fused
multiply-add, one exp2, one add - what the scoring passes do) share a SIMD of gfx950.

Every kernel is one inline-asm loop over registers only (no memory, no LDS), so the
numbers are the issue limits of the SIMD itself.  Variants: the tile as 8 instructions
32x32x16 or as 16 instructions 16x16x32; matrix work alone, vector work alone (all of it,
only the exp2, only the plain operations, without the multiply-add), and both
interleaved; with one and with two waves per SIMD.

  python issue_port.py && hipcc --offload-arch=gfx950 -O3 -o issue_port issue_port.hip && ./issue_port
"""
import os

U0, T0, NEGL = 80, 96, 112      # column sums, temporaries, the per-row constant


def vector_work(srcs, fma=True, exp=True, add=True):
    """the three operations per accumulator value, software-pipelined by one value each"""
    ops, n = [], len(srcs)
    for g in range(n + 2):
        if g < n and fma:
            ops.append(f"v_fma_f32 v{T0 + g % 8}, v{srcs[g]}, s4, v{NEGL}")
        if 1 <= g <= n and exp:
            src = T0 + (g - 1) % 8 if fma else srcs[g - 1]
            ops.append(f"v_exp_f32 v{T0 + (g - 1) % 8}, v{src}")
        if g >= 2 and add:
            ops.append(f"v_add_f32 v{U0 + (g - 2) % 16}, v{U0 + (g - 2) % 16}, v{T0 + (g - 2) % 8}")
    return ops


def interleave(m, v):
    if not v:
        return m
    if not m:
        return v
    per, done, out = len(v) / len(m), 0, []
    for s, x in enumerate(m):
        out.append(x)
        upto = round(per * (s + 1))
        out += v[done:upto]
        done = upto
    return out


def tile32(acc):
    return [f"v_mfma_f32_32x32x16_bf16 v[{acc}:{acc + 15}], v[64:67], v[68:71], "
            f"{'0' if s == 0 else f'v[{acc}:{acc + 15}]'}" for s in range(8)]


def tile16(acc):
    out = []
    for s in range(4):
        for sub in range(4):
            a = acc + 4 * sub
            out.append(f"v_mfma_f32_16x16x32_bf16 v[{a}:{a + 3}], v[64:67], v[68:71], "
                       f"{'0' if s == 0 else f'v[{a}:{a + 3}]'}")
    return out


def two_tiles(kind, matrix=True, **vec):
    """one loop iteration: the matrix instructions of two tiles (accumulators v0-15, v16-31),
    the vector work on the two tiles before them (v32-63)"""
    m = []
    if matrix:
        mk = tile32 if kind == 32 else tile16
        for x, y in zip(mk(0), mk(16)):
            m += [x, y]
    v = vector_work(list(range(32, 64)), **vec) if vec is not None and vec.get("on", True) else []
    return interleave(m, v)


def vec(**kw):
    d = dict(fma=True, exp=True, add=True)
    d.update(kw)
    return d


VARIANTS = [
    ("matrix 32x32x16 alone", interleave(two_tiles(32, True, on=False), [])),
    ("matrix 16x16x32 alone", interleave(two_tiles(16, True, on=False), [])),
    ("vector alone (fma, exp2, add)", interleave([], vector_work(list(range(32, 64))))),
    ("vector alone: exp2 only", vector_work(list(range(32, 64)), fma=False, add=False)),
    ("vector alone: fma and add only", vector_work(list(range(32, 64)), exp=False)),
    ("vector alone: exp2 and add, no fma", vector_work(list(range(32, 64)), fma=False)),
    ("32x32x16 + vector", interleave(two_tiles(32, True, on=False), vector_work(list(range(32, 64))))),
    ("16x16x32 + vector", interleave(two_tiles(16, True, on=False), vector_work(list(range(32, 64))))),
    ("32x32x16 + exp2 only", interleave(two_tiles(32, True, on=False), vector_work(list(range(32, 64)), fma=False, add=False))),
    ("32x32x16 + fma and add only", interleave(two_tiles(32, True, on=False), vector_work(list(range(32, 64)), exp=False))),
    ("32x32x16 + exp2 and add, no fma", interleave(two_tiles(32, True, on=False), vector_work(list(range(32, 64)), fma=False))),
]


def main():
    clob = ",".join(f'"v{i}"' for i in range(120)) + ', "s4", "s5", "s6", "scc", "vcc", "memory"'
    init = ('"v_mbcnt_lo_u32_b32 v119, -1, 0\\n\\t" "v_mbcnt_hi_u32_b32 v119, -1, v119\\n\\t" "v_cvt_f32_u32 v118, v119\\n\\t"'
            ' "v_mul_f32 v118, 0x3c23d70a, v118\\n\\t" "s_mov_b32 s4, 0x3e028f5c\\n\\t" "v_mov_b32 v112, 0xc0400000\\n\\t"\n' +
            "".join(f'    "v_add_f32 v{i}, {float(i % 7) * 0.25 + 0.5}, v118\\n\\t"\n' for i in range(64)) +
            "".join(f'    "v_mov_b32 v{i}, 0x3f803f80\\n\\t" "v_xor_b32 v{i}, v{i}, v119\\n\\t"\n' for i in range(64, 76)) +
            "".join(f'    "v_mov_b32 v{i}, 0\\n\\t"\n' for i in range(76, 112)))
    out = ["// written by issue_port.py - do not edit\n#include <hip/hip_runtime.h>\n#include <cstdio>\n"
           f"#define CLOB {clob}\n"
           "__device__ unsigned long long clk[2];\n"]
    for vi, (name, body) in enumerate(VARIANTS):
        asm = "\\n\\t".join(body)
        out.append(f'''
__global__ __launch_bounds__(256) void k{vi}(float* out, int iters, float seed) {{
  float r = 0.f;
  const unsigned long long c0 = clock64(), w0 = wall_clock64();
  asm volatile({init}
    "s_mov_b32 s5, %1\\n\\t"
    "1:\\n\\t"
    "{asm}\\n\\t"
    "s_sub_u32 s5, s5, 1\\n\\t" "s_cmp_lg_u32 s5, 0\\n\\t" "s_cbranch_scc1 1b\\n\\t"
    "s_nop 7\\n\\t s_nop 7\\n\\t s_nop 7\\n\\t"
    "v_add_f32 %0, v{U0}, v0\\n\\t" "v_add_f32 %0, %0, v16\\n\\t"
    : "=v"(r) : "s"(iters) : CLOB);
  if (blockIdx.x == 0 && threadIdx.x == 0) {{ clk[0] = clock64() - c0; clk[1] = wall_clock64() - w0; }}
  out[blockIdx.x * 256 + threadIdx.x] = r + seed;
}}
''')
    names = ", ".join(f'{{"{n}", k{i}}}' for i, (n, _) in enumerate(VARIANTS))
    out.append('''
typedef void (*kern_t)(float*, int, float);
struct Variant { const char* name; kern_t k; };
int main() {
  Variant vs[] = {''' + names + '''};
  const int nv = sizeof(vs) / sizeof(vs[0]);
  float* out;
  if (hipMalloc(&out, 256 * 16 * 256 * 4) != hipSuccess) return 1;
  const int iters = 6000;
  hipEvent_t e0, e1; (void)hipEventCreate(&e0); (void)hipEventCreate(&e1);
  // 256 workgroups of 4 waves = one wave per SIMD of the chip; 512 workgroups = two
  for (int w : {1, 2})
    for (int v = 0; v < nv; ++v) {
      hipLaunchKernelGGL(vs[v].k, dim3(256 * w), dim3(256), 0, 0, out, 200, 0.f);
      (void)hipEventRecord(e0);
      for (int i = 0; i < 3; ++i) hipLaunchKernelGGL(vs[v].k, dim3(256 * w), dim3(256), 0, 0, out, iters, 0.f);
      (void)hipEventRecord(e1); (void)hipEventSynchronize(e1);
      float ms; (void)hipEventElapsedTime(&ms, e0, e1); ms /= 3;
      unsigned long long c[2]; (void)hipMemcpyFromSymbol(c, HIP_SYMBOL(clk), sizeof(c));
      const double ghz = (double)c[0] / ((double)c[1] * 10.0);   // wall clock ticks of 10 ns
      const double ns = ms * 1e6 / (2.0 * iters * w);
      printf("%-36s %d wave(s) per SIMD: %7.1f ns = %5.0f clocks per tile per SIMD (%.2f GHz)\\n", vs[v].name, w, ns, ns * ghz, ghz);
      fflush(stdout);
    }
  return hipGetLastError() == hipSuccess ? 0 : 1;
}
''')
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "issue_port.hip")
    open(path, "w").write("".join(out))
    print("wrote", path)


if __name__ == "__main__":
    main()
