#!/usr/bin/env python3
"""Instruction-issue probe for the scan's inner loop on gfx950.

Writes issue_patterns.hip: one kernel per way of interleaving the eight (or nine) dependent
v_mfma_f32_32x32x16_bf16 of one 32x32 logit tile with the vector work on the previous tile (per logit one
FMA or multiply, one v_exp_f32, one add; plus the maximum tracking of the first pass), each written as a
single asm block so that the order is exactly as given; one wave per SIMD, operands in registers, no
memory traffic. Prints shader cycles per tile for every pattern: the cost of a (key tile, query tile) pair
if nothing but these instructions were issued.
Build and run: python -m paper_2602_08686_amd.build probes && paper_2602_08686_amd/probes/issue_patterns"""
import itertools
pats = {}
def triples(n_logits, first=0):
    # returns list of VALU instructions for logits first..first+n-1 : fma, exp, add (software-ordered: fma block, exp block, add block per group of 2)
    out = []
    for r in range(first, first + n_logits, 2):
        for q in (r, r + 1): out.append(('fma', q))
        for q in (r, r + 1): out.append(('exp', q))
        for q in (r, r + 1): out.append(('add', q))
    return out
def emit(seq):
    # seq: list of 'M' or ('fma'|'exp'|'add'|'mul'|'max', r)
    lines = []
    for it in seq:
        if it == 'M':
            lines.append('v_mfma_f32_32x32x16_bf16 %[n], %[a], %[b], %[n]')
        else:
            op, r = it
            if op == 'fma': lines.append(f'v_fma_f32 %[t{r%4}], %[c][{r}], %[sc], %[ref]'.replace('%[c]['+str(r)+']', f'%[c{r}]'))
            elif op == 'mul': lines.append(f'v_mul_f32 %[t{r%4}], %[c{r}], %[sc]')
            elif op == 'exp': lines.append(f'v_exp_f32 %[t{r%4}], %[t{r%4}]')
            elif op == 'add': lines.append(f'v_add_f32 %[s{r%4}], %[s{r%4}], %[t{r%4}]')
            elif op == 'max': lines.append(f'v_max3_f32 %[s{r%4}], %[c{r}], %[c{(r+1)%16}], %[s{r%4}]')
    return lines
V51 = triples(16) + [('max', 0), ('max', 4), ('max', 8)]
V66 = triples(16) + [('max', i) for i in range(0, 16, 2)] + [('max', i) for i in range(0, 14, 2)]
V52m = [x if x[0] != 'fma' else ('mul', x[1]) for x in triples(16)] + [('add', 0), ('add', 1), ('add', 2), ('add', 3)]
def spread(V, per, n_m=8, tailfirst=False):
    seq = []; v = list(V)
    for k in range(n_m):
        seq.append('M'); seq += v[:per]; v = v[per:]
    return seq + v
pats['a_51_M6'] = spread(V51, 6)
pats['b_51_M7'] = spread(V51, 7)
pats['c_51_M5'] = spread(V51, 5)
pats['d_51_M4'] = spread(V51, 4)
pats['e_51_M3'] = spread(V51, 3)
pats['f_51_Mfirst'] = ['M'] * 8 + V51
pats['g_51_MM12'] = sum([['M', 'M'] + V51[12*k:12*k+12] for k in range(4)], []) + V51[48:]
pats['h_66_M8'] = spread(V66, 8)
pats['i_66_M6'] = spread(V66, 6)
pats['j_52mul_M9x5'] = spread(V52m, 5, 9)
pats['k_52mul_M9x6'] = spread(V52m, 6, 9)
pats['l_52mul_M9x4'] = spread(V52m, 4, 9)
pats['m_valu51_only'] = list(V51)
pats['n_mfma8_only'] = ['M'] * 8
# exps first within group vs interleaved
def grouped(n_m, per_group):
    # per MFMA: 2 fma, 2 exp(prev), 2 add(prev-prev) software pipelined -> no back-to-back dependency
    f = [('fma', r) for r in range(16)]; e = [('exp', r) for r in range(16)]; a = [('add', r) for r in range(16)]
    seq = []
    for k in range(8):
        seq.append('M'); seq += f[2*k:2*k+2] + e[2*k:2*k+2] + a[2*k:2*k+2]
    return seq
pats['o_48_M6'] = grouped(8, 6)
src = ['#include <hip/hip_runtime.h>', '#include <cstdio>', 'typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;', 'typedef __attribute__((ext_vector_type(16))) float f32x16;']
for name, seq in pats.items():
    body = '\\n\\t'.join(emit(seq))
    cregs = ', '.join(f'[c{r}] "v"(c[{r}])' for r in range(16))
    src.append(f'''
__global__ void __launch_bounds__(256) k_{name}(const bf16x8* in, float* out, int iters, long long* cyc) {{
  bf16x8 a = in[threadIdx.x], b = in[threadIdx.x + 256];
  f32x16 n, c;
  for (int r = 0; r < 16; ++r) {{ n[r] = 0.f; c[r] = threadIdx.x * 1e-3f + r; }}
  float t0 = 0, t1 = 0, t2 = 0, t3 = 0, s0 = 0, s1 = 0, s2 = 0, s3 = 0;
  const float c2 = out[0] + 0.127f, ref = out[1] + 3.0f;
  long long q0 = clock64();
  for (int it = 0; it < iters; ++it) {{
    asm volatile("{body}"
      : [n] "+v"(n), [t0] "+v"(t0), [t1] "+v"(t1), [t2] "+v"(t2), [t3] "+v"(t3), [s0] "+v"(s0), [s1] "+v"(s1), [s2] "+v"(s2), [s3] "+v"(s3)
      : [a] "v"(a), [b] "v"(b), [sc] "v"(c2), [ref] "v"(ref), {cregs});
  }}
  long long q1 = clock64();
  float tot = s0 + s1 + s2 + s3 + t0 + t1 + t2 + t3;
  for (int r = 0; r < 16; ++r) tot += n[r];
  out[2 + blockIdx.x * 256 + threadIdx.x] = tot;
  if (blockIdx.x == 0 && threadIdx.x == 0) cyc[0] = q1 - q0;
}}''')
src.append('int main() { bf16x8* in; float* out; long long* cyc; long long h; hipMalloc(&in, 512 * 16); hipMemset(in, 0, 512 * 16); hipMalloc(&out, 4 * (2 + 256 * 256)); hipMemset(out, 0, 8); hipMalloc(&cyc, 16); const int iters = 2000;')
for name, seq in pats.items():
    nm = seq.count('M'); nv = len(seq) - nm
    src.append(f'  for (int rep = 0; rep < 2; ++rep) hipLaunchKernelGGL(k_{name}, dim3(256), dim3(256), 0, 0, in, out, iters, cyc); hipDeviceSynchronize(); hipMemcpy(&h, cyc, 8, hipMemcpyDeviceToHost); printf("%-16s mfma {nm} valu {nv}: %7.1f cycles/iter\\n", "{name}", (double)h / iters);')
src.append('  return 0; }')
open(__import__('os').path.join(__import__('os').path.dirname(__import__('os').path.abspath(__file__)), 'issue_patterns.hip'), 'w').write('\n'.join(src))
