// Tuning hook of a -DPF_TUNING build (tile, ring-depth and split sweeps on the GPU).  The shipped library is built
// without PF_TUNING: there the plan constants of ops.h are compile-time constants and this hook does not exist.
#pragma once
#ifdef PF_TUNING
extern "C" {
// 0..99: pins one GEMM tile configuration for every following launch (0 = heuristic); 100 + v: attention kernel generation;
// 200 / 201: fused K/V routing of the QKV projection off / on; 300 + s: attention ring depth; 400 + k: smallest K (units of
// 64) and 500 + t: largest tile count (units of 16 tiles of 64 x 64) for the wave-split-K GEMM; 600 + s: key-split count of
// the stage's attention launches (600 = heuristic); 700 / 701 / 702: 256-query attention workgroups by launch size /
// never / always; 800 / 801: folding of the softmax exponent factor into q off / on.
void pf_tune(int id);
// Shader-clock stamps of the 8-wave attention kernel's last launch: out[wave][step * 6 + k] for the four tile steps of
// one outer loop iteration of workgroup 0, k = 0 step entered, 1 behind the barrier, 2 .. 4 phase boundaries.
int pf_attn_trace_read(unsigned long long *out);
}
#endif
