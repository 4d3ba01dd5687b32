// Measurement aid: how matrix-core and vector-ALU instructions share a SIMD on this part.
// Each variant runs `iters` iterations of the per-tile instruction mix of the key sweeps
// (Sec. 2 softmax over the window logits: per wave and 64-key tile 16 v_mfma_f32_32x32x16_bf16
// and, for 32 logits per lane, scale-and-subtract, exp2, running maximum, sum) on registers
// only, one workgroup of eight waves per compute unit, as the sweeps run.  The benchmark
// prints the times side by side: matrix work alone, vector work alone, both (the vector work
// depending on the matrix results, as in the sweeps), and both interleaved by hand on
// independent data, and both in barrier intervals of one kind each (matrix or vector), with the
// waves taking the kinds in the same or in opposite order.  They decide what a sweep can reach
// at best: max(a, b) if the two pipes overlap, a + b if they do not.
#include "common.hpp"

namespace caote {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;

template <int VARIANT>
__global__ __launch_bounds__(512) void k_issue_probe(float* out, int iters, float c2) {
  const int lane = threadIdx.x & 63;
  bf16x8 a[8], b[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    uint4 u = make_uint4(0x3c003c00u + lane + i, 0x3c003c00u, 0x3c003c00u, 0x3c003c00u);
    a[i] = __builtin_bit_cast(bf16x8, u);
    u.x += 0x00010003u * (lane + 1); u.y ^= 0x00020001u;
    b[i] = __builtin_bit_cast(bf16x8, u);
  }
  f32x16 acc0, acc1, acc2, acc3;
#pragma unroll
  for (int i = 0; i < 16; ++i) {
    acc0[i] = lane * 0.001f + i; acc1[i] = lane * 0.002f - i;
    acc2[i] = lane * 0.003f + i; acc3[i] = lane * 0.004f - i;
  }
  float l0 = 0.f, l1 = 0.f, m0 = 0.f;
  const f32x16 zero = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
  for (int it = 0; it < iters; ++it) {
    if (VARIANT == 0 || VARIANT == 2) {          // 16 MFMAs (two chains of eight), alone or first
      f32x16 x0 = zero, x1 = zero;
#pragma unroll
      for (int ks = 0; ks < 8; ++ks) {
        x0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[ks], b[ks], x0, 0, 0, 0);
        x1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(b[ks], a[ks], x1, 0, 0, 0);
      }
      if (VARIANT == 0) { l0 += x0[0]; l1 += x1[0]; }
      else { acc0 = x0; acc1 = x1; }
    }
    if (VARIANT == 1 || VARIANT == 2) {          // the vector work of a tile: 32 x (fma, exp2), maxima, sums
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        const f32x16& x = h ? acc1 : acc0;
        float mx = x[0];
#pragma unroll
        for (int i = 1; i < 16; ++i) mx = __builtin_fmaxf(mx, x[i]);
        const float mn = __builtin_fmaxf(m0, mx * c2);
        float e[16];
#pragma unroll
        for (int i = 0; i < 16; ++i) e[i] = __builtin_amdgcn_exp2f(__builtin_fmaf(x[i], c2, -mn));
        const float s = (((e[0] + e[1]) + (e[2] + e[3])) + ((e[4] + e[5]) + (e[6] + e[7]))) +
                        (((e[8] + e[9]) + (e[10] + e[11])) + ((e[12] + e[13]) + (e[14] + e[15])));
        if (h) l1 += s; else l0 += s;
        m0 = mn * 0.5f;
      }
      if (VARIANT == 1) { acc0[0] += 1e-3f; acc1[0] += 1e-3f; }
    }
    if (VARIANT == 3) {                          // 16 x (one MFMA, then 8 independent fma), order pinned
      f32x16 x0 = zero, x1 = zero;
#pragma unroll
      for (int ks = 0; ks < 8; ++ks) {
        x0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[ks], b[ks], x0, 0, 0, 0);
#pragma unroll
        for (int i = 0; i < 8; ++i) acc0[i] = __builtin_fmaf(acc0[i], c2, acc0[i + 8]);
        __builtin_amdgcn_sched_barrier(0);
        x1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(b[ks], a[ks], x1, 0, 0, 0);
#pragma unroll
        for (int i = 0; i < 8; ++i) acc1[i] = __builtin_fmaf(acc1[i], c2, acc1[i + 8]);
        __builtin_amdgcn_sched_barrier(0);
      }
      l0 += x0[0]; l1 += x1[0];
    }
    if (VARIANT >= 5) {
      // Two tiles' worth per iteration (iters is halved by the launcher): every wave issues 32
      // MFMAs (four chains) in one barrier interval and the vector work on their results in
      // the other.  Variant 5: waves 0-3 and waves 4-7 take the two kinds of interval in
      // opposite order, so that in every interval half the waves feed the matrix pipe and half
      // the vector ALUs; variant 7: the same with the waves split by parity (which of the two
      // splits puts one wave of each kind on every SIMD depends on how waves are placed);
      // variant 6: all waves in the same order (the barriers alone).
      const int wave = threadIdx.x >> 6;
      const bool late = VARIANT == 5 ? (wave >> 2) != 0 : VARIANT == 7 ? (wave & 1) != 0 : false;
      auto matrix = [&]() {
        f32x16 x0 = zero, x1 = zero, x2 = zero, x3 = zero;
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) {
          x0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[ks], b[ks], x0, 0, 0, 0);
          x1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(b[ks], a[ks], x1, 0, 0, 0);
          x2 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[ks], a[ks], x2, 0, 0, 0);
          x3 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(b[ks], b[ks], x3, 0, 0, 0);
        }
        acc0 = x0; acc1 = x1; acc2 = x2; acc3 = x3;
      };
      auto vector = [&]() {
#pragma unroll
        for (int h = 0; h < 4; ++h) {
          const f32x16& x = h == 0 ? acc0 : h == 1 ? acc1 : h == 2 ? acc2 : acc3;
          float mx = x[0];
#pragma unroll
          for (int i = 1; i < 16; ++i) mx = __builtin_fmaxf(mx, x[i]);
          const float mn = __builtin_fmaxf(m0, mx * c2);
          float e[16];
#pragma unroll
          for (int i = 0; i < 16; ++i) e[i] = __builtin_amdgcn_exp2f(__builtin_fmaf(x[i], c2, -mn));
          const float s = (((e[0] + e[1]) + (e[2] + e[3])) + ((e[4] + e[5]) + (e[6] + e[7]))) +
                          (((e[8] + e[9]) + (e[10] + e[11])) + ((e[12] + e[13]) + (e[14] + e[15])));
          if (h & 1) l1 += s; else l0 += s;
          m0 = mn * 0.5f;
        }
      };
      __builtin_amdgcn_s_barrier();
      if (late) vector(); else matrix();
      __builtin_amdgcn_s_barrier();
      if (late) matrix(); else vector();
    }
    if (VARIANT == 4) {                          // the 128 fma of variant 3 alone
#pragma unroll
      for (int r = 0; r < 8; ++r) {
#pragma unroll
        for (int i = 0; i < 8; ++i) acc0[i] = __builtin_fmaf(acc0[i], c2, acc0[i + 8]);
#pragma unroll
        for (int i = 0; i < 8; ++i) acc1[i] = __builtin_fmaf(acc1[i], c2, acc1[i + 8]);
      }
    }
  }
  out[blockIdx.x * blockDim.x + threadIdx.x] = l0 + l1 + m0 + acc0[3] + acc1[5] + (VARIANT >= 5 ? acc2[7] + acc3[9] : 0.f);
}

}  // namespace

// 256 workgroups of 512 threads; `out` holds 256 * 512 floats.
hipError_t launch_issue_probe(int variant, int iters, float* out, hipStream_t s) {
  const dim3 grid(256), block(512);
  switch (variant) {
    case 0: hipLaunchKernelGGL(k_issue_probe<0>, grid, block, 0, s, out, iters, 0.127f); break;
    case 1: hipLaunchKernelGGL(k_issue_probe<1>, grid, block, 0, s, out, iters, 0.127f); break;
    case 2: hipLaunchKernelGGL(k_issue_probe<2>, grid, block, 0, s, out, iters, 0.127f); break;
    case 3: hipLaunchKernelGGL(k_issue_probe<3>, grid, block, 0, s, out, iters, 0.127f); break;
    case 4: hipLaunchKernelGGL(k_issue_probe<4>, grid, block, 0, s, out, iters, 0.127f); break;
    case 5: hipLaunchKernelGGL(k_issue_probe<5>, grid, block, 0, s, out, (iters + 1) / 2, 0.127f); break;
    case 6: hipLaunchKernelGGL(k_issue_probe<6>, grid, block, 0, s, out, (iters + 1) / 2, 0.127f); break;
    case 7: hipLaunchKernelGGL(k_issue_probe<7>, grid, block, 0, s, out, (iters + 1) / 2, 0.127f); break;
    default: return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

}  // namespace caote
