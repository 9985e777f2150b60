// Wave-level building blocks for tiny bias-free MLPs on the fp32 matrix cores of gfx950.
//
// One wavefront (64 lanes) owns a tile of 32 points.  A per-point vector of up to 64
// neurons lives in registers in the layout that v_mfma_f32_32x32x2_f32 produces:
//
//     lane = 32*h + j   (j = point within the tile, h = 0/1)
//     v[b][r], b = block of 32 neurons, r = 0..15  <->  neuron 32*b + 8*(r/4) + 4*h + (r%4)
//
// The instruction computes D(32x32) += A(32x2) * B(2x32) with lane (i,k) holding A[i][k]
// and lane (k,j) holding B[k][j].  Because the order in which the contraction index is
// walked does not matter, register r of a vector in the layout above can be fed back as
// the B operand of step r, with the A operand (the weights, read from LDS) indexed by the
// same neuron number.  Activations therefore never leave registers between layers, in
// forward mode (z = W x), in reverse mode (x = W^T z, using a transposed copy of W) and in
// the forward-mode sweep of the second-order term.
//
// Weight gradients contract over points instead: both factors are written to a per-wave
// LDS tile [point][neuron] and read back with the point as the contraction index.
#pragma once

#include <hip/hip_runtime.h>

namespace neus2 {

typedef float v16f __attribute__((ext_vector_type(16)));

constexpr int kLd64 = 68;   // row stride (floats) of LDS matrices / tiles with 64 columns

__device__ __forceinline__ v16f mfma32(float a, float b, v16f c) {
    return __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, c, 0, 0, 0);
}

__device__ __forceinline__ v16f zero16() {
    v16f z;
#pragma unroll
    for (int r = 0; r < 16; ++r) z[r] = 0.f;
    return z;
}

// neuron (within its block of 32) that register r of lane half h holds
__device__ __forceinline__ constexpr int neuron_of(int r, int h) { return 8 * (r >> 2) + 4 * h + (r & 3); }

// z[mb] = sum_k W[32*mb + j][k] * x[k] for MB blocks of outputs and KB blocks of inputs.
// W is an LDS matrix with row stride LD (multiple of 4 floats).  Only the first RLAST
// registers of the last input block are used (inputs narrower than a multiple of 32).
template <int MB, int KB, int LD, int RLAST = 16>
__device__ __forceinline__ void matvec(const float* __restrict__ W, const v16f* x, v16f* z, int j, int h) {
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) {
        v16f acc = zero16();
#pragma unroll
        for (int kb = 0; kb < KB; ++kb) {
            const int groups = (kb == KB - 1 ? RLAST : 16) / 4;
#pragma unroll
            for (int g = 0; g < groups; ++g) {
                const float4 a = *reinterpret_cast<const float4*>(&W[(32 * mb + j) * LD + 32 * kb + 8 * g + 4 * h]);
                acc = mfma32(a.x, x[kb][4 * g + 0], acc);
                acc = mfma32(a.y, x[kb][4 * g + 1], acc);
                acc = mfma32(a.z, x[kb][4 * g + 2], acc);
                acc = mfma32(a.w, x[kb][4 * g + 3], acc);
            }
        }
        z[mb] = acc;
    }
}

// ReLU in place; returns the mask bits of this lane's 16*NB neurons (bit 16*b + r).
// The mask is 1 only for strictly positive pre-activations (Definition 1 of the paper).
template <int NB>
__device__ __forceinline__ uint32_t relu_mask(v16f* z) {
    uint32_t m = 0;
#pragma unroll
    for (int b = 0; b < NB; ++b)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const bool on = z[b][r] > 0.f;
            m |= (on ? 1u : 0u) << (16 * b + r);
            z[b][r] = on ? z[b][r] : 0.f;
        }
    return m;
}

template <int NB>
__device__ __forceinline__ void apply_mask(v16f* z, uint32_t m) {
#pragma unroll
    for (int b = 0; b < NB; ++b)
#pragma unroll
        for (int r = 0; r < 16; ++r) z[b][r] = ((m >> (16 * b + r)) & 1u) ? z[b][r] : 0.f;
}

// Write a register vector to a per-wave LDS tile [32 points][LD].
template <int NB, int LD>
__device__ __forceinline__ void stage(float* __restrict__ tile, const v16f* v, int j, int h) {
#pragma unroll
    for (int b = 0; b < NB; ++b)
#pragma unroll
        for (int g = 0; g < 4; ++g)
            *reinterpret_cast<float4*>(&tile[j * LD + 32 * b + 8 * g + 4 * h]) =
                make_float4(v[b][4 * g], v[b][4 * g + 1], v[b][4 * g + 2], v[b][4 * g + 3]);
}

// Orders a wave's LDS writes before its following LDS reads by other lanes.
__device__ __forceinline__ void wave_lds_fence() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// G[mb][nb] += sum over the tile's 32 points of Z[point][32*mb + .] (x) X[point][32*nb + .]
// G is in the register layout above with rows = neurons of Z, columns (lane j) = neurons of X.
template <int ZB, int XB, int LDZ, int LDX>
__device__ __forceinline__ void outer_accumulate(v16f (*G)[XB], const float* __restrict__ Zt,
                                                 const float* __restrict__ Xt, int j, int h) {
#pragma unroll
    for (int s = 0; s < 16; ++s) {
        float a[ZB], b[XB];
#pragma unroll
        for (int mb = 0; mb < ZB; ++mb) a[mb] = Zt[(2 * s + h) * LDZ + 32 * mb + j];
#pragma unroll
        for (int nb = 0; nb < XB; ++nb) b[nb] = Xt[(2 * s + h) * LDX + 32 * nb + j];
#pragma unroll
        for (int mb = 0; mb < ZB; ++mb)
#pragma unroll
            for (int nb = 0; nb < XB; ++nb) G[mb][nb] = mfma32(a[mb], b[nb], G[mb][nb]);
    }
}

// Sum one register vector over the block's WAVES waves through a 1024-float LDS scratch;
// the result is valid in the last wave.  Every thread of the block must call it.
template <int WAVES>
__device__ __forceinline__ v16f block_sum(float* __restrict__ scratch, v16f v, int wave, int lane) {
    for (int wv = 0; wv < WAVES; ++wv) {
        if (wave == wv) {
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                float* p = scratch + r * 64 + lane;
                if (wv == 0) *p = v[r];
                else if (wv < WAVES - 1) *p += v[r];
                else v[r] += *p;
            }
        }
        __syncthreads();
    }
    return v;
}

}  // namespace neus2
