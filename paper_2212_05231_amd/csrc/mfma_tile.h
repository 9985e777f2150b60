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
    // The weights of the next group of four steps are requested from LDS before the four
    // MFMAs of the current group are issued, and the scheduler is told not to move anything
    // across group boundaries: left alone it hoists every LDS read of the kernel to the top
    // and needs more than 256 registers for what is a 130-register computation.
    constexpr int kGroupsLast = RLAST / 4;
    constexpr int kGroupsPerMb = (KB - 1) * 4 + kGroupsLast;
    constexpr int kTotal = MB * kGroupsPerMb;
    const float* base = W + j * LD + 4 * h;
    auto address = [&](int t) -> const float4* {
        const int mb = t / kGroupsPerMb, u = t % kGroupsPerMb;
        const int kb = u / 4, g = u % 4;
        return reinterpret_cast<const float4*>(base + 32 * mb * LD + 32 * kb + 8 * g);
    };
    float4 cur = *address(0);
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) {
        v16f acc = zero16();
#pragma unroll
        for (int u = 0; u < kGroupsPerMb; ++u) {
            const int t = mb * kGroupsPerMb + u;
            const int kb = u / 4, g = u % 4;
            float4 nxt = cur;
            if (t + 1 < kTotal) nxt = *address(t + 1);
            acc = mfma32(cur.x, x[kb][4 * g + 0], acc);
            acc = mfma32(cur.y, x[kb][4 * g + 1], acc);
            acc = mfma32(cur.z, x[kb][4 * g + 2], acc);
            acc = mfma32(cur.w, x[kb][4 * g + 3], acc);
            cur = nxt;
            __builtin_amdgcn_sched_barrier(0);
        }
        z[mb] = acc;
    }
}

// ReLU in place; returns the mask bits of this lane's 16*NB neurons (bit 16*b + r).
// The mask is 1 only for strictly positive pre-activations (Definition 1 of the paper).
// Neither direction uses a compare instruction: the result of a compare is a lane mask in a
// scalar register pair, 32 of them per mask word, which the compiler parks in vector-register
// lanes and fetches back for every use.  A float is positive exactly when its bit pattern is a
// positive integer, so the ReLU is an integer maximum with 0 on the pattern, the mask bit the
// unsigned minimum of the result with 1, and a one-bit sign-extending field extract turns a mask
// bit back into an all-ones or all-zeros word to AND with.  The instructions are written out
// because the compiler rewrites the equivalent C expressions into compares and selects.
template <int NB>
__device__ __forceinline__ uint32_t relu_mask(v16f* z) {
    uint32_t m = 0;
#pragma unroll
    for (int b = 0; b < NB; ++b)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            float zf = z[b][r];
            uint32_t on;
            asm("v_max_i32 %0, 0, %0" : "+v"(zf));
            asm("v_min_u32 %0, 1, %1" : "=v"(on) : "v"(zf));
            asm("v_lshl_or_b32 %0, %1, %2, %0" : "+v"(m) : "v"(on), "n"(16 * b + r));
            z[b][r] = zf;
        }
    return m;
}

template <int NB>
__device__ __forceinline__ void apply_mask(v16f* z, uint32_t m) {
#pragma unroll
    for (int b = 0; b < NB; ++b)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            float zf = z[b][r];
            uint32_t keep;
            asm("v_bfe_i32 %0, %1, %2, 1" : "=v"(keep) : "v"(m), "n"(16 * b + r));
            asm("v_and_b32 %0, %0, %1" : "+v"(zf) : "v"(keep));
            z[b][r] = zf;
        }
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
    // operands of step s+1 are read from LDS before the MFMAs of step s are issued
    float a[ZB], b[XB], an[ZB], bn[XB];
#pragma unroll
    for (int mb = 0; mb < ZB; ++mb) a[mb] = Zt[h * LDZ + 32 * mb + j];
#pragma unroll
    for (int nb = 0; nb < XB; ++nb) b[nb] = Xt[h * LDX + 32 * nb + j];
#pragma unroll
    for (int s = 0; s < 16; ++s) {
        if (s + 1 < 16) {
#pragma unroll
            for (int mb = 0; mb < ZB; ++mb) an[mb] = Zt[(2 * s + 2 + h) * LDZ + 32 * mb + j];
#pragma unroll
            for (int nb = 0; nb < XB; ++nb) bn[nb] = Xt[(2 * s + 2 + h) * LDX + 32 * nb + j];
        }
#pragma unroll
        for (int mb = 0; mb < ZB; ++mb)
#pragma unroll
            for (int nb = 0; nb < XB; ++nb) G[mb][nb] = mfma32(a[mb], b[nb], G[mb][nb]);
#pragma unroll
        for (int mb = 0; mb < ZB; ++mb) a[mb] = an[mb];
#pragma unroll
        for (int nb = 0; nb < XB; ++nb) b[nb] = bn[nb];
        __builtin_amdgcn_sched_barrier(0);
    }
}

// ---- weight gradients on the bf16 matrix cores --------------------------------------------
// A weight gradient is a sum over all points of products of two per-point numbers; it is
// compared with a reference at gradient tolerance, not at forward tolerance, and its rounding
// errors average out over the sum.  Both factors are therefore split into two bf16 numbers,
// x = hi + mid (round to nearest even each time, |x - hi - mid| <= 2^-16 |x|), and the product
// is taken as hi*hi + hi*mid + mid*hi on v_mfma_f32_32x32x16_bf16, which contracts 16 points
// per instruction in half the time the fp32 instruction takes for 2: 12 instructions of 32
// clocks for a 32x32 block over a tile's 32 points, instead of 16 of 64 clocks.
//   D(32x32) += A(32x16) B(16x32); lane l holds A[l%32][8*(l/32) + s] and B[8*(l/32) + s][l%32],
//   s = 0..7, and D in the register layout at the top of this file (checked on the chip).
// The contraction index (the point) must run along a lane's eight operand slots, so the tile
// is kept transposed, [neuron][point], one 32-bit word [hi | mid] per element, row stride
// kLdT words: a lane reads its eight points as two 16-byte words, conflict-free.
typedef __bf16 bf8 __attribute__((ext_vector_type(8)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int kLdT = 36;    // row stride (words) of a transposed split tile [64 neurons][32 points]
constexpr int kTileWords = 64 * kLdT;   // a per-wave tile holds either layout: [32 points][kLd64] floats or this

__device__ __forceinline__ uint32_t split_bf16(float x) {
    const __bf16 hi = (__bf16)x;
    const __bf16 mid = (__bf16)(x - (float)hi);
    return ((uint32_t)__builtin_bit_cast(uint16_t, hi) << 16) | (uint32_t)__builtin_bit_cast(uint16_t, mid);
}

// Write a register vector to a per-wave transposed split tile.
template <int NB>
__device__ __forceinline__ void stage_split(uint32_t* __restrict__ tile, const v16f* v, int j, int h) {
#pragma unroll
    for (int b = 0; b < NB; ++b)
#pragma unroll
        for (int r = 0; r < 16; ++r) tile[(32 * b + neuron_of(r, h)) * kLdT + j] = split_bf16(v[b][r]);
}

// Eight [hi | mid] words -> the eight hi halves and the eight mid halves as MFMA operands.
__device__ __forceinline__ void unpack_split(const u32x4& p, const u32x4& q, bf8& hi, bf8& mid) {
    u32x4 vh, vm;
    vh[0] = __builtin_amdgcn_perm(p[1], p[0], 0x07060302u);
    vh[1] = __builtin_amdgcn_perm(p[3], p[2], 0x07060302u);
    vh[2] = __builtin_amdgcn_perm(q[1], q[0], 0x07060302u);
    vh[3] = __builtin_amdgcn_perm(q[3], q[2], 0x07060302u);
    vm[0] = __builtin_amdgcn_perm(p[1], p[0], 0x05040100u);
    vm[1] = __builtin_amdgcn_perm(p[3], p[2], 0x05040100u);
    vm[2] = __builtin_amdgcn_perm(q[1], q[0], 0x05040100u);
    vm[3] = __builtin_amdgcn_perm(q[3], q[2], 0x05040100u);
    hi = __builtin_bit_cast(bf8, vh);
    mid = __builtin_bit_cast(bf8, vm);
}

// G[mb][nb] += sum over the tile's 32 points of Z[32*mb + .][point] (x) X[32*nb + .][point], both
// tiles transposed and split as above; G as in outer_accumulate.
template <int ZB, int XB>
__device__ __forceinline__ void outer_accumulate_split(v16f (*G)[XB], const uint32_t* __restrict__ Zt,
                                                       const uint32_t* __restrict__ Xt, int lane) {
    const int i = lane & 31, g = lane >> 5;
#pragma unroll
    for (int t = 0; t < 2; ++t) {
        bf8 bh[XB], bm[XB];
#pragma unroll
        for (int nb = 0; nb < XB; ++nb) {
            const u32x4* src = reinterpret_cast<const u32x4*>(Xt + (32 * nb + i) * kLdT + 16 * t + 8 * g);
            unpack_split(src[0], src[1], bh[nb], bm[nb]);
        }
#pragma unroll
        for (int mb = 0; mb < ZB; ++mb) {
            const u32x4* src = reinterpret_cast<const u32x4*>(Zt + (32 * mb + i) * kLdT + 16 * t + 8 * g);
            bf8 ah, am;
            unpack_split(src[0], src[1], ah, am);
#pragma unroll
            for (int nb = 0; nb < XB; ++nb) {
                G[mb][nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ah, bh[nb], G[mb][nb], 0, 0, 0);
                G[mb][nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ah, bm[nb], G[mb][nb], 0, 0, 0);
                G[mb][nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(am, bh[nb], G[mb][nb], 0, 0, 0);
            }
        }
        __builtin_amdgcn_sched_barrier(0);
    }
}

// ---- matrix-vector products on the bf16 matrix cores ---------------------------------------
// The same splitting carries the products W x of the backward kernels.  With two terms per
// factor and three products the relative error of a product is about 2^-16, which is enough
// for quantities that are compared at gradient tolerance (the adjoint sweeps).  With three
// terms, x = hi + mid + lo (|x - hi - mid - lo| <= 2^-24 |x|), and the six products hi*hi,
// hi*mid, mid*hi, mid*mid, hi*lo, lo*hi the result is as accurate as an fp32 product: that is
// used where a ReLU mask is decided from the result (the recomputed forward pass), in 6/16 of
// the matrix-pipe time of the fp32 instruction.
//
// Register side: a vector in the layout at the top of this file is turned into one word
// [hi | mid] per element (and, for three terms, one word per two elements holding both lo
// parts).  Registers 8q..8q+7 of input block kb are the eight operand slots of k-step
// u = 2 kb + q, so slot s of lane half g stands for input 32 kb + 16 q + 8 (s/4) + 4 g + s%4.
// LDS side: a matrix is stored per output row as [k-step][lane half][plane][8 bf16], the slots in
// the order just given, so that a lane reads each plane of its operand as one 16-byte word;
// the row stride leaves 16 bytes of padding, which makes those reads conflict-free.
template <int KSTEPS, int PS>
struct SplitMatrix {
    static constexpr int kLd = KSTEPS * 2 * PS * 16 + 16;     // bytes per output row
    // byte offset of plane 0 of (output row o, input c)
    __device__ static __forceinline__ int offset(int o, int c) {
        const int u = c >> 4, rem = c & 15;
        const int g = (rem >> 2) & 1, s = ((rem >> 3) << 2) | (rem & 3);
        return o * kLd + (2 * u + g) * (PS * 16) + 2 * s;
    }
    // store one weight, split into PS bf16 terms
    __device__ static __forceinline__ void store(unsigned char* __restrict__ W, int o, int c, float v) {
        unsigned char* dst = W + offset(o, c);
#pragma unroll
        for (int p = 0; p < PS; ++p) {
            const __bf16 t = (__bf16)v;
            *reinterpret_cast<__bf16*>(dst + 16 * p) = t;
            v -= (float)t;
        }
    }
};

// v -> words [hi | mid]
template <int NB>
__device__ __forceinline__ void split2(const v16f* v, uint32_t (*w)[16]) {
#pragma unroll
    for (int b = 0; b < NB; ++b)
#pragma unroll
        for (int r = 0; r < 16; ++r) w[b][r] = split_bf16(v[b][r]);
}

// v -> words [hi | mid] and, per two elements, one word [lo(2p+1) | lo(2p)]
template <int NB>
__device__ __forceinline__ void split3(const v16f* v, uint32_t (*w)[16], uint32_t (*l)[8]) {
#pragma unroll
    for (int b = 0; b < NB; ++b)
#pragma unroll
        for (int p = 0; p < 8; ++p) {
            uint16_t lo[2];
#pragma unroll
            for (int e = 0; e < 2; ++e) {
                const float x = v[b][2 * p + e];
                const __bf16 hi = (__bf16)x;
                const float r1 = x - (float)hi;
                const __bf16 mid = (__bf16)r1;
                const __bf16 lw = (__bf16)(r1 - (float)mid);
                w[b][2 * p + e] = ((uint32_t)__builtin_bit_cast(uint16_t, hi) << 16) | (uint32_t)__builtin_bit_cast(uint16_t, mid);
                lo[e] = __builtin_bit_cast(uint16_t, lw);
            }
            l[b][p] = ((uint32_t)lo[1] << 16) | (uint32_t)lo[0];
        }
}

// Write words [hi | mid] to a per-wave transposed split tile.
template <int NB>
__device__ __forceinline__ void stage_words(uint32_t* __restrict__ tile, const uint32_t (*w)[16], int j, int h) {
#pragma unroll
    for (int b = 0; b < NB; ++b)
#pragma unroll
        for (int r = 0; r < 16; ++r) tile[(32 * b + neuron_of(r, h)) * kLdT + j] = w[b][r];
}

// The three terms of a vector, each packed two elements to a word ([term(2p+1) | term(2p)]):
// words 4q..4q+3 of block kb are the operand of k-step 2 kb + q as they stand.  This is the
// cheapest form to produce (one conversion instruction yields a word) and is used where a vector
// only feeds matrix-vector products; vectors that also go into a weight gradient use the
// per-element words above.
template <int NB>
struct SplitPairs {
    uint32_t h[NB][8], m[NB][8], l[NB][8];
};

template <int NB>
__device__ __forceinline__ void split3_pairs(const v16f* v, SplitPairs<NB>& out) {
    typedef __bf16 bf2 __attribute__((ext_vector_type(2)));
    typedef float f2 __attribute__((ext_vector_type(2)));
#pragma unroll
    for (int b = 0; b < NB; ++b)
#pragma unroll
        for (int p = 0; p < 8; ++p) {
            const float x0 = v[b][2 * p], x1 = v[b][2 * p + 1];
            const uint32_t hp = __builtin_bit_cast(uint32_t, __builtin_convertvector(f2{x0, x1}, bf2));
            const float r0 = x0 - __builtin_bit_cast(float, hp << 16);
            const float r1 = x1 - __builtin_bit_cast(float, hp & 0xffff0000u);
            const uint32_t mp = __builtin_bit_cast(uint32_t, __builtin_convertvector(f2{r0, r1}, bf2));
            const float q0 = r0 - __builtin_bit_cast(float, mp << 16);
            const float q1 = r1 - __builtin_bit_cast(float, mp & 0xffff0000u);
            out.h[b][p] = hp;
            out.m[b][p] = mp;
            out.l[b][p] = __builtin_bit_cast(uint32_t, __builtin_convertvector(f2{q0, q1}, bf2));
        }
}

// z[mb] = sum_c W[32 mb + .][c] x[c] for MB blocks of outputs and KSTEPS * 16 inputs; W is a
// SplitMatrix<KSTEPS, PS>; `operand(u, bh, bm, bl)` hands over the terms of x for k-step u
// (P = 2: three products, P = 3: six; P <= PS).
template <int MB, int KSTEPS, int PS, int P, typename Operand>
__device__ __forceinline__ void matvec_split_core(const unsigned char* __restrict__ W, Operand operand, v16f* z, int lane) {
    static_assert(P == 2 || P == 3, "two or three terms");
    static_assert(P <= PS, "the matrix holds fewer terms than asked for");
    constexpr int kLd = SplitMatrix<KSTEPS, PS>::kLd;
    constexpr int kTotal = KSTEPS * MB;
    const int i = lane & 31, g = lane >> 5;
    const unsigned char* base = W + i * kLd + g * (PS * 16);
    auto address = [&](int t) -> const u32x4* {
        const int u = t / MB, mb = t % MB;
        return reinterpret_cast<const u32x4*>(base + 32 * mb * kLd + u * (2 * PS * 16));
    };
    u32x4 cur[P], nxt[P];
#pragma unroll
    for (int p = 0; p < P; ++p) cur[p] = address(0)[p];
    v16f acc[MB];
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) acc[mb] = zero16();
#pragma unroll
    for (int u = 0; u < KSTEPS; ++u) {
        bf8 bh, bm, bl;
        operand(u, bh, bm, bl);
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) {
            const int t = u * MB + mb;
#pragma unroll
            for (int p = 0; p < P; ++p) nxt[p] = cur[p];
            if (t + 1 < kTotal) {
#pragma unroll
                for (int p = 0; p < P; ++p) nxt[p] = address(t + 1)[p];
            }
            const bf8 ah = __builtin_bit_cast(bf8, cur[0]), am = __builtin_bit_cast(bf8, cur[1]);
            acc[mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ah, bh, acc[mb], 0, 0, 0);
            acc[mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ah, bm, acc[mb], 0, 0, 0);
            acc[mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(am, bh, acc[mb], 0, 0, 0);
            if (P == 3) {
                const bf8 al = __builtin_bit_cast(bf8, cur[P - 1]);
                acc[mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(am, bm, acc[mb], 0, 0, 0);
                acc[mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ah, bl, acc[mb], 0, 0, 0);
                acc[mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(al, bh, acc[mb], 0, 0, 0);
            }
#pragma unroll
            for (int p = 0; p < P; ++p) cur[p] = nxt[p];
            __builtin_amdgcn_sched_barrier(0);
        }
    }
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) z[mb] = acc[mb];
}

// x as the per-element words of split2 / split3
template <int MB, int KSTEPS, int PS, int P>
__device__ __forceinline__ void matvec_split(const unsigned char* __restrict__ W, const uint32_t (*wx)[16],
                                             const uint32_t (*lx)[8], v16f* z, int lane) {
    matvec_split_core<MB, KSTEPS, PS, P>(W, [&](int u, bf8& bh, bf8& bm, bf8& bl) {
        const uint32_t* s = &wx[u >> 1][8 * (u & 1)];
        u32x4 vh, vm, vl;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            vh[e] = __builtin_amdgcn_perm(s[2 * e + 1], s[2 * e], 0x07060302u);
            vm[e] = __builtin_amdgcn_perm(s[2 * e + 1], s[2 * e], 0x05040100u);
            vl[e] = P == 3 ? lx[u >> 1][4 * (u & 1) + e] : 0u;
        }
        bh = __builtin_bit_cast(bf8, vh); bm = __builtin_bit_cast(bf8, vm); bl = __builtin_bit_cast(bf8, vl);
    }, z, lane);
}

// x as SplitPairs, all three terms (six products)
template <int MB, int KSTEPS, int PS, int NB>
__device__ __forceinline__ void matvec_split(const unsigned char* __restrict__ W, const SplitPairs<NB>& x, v16f* z, int lane) {
    matvec_split_core<MB, KSTEPS, PS, 3>(W, [&](int u, bf8& bh, bf8& bm, bf8& bl) {
        u32x4 vh, vm, vl;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            vh[e] = x.h[u >> 1][4 * (u & 1) + e];
            vm[e] = x.m[u >> 1][4 * (u & 1) + e];
            vl[e] = x.l[u >> 1][4 * (u & 1) + e];
        }
        bh = __builtin_bit_cast(bf8, vh); bm = __builtin_bit_cast(bf8, vm); bl = __builtin_bit_cast(bf8, vl);
    }, z, lane);
}

// The same for a factor Z with at most 16 columns (the 16-wide output adjoint, the 3 colour
// adjoints), on v_mfma_f32_16x16x4_f32: half the matrix-pipe time of a 32-row block that is
// half or nearly all padding, and a quarter of the accumulator registers per 32 columns.
//   D(16x16) += A(16x4) B(4x16); lane l holds A[l%16][l/16] and B[l/16][l%16], and register v
//   of lane l holds D[4*(l/16) + v][l%16]   (checked on the chip).
// G[cb][v] accumulates row 4*(lane/16) + v, column 16*cb + lane%16 of Z^T X.
typedef float v4f __attribute__((ext_vector_type(4)));

template <int XB, int LDZ, int LDX>
__device__ __forceinline__ void outer_accumulate16(v4f* G, const float* __restrict__ Zt, const float* __restrict__ Xt,
                                                   int lane) {
    constexpr int CB = 2 * XB;
    const int i = lane & 15, k = lane >> 4;
    float a = Zt[k * LDZ + i], an = 0.f, b[CB], bn[CB];
#pragma unroll
    for (int cb = 0; cb < CB; ++cb) b[cb] = Xt[k * LDX + 16 * cb + i];
#pragma unroll
    for (int s = 0; s < 8; ++s) {
        if (s + 1 < 8) {
            an = Zt[(4 * s + 4 + k) * LDZ + i];
#pragma unroll
            for (int cb = 0; cb < CB; ++cb) bn[cb] = Xt[(4 * s + 4 + k) * LDX + 16 * cb + i];
        }
#pragma unroll
        for (int cb = 0; cb < CB; ++cb) G[cb] = __builtin_amdgcn_mfma_f32_16x16x4f32(a, b[cb], G[cb], 0, 0, 0);
        a = an;
#pragma unroll
        for (int cb = 0; cb < CB; ++cb) b[cb] = bn[cb];
        __builtin_amdgcn_sched_barrier(0);
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

// Sum V register vectors over the block's WAVES waves; the result is valid in wave 0.  The
// other waves park their vectors in LDS, HALF = ceil(V/2) at a time (scratch holds
// (WAVES-1) * HALF * 1024 floats), and wave 0 adds them: four barriers for any V instead of
// WAVES per vector.  Every thread of the block must call it.
template <int WAVES, int V>
__device__ __forceinline__ void block_sum_all(float* __restrict__ scratch, v16f* (&vec)[V], int wave, int lane) {
    constexpr int HALF = (V + 1) / 2;
#pragma unroll
    for (int round = 0; round < 2; ++round) {
        if (wave > 0) {
#pragma unroll
            for (int k = 0; k < HALF; ++k)
                if (round * HALF + k < V) {
#pragma unroll
                    for (int r = 0; r < 16; ++r)
                        scratch[((wave - 1) * HALF + k) * 1024 + r * 64 + lane] = (*vec[round * HALF + k])[r];
                }
        }
        __syncthreads();
        if (wave == 0) {
#pragma unroll
            for (int k = 0; k < HALF; ++k)
                if (round * HALF + k < V) {
#pragma unroll
                    for (int wv = 0; wv < WAVES - 1; ++wv)
#pragma unroll
                        for (int r = 0; r < 16; ++r)
                            (*vec[round * HALF + k])[r] += scratch[(wv * HALF + k) * 1024 + r * 64 + lane];
                }
        }
        __syncthreads();
    }
}

}  // namespace neus2
