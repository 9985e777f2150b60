// Wave-level building blocks for tiny bias-free MLPs on the matrix cores of gfx950.
//
// One wavefront (64 lanes) owns a tile of 32 points.  A per-point vector of up to 64 neurons
// lives in fp32 registers in the layout that the 32x32 matrix instructions produce:
//
//     lane = 32*h + j   (j = point within the tile, h = 0/1)
//     v[b][r], b = block of 32 neurons, r = 0..15  <->  neuron 32*b + 8*(r/4) + 4*h + (r%4)
//
// Products run on v_mfma_f32_32x32x16_bf16, which has 16 times the rate of the fp32 matrix
// instruction: every fp32 factor is written as a sum of bf16 terms (round to nearest even each
// time) and the product as a sum of products of terms, accumulated in fp32.
//   * three terms, x = hi + mid + lo (|x - hi - mid - lo| <= 2^-24 |x|), and the six products
//     hi*hi, hi*mid, mid*hi, mid*mid, hi*lo, lo*hi: as accurate as an fp32 product.  Used for
//     everything that is compared at forward tolerance or decides a ReLU mask (the forward kernels,
//     and the forward pass where a backward kernel recomputes it: the same arithmetic in both, so
//     the masks agree bit for bit).
//   * two terms and the three products hi*hi, hi*mid, mid*hi: relative error about 2^-16 per
//     product.  Used for quantities compared at gradient tolerance: the adjoint, S and t sweeps
//     and the weight gradients, whose rounding errors moreover average out over the points.
//
//   D(32x32) += A(32x16) B(16x32); lane l holds A[l%32][8*(l/32) + s] and B[8*(l/32) + s][l%32],
//   s = 0..7, and D in the register layout above (checked on the chip).
//
// Matrix-vector products z = W x: x is the B operand.  Registers 8q..8q+7 of input block kb are
// the eight operand slots of k-step u = 2 kb + q as they stand, so slot s of lane half g is input
// 32 kb + 16 q + 8 (s/4) + 4 g + s%4, and W is stored in LDS with its columns in that order
// (SplitMatrix).  Activations therefore never leave registers between layers, in forward mode
// (z = W x), in reverse mode (x = W^T z, from a transposed copy) and in the forward-mode sweep of
// the second-order term.
//
// Weight gradients contract over points instead, and the contraction index must run along a
// lane's eight operand slots: both factors go through a per-wave LDS tile kept transposed,
// [neuron][point], one 32-bit word [hi | mid] per element; a lane reads its eight points as two
// 16-byte words (row stride kLdT words: conflict-free).
#pragma once

#include <hip/hip_runtime.h>

namespace neus2 {

typedef float v16f __attribute__((ext_vector_type(16)));
typedef float v4f __attribute__((ext_vector_type(4)));
typedef __bf16 bf8 __attribute__((ext_vector_type(8)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int kLd64 = 68;   // row stride (floats) of fp32 tiles [32 points][64 neurons]
constexpr int kLdT = 36;    // row stride (words) of a transposed split tile [64 neurons][32 points]
constexpr int kTileWords = 64 * kLdT;   // a per-wave tile holds either layout

__device__ __forceinline__ v16f zero16() {
    v16f z;
#pragma unroll
    for (int r = 0; r < 16; ++r) z[r] = 0.f;
    return z;
}

// neuron (within its block of 32) that register r of lane half h holds
__device__ __forceinline__ constexpr int neuron_of(int r, int h) { return 8 * (r >> 2) + 4 * h + (r & 3); }

// ReLU in place; returns the mask bits of this lane's 16*NB neurons (bit 16*b + r).
// The mask is 1 only for strictly positive pre-activations (Definition 1 of the paper).
// Neither direction uses a compare instruction: the result of a compare is a lane mask in a
// scalar register pair, 32 of them per mask word, which the compiler parks in vector-register
// lanes and fetches back for every use.  A float is positive exactly when its bit pattern is a
// positive integer, so the ReLU is an integer maximum with 0 on the pattern, the mask bit the
// unsigned minimum of the result with 1, and a one-bit sign-extending field extract turns a mask
// bit back into an all-ones or all-zeros word to AND with.  The mask instructions are written out
// because the compiler rewrites the equivalent C expressions into compares and selects; the
// instruction that first touches a result of a matrix instruction (the maximum, the AND) is left to
// the compiler, which knows the wait states a matrix result needs and does not look into asm text.
template <int NB>
__device__ __forceinline__ uint32_t relu_mask(v16f* z) {
    uint32_t m = 0;
#pragma unroll
    for (int b = 0; b < NB; ++b)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const float zf = z[b][r];       // a copy: a bit cast of the vector element itself reads element 0
            const int zi = max(__builtin_bit_cast(int, zf), 0);
            uint32_t on;
            asm("v_min_u32 %0, 1, %1" : "=v"(on) : "v"(zi));
            asm("v_lshl_or_b32 %0, %1, %2, %0" : "+v"(m) : "v"(on), "n"(16 * b + r));
            z[b][r] = __builtin_bit_cast(float, zi);
        }
    return m;
}

// ReLU in place without building the mask (for a kernel that is handed the masks).
template <int NB>
__device__ __forceinline__ void relu(v16f* z) {
#pragma unroll
    for (int b = 0; b < NB; ++b)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const float zf = z[b][r];
            z[b][r] = __builtin_bit_cast(float, max(__builtin_bit_cast(int, zf), 0));
        }
}

template <int NB>
__device__ __forceinline__ void apply_mask(v16f* z, uint32_t m) {
#pragma unroll
    for (int b = 0; b < NB; ++b)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            uint32_t keep;
            asm("v_bfe_i32 %0, %1, %2, 1" : "=v"(keep) : "v"(m), "n"(16 * b + r));
            const float zf = z[b][r];
            z[b][r] = __builtin_bit_cast(float, __builtin_bit_cast(uint32_t, zf) & keep);
        }
}

// Write a register vector to a per-wave fp32 tile [32 points][LD].
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

// ---- split vectors ---------------------------------------------------------------------------
// The P terms of a vector, each packed two elements to a word ([term(2p+1) | term(2p)]): words
// 4q..4q+3 of block kb are the operand of k-step 2 kb + q as they stand, and one conversion
// instruction yields a word.
template <int NB, int P>
struct Split {
    uint32_t t[P][NB][8];
};

// The remainder x - term is exact in binary32 (the term is x rounded to 8 significant bits), and
// one v_dot2c_f32_bf16 yields it from the packed word: x + (-1) * term(this element) + 0 * term(the
// other element), also exact (checked on the chip over all exponents).  The selector words are kept
// in registers: written as literals the compiler turns (-1, 0) into the inline constant -1.0, which
// the instruction reads as (0, -1).  A non-finite neighbour turns the remainder into NaN (0 * inf).
// (The asm statement is one instruction, not an empty one: the compiler counts every asm statement as
// an instruction when it works out the wait states between a matrix instruction and its reader.)
template <uint32_t V>
__device__ __forceinline__ uint32_t in_register() {
    uint32_t r;
    asm("s_mov_b32 %0, %1" : "=s"(r) : "n"(V));
    return r;
}

template <int NB, int P>
__device__ __forceinline__ void split(const v16f* v, Split<NB, P>& out) {
    typedef __bf16 bf2 __attribute__((ext_vector_type(2)));
    typedef float f2 __attribute__((ext_vector_type(2)));
    static_assert(P == 2 || P == 3, "two or three terms");
    const bf2 minus_low = __builtin_bit_cast(bf2, in_register<0x0000bf80u>());
    const bf2 minus_high = __builtin_bit_cast(bf2, in_register<0xbf800000u>());
#pragma unroll
    for (int b = 0; b < NB; ++b)
#pragma unroll
        for (int p = 0; p < 8; ++p) {
            float x0 = v[b][2 * p], x1 = v[b][2 * p + 1];
#pragma unroll
            for (int term = 0; term < P; ++term) {
                const uint32_t w = __builtin_bit_cast(uint32_t, __builtin_convertvector(f2{x0, x1}, bf2));
                out.t[term][b][p] = w;
                if (term + 1 < P && P == 2) {
                    x0 = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf2, w), minus_low, x0, false);
                    x1 = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf2, w), minus_high, x1, false);
                } else if (term + 1 < P) {
                    // the three-term splits of the forward kernels run two waves to a SIMD and measured
                    // slower with the dot instruction: shift or mask, and subtract
                    x0 -= __builtin_bit_cast(float, w << 16);
                    x1 -= __builtin_bit_cast(float, w & 0xffff0000u);
                }
            }
        }
}

// Write the first two terms to a per-wave transposed tile, one word [hi | mid] per element.
template <int NB, int P>
__device__ __forceinline__ void stage_split(uint32_t* __restrict__ tile, const Split<NB, P>& x, int j, int h) {
#pragma unroll
    for (int b = 0; b < NB; ++b)
#pragma unroll
        for (int p = 0; p < 8; ++p) {
            const uint32_t hp = x.t[0][b][p], mp = x.t[1][b][p];
            tile[(32 * b + neuron_of(2 * p, h)) * kLdT + j] = __builtin_amdgcn_perm(hp, mp, 0x05040100u);
            tile[(32 * b + neuron_of(2 * p + 1, h)) * kLdT + j] = __builtin_amdgcn_perm(hp, mp, 0x07060302u);
        }
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
// tiles transposed and split as above: 12 instructions of 32 clocks for a 32x32 block.  G is in
// the register layout at the top with rows = neurons of Z, columns (lane j) = neurons of X.
template <int ZB, int XB>
__device__ __forceinline__ void outer_accumulate_split(v16f (*G)[XB], const uint32_t* __restrict__ Zt,
                                                       const uint32_t* __restrict__ Xt, int lane) {
    const int i = lane & 31, g = lane >> 5;
    // the words of the second k-step are requested before the instructions of the first are issued
    u32x4 raw[2][ZB + XB][2];
    auto request = [&](int t) {
#pragma unroll
        for (int nb = 0; nb < XB; ++nb) {
            const u32x4* src = reinterpret_cast<const u32x4*>(Xt + (32 * nb + i) * kLdT + 16 * t + 8 * g);
            raw[t][nb][0] = src[0]; raw[t][nb][1] = src[1];
        }
#pragma unroll
        for (int mb = 0; mb < ZB; ++mb) {
            const u32x4* src = reinterpret_cast<const u32x4*>(Zt + (32 * mb + i) * kLdT + 16 * t + 8 * g);
            raw[t][XB + mb][0] = src[0]; raw[t][XB + mb][1] = src[1];
        }
    };
    request(0);
#pragma unroll
    for (int t = 0; t < 2; ++t) {
        bf8 bh[XB], bm[XB], ah[ZB], am[ZB];
#pragma unroll
        for (int nb = 0; nb < XB; ++nb) unpack_split(raw[t][nb][0], raw[t][nb][1], bh[nb], bm[nb]);
#pragma unroll
        for (int mb = 0; mb < ZB; ++mb) unpack_split(raw[t][XB + mb][0], raw[t][XB + mb][1], ah[mb], am[mb]);
        if (t == 0) request(1);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int mb = 0; mb < ZB; ++mb)
#pragma unroll
            for (int nb = 0; nb < XB; ++nb) {
                G[mb][nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ah[mb], bh[nb], G[mb][nb], 0, 0, 0);
                G[mb][nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ah[mb], bm[nb], G[mb][nb], 0, 0, 0);
                G[mb][nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(am[mb], bh[nb], G[mb][nb], 0, 0, 0);
            }
        __builtin_amdgcn_sched_barrier(0);
    }
}

// ---- split matrices ----------------------------------------------------------------------------
// A matrix in LDS for the products above: per output row [k-step][lane half][term][8 bf16], the
// slots in the order given at the top, so that a lane reads each term of its operand as one
// 16-byte word; the row stride leaves 16 bytes of padding, which makes those reads conflict-free.
template <int KSTEPS, int PS>
struct SplitMatrix {
    static constexpr int kLd = KSTEPS * 2 * PS * 16 + 16;     // bytes per output row

    // Fills rows 0..ROWS-1 of the matrix at W, every slot of them (what lies outside the caller's
    // matrix is written as zero, so W needs no clearing): element (r, c) is get(r, c).  A thread
    // takes whole operand words: it fetches the eight inputs of one (row, k-step, lane half),
    // splits them and writes each term as one 16-byte word.  load() only issues the fetches, so
    // that a kernel can have those of all its matrices in flight before the first store() waits.
    // ROW_FASTEST says which index runs along the lanes: the one contiguous in the source.
    template <int ROWS, int THREADS, bool ROW_FASTEST>
    struct Fill {
        static constexpr int kUnits = ROWS * KSTEPS * 2;
        static constexpr int kPer = (kUnits + THREADS - 1) / THREADS;
        float v[kPer > 0 ? kPer : 1][8];

        __device__ static __forceinline__ void decode(int unit, int& r, int& ug) {
            constexpr int kRows = ROWS > 0 ? ROWS : 1;
            if (ROW_FASTEST) { r = unit % kRows; ug = unit / kRows; }
            else { ug = unit % (2 * KSTEPS); r = unit / (2 * KSTEPS); }
        }
        template <class Get>
        __device__ __forceinline__ void load(int tid, Get get) {
#pragma unroll
            for (int k = 0; k < kPer; ++k) {
                const int unit = tid + k * THREADS;
                if (kUnits % THREADS != 0 && unit >= kUnits) break;
                int r, ug;
                decode(unit, r, ug);
                const int c0 = 16 * (ug >> 1) + 4 * (ug & 1);
#pragma unroll
                for (int s = 0; s < 8; ++s) v[k][s] = get(r, c0 + 8 * (s >> 2) + (s & 3));
            }
        }
        __device__ __forceinline__ void store(unsigned char* __restrict__ W, int tid) const {
            typedef __bf16 bf2 __attribute__((ext_vector_type(2)));
            typedef float f2 __attribute__((ext_vector_type(2)));
#pragma unroll
            for (int k = 0; k < kPer; ++k) {
                const int unit = tid + k * THREADS;
                if (kUnits % THREADS != 0 && unit >= kUnits) break;
                int r, ug;
                decode(unit, r, ug);
                unsigned char* dst = W + r * kLd + ug * (PS * 16);
                float x[8];
#pragma unroll
                for (int s = 0; s < 8; ++s) x[s] = v[k][s];
#pragma unroll
                for (int term = 0; term < PS; ++term) {
                    u32x4 word;
#pragma unroll
                    for (int p = 0; p < 4; ++p) {
                        const uint32_t w = __builtin_bit_cast(uint32_t, __builtin_convertvector(f2{x[2 * p], x[2 * p + 1]}, bf2));
                        word[p] = w;
                        x[2 * p] -= __builtin_bit_cast(float, w << 16);
                        x[2 * p + 1] -= __builtin_bit_cast(float, w & 0xffff0000u);
                    }
                    *reinterpret_cast<u32x4*>(dst + 16 * term) = word;
                }
            }
        }
    };
};

// z[mb] = sum_c W[32 mb + .][c] x[c] for MB blocks of outputs and KSTEPS * 16 inputs; W is a
// SplitMatrix<KSTEPS, PS>; P terms of W and of x are used (P = 2: three products, P = 3: six).
template <int MB, int KSTEPS, int PS, int P, int NB, int PX>
__device__ __forceinline__ void matvec_split(const unsigned char* __restrict__ W, const Split<NB, PX>& x, v16f* z, int lane) {
    static_assert(P == 2 || P == 3, "two or three terms");
    static_assert(P <= PS && P <= PX, "a factor holds fewer terms than asked for");
    static_assert(KSTEPS <= 2 * NB, "the vector is shorter than the matrix is wide");
    constexpr int kLd = SplitMatrix<KSTEPS, PS>::kLd;
    constexpr int kTotal = KSTEPS * MB;
    const int i = lane & 31, g = lane >> 5;
    const unsigned char* base = W + i * kLd + g * (PS * 16);
    // The weights of the next step are requested from LDS before the instructions of the current
    // step are issued, and the scheduler is told not to move anything across step boundaries: left
    // alone it hoists every LDS read of the kernel to the top and runs out of registers (letting
    // only ALU instructions cross was measured and is slower).  Output blocks are computed one
    // after the other (step t = mb * KSTEPS + u).
    auto address = [&](int t) -> const u32x4* {
        const int mb = t / KSTEPS, u = t % KSTEPS;
        return reinterpret_cast<const u32x4*>(base + 32 * mb * kLd + u * (2 * PS * 16));
    };
    u32x4 cur[P], nxt[P];
#pragma unroll
    for (int p = 0; p < P; ++p) cur[p] = address(0)[p];
    v16f acc[MB];
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) acc[mb] = zero16();
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) {
#pragma unroll
        for (int u = 0; u < KSTEPS; ++u) {
            bf8 bt[P];
#pragma unroll
            for (int p = 0; p < P; ++p) {
                u32x4 v;
#pragma unroll
                for (int e = 0; e < 4; ++e) v[e] = x.t[p][u >> 1][4 * (u & 1) + e];
                bt[p] = __builtin_bit_cast(bf8, v);
            }
            const int t = mb * KSTEPS + u;
#pragma unroll
            for (int p = 0; p < P; ++p) nxt[p] = cur[p];
            if (t + 1 < kTotal) {
#pragma unroll
                for (int p = 0; p < P; ++p) nxt[p] = address(t + 1)[p];
            }
            const bf8 ah = __builtin_bit_cast(bf8, cur[0]), am = __builtin_bit_cast(bf8, cur[1]);
            acc[mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ah, bt[0], acc[mb], 0, 0, 0);
            acc[mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ah, bt[1], acc[mb], 0, 0, 0);
            acc[mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(am, bt[0], acc[mb], 0, 0, 0);
            if (P == 3) {
                const bf8 al = __builtin_bit_cast(bf8, cur[P - 1]);
                acc[mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(am, bt[1], acc[mb], 0, 0, 0);
                acc[mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ah, bt[P - 1], acc[mb], 0, 0, 0);
                acc[mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(al, bt[0], acc[mb], 0, 0, 0);
            }
#pragma unroll
            for (int p = 0; p < P; ++p) cur[p] = nxt[p];
            __builtin_amdgcn_sched_barrier(0);
        }
    }
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) z[mb] = acc[mb];
}

// Weight gradient of a factor Z with at most 16 columns (the 16-wide output adjoint, the 3
// colour adjoints), in fp32 on v_mfma_f32_16x16x4_f32, from tiles [32 points][LD] of floats.
//   D(16x16) += A(16x4) B(4x16); lane l holds A[l%16][l/16] and B[l/16][l%16], and register v
//   of lane l holds D[4*(l/16) + v][l%16]   (checked on the chip).
// G[cb][v] accumulates row 4*(lane/16) + v, column 16*cb + lane%16 of Z^T X.
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

// Sum V register vectors over the block's WAVES waves such that every wave ends up with a share of
// the totals: wave w holds, in registers 16/WAVES * w .. 16/WAVES * (w+1) - 1 of every vector, the
// block's sums (its other registers keep its own partial sums).  All waves then flush their share
// in parallel.  scratch: WAVES * V * 1024 floats of LDS nobody reads any more; one barrier inside,
// and the caller has put one before (the scratch overlays memory other waves may still be using).
// Every thread of the block must call it.
template <int WAVES, int V>
__device__ __forceinline__ void block_sum_shared(float* __restrict__ scratch, v16f* (&vec)[V], int wave, int lane) {
    static_assert(16 % WAVES == 0, "registers are dealt out evenly");
    constexpr int kShare = 16 / WAVES;
#pragma unroll
    for (int k = 0; k < V; ++k)
#pragma unroll
        for (int r = 0; r < 16; ++r) scratch[((wave * V + k) * 16 + r) * 64 + lane] = (*vec[k])[r];
    __syncthreads();
#pragma unroll
    for (int k = 0; k < V; ++k)
#pragma unroll
        for (int q = 0; q < kShare; ++q) {
            float sum = 0.f;
#pragma unroll
            for (int w = 0; w < WAVES; ++w) sum += scratch[((w * V + k) * 16 + wave * kShare + q) * 64 + lane];
            // written through a loop over constant register numbers: the share's first register depends on the wave
#pragma unroll
            for (int r = 0; r < 16; ++r)
                if (r == wave * kShare + q) (*vec[k])[r] = sum;
        }
}

}  // namespace neus2
