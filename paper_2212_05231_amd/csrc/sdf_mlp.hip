// SDF network: forward + analytic input gradient, and the backward pass with the
// second-order term, fused per 32-point tile on the matrix cores (fp32 values as sums of bf16
// terms, see mfma_tile.h).
//
// Paper: Eq. 1 ((d,g) = f_Theta(e)), Definition 1 (bias-free ReLU MLP, masks G_l, vectors
// P_l^j and S_l^i), Eq. 2 (n = grad_x d), supplement Sec. B (dy/dx = H_L G_L ... G_2 H_1),
// Theorem 1 (d(dy/dx)_(i,j)/dH_l = (P_l^j S_l^i)^T, second input derivative zero) and
// Eqs. 7-8 (what is left of the chain rule).
//
// With i = 0 (the SDF output), S_l is the reverse sweep from row 0 of the last matrix and
// the sum over j of P_l^j weighted by (de/dx) dL/dn is ONE forward-mode sweep t_l, so
//     dL/dH_l = delta_l a_{l-1}^T  +  S_l^T t_{l-1}^T        (first + second order)
// Both products contract over points and run as MFMA outer-product accumulations.
// Activations and masks are recomputed in the backward kernel from the encoding (cheaper
// than storing and re-reading four 64-wide vectors per point).
#include "common.h"
#include "mfma_tile.h"

namespace neus2 {

namespace {

constexpr int kThreads = 256;
constexpr int kWaves = kThreads / 64;

struct SdfArgs {
    const float* enc; const float* jac; const float* H[3];
    const float* d_y; const float* d_normal;
    float* y; float* q; float* normal;
    float* dH[3]; float* d_enc; float* d_pos;
    uint32_t* masks;           // optional [2][n][2]: written by the forward kernel, read by the backward kernel
    int64_t n; int active_levels;
    bool stream_q;             // q (forward kernel) and dL/de (backward kernel) with non-temporal stores
};

// The ReLU masks of a point as the kernels keep them: one word per hidden layer and lane half h,
// bit 16 b + r for neuron 32 b + neuron_of(r, h); word (layer * n + i) * 2 + h of the buffer.
__device__ __forceinline__ int64_t mask_word(int layer, int64_t n, int64_t i, int h) { return ((int64_t)layer * n + i) * 2 + h; }

// LDS copies of the matrices, split into bf16 terms (see mfma_tile.h), in the orientations a
// kernel needs ("f": rows = outputs, "t": rows = inputs).  Everything the forward kernel
// computes, and the forward pass where the backward kernel recomputes it, uses three terms per
// factor and six products: as accurate as fp32 arithmetic, and the same arithmetic in both
// kernels, so the ReLU masks agree.  The adjoint, S and t sweeps of the backward kernel use
// two terms and three products.
template <int D, int K, bool BWD>
struct SdfWeights {
    static constexpr int KS1 = D / 16;
    typedef SplitMatrix<KS1, 3> M1f;               // [64][D]
    typedef SplitMatrix<4, 3> M2f;                 // [64][64]
    typedef SplitMatrix<4, 3> MLf;                 // last matrix [16 -> 32][64]
    typedef SplitMatrix<4, BWD ? 2 : 3> M1t;       // [D -> 32][64]
    typedef SplitMatrix<4, BWD ? 2 : 3> M2t;
    typedef SplitMatrix<1, 2> MLt;                 // [64][16]
    alignas(16) unsigned char H1f[64 * M1f::kLd];
    alignas(16) unsigned char H1t[32 * M1t::kLd];
    alignas(16) unsigned char H2f[K == 3 ? 64 * M2f::kLd : 16];
    alignas(16) unsigned char H2t[K == 3 ? 64 * M2t::kLd : 16];
    alignas(16) unsigned char HLf[BWD ? 16 : 32 * MLf::kLd];
    alignas(16) unsigned char HLt[BWD ? 64 * MLt::kLd : 16];
    // Row 0 of the last matrix (the SDF output), already split and packed as a lane holds it
    // (Split<2, 3>): [lane half][term][word 8 b + p]
    alignas(16) uint32_t HLrow0[2][3][16];
};

// Every matrix is fetched from global memory before the first is written to LDS, so the fetches
// are in flight together; the copies cover every slot a product reads, so nothing is cleared.
template <int D, int K, bool BWD, int THREADS>
__device__ void load_weights(SdfWeights<D, K, BWD>& w, const SdfArgs& a) {
    typedef SdfWeights<D, K, BWD> W;
    const int tid = threadIdx.x;
    const float* __restrict__ H1 = a.H[0];
    const float* __restrict__ H2 = a.H[1];
    const float* __restrict__ HL = a.H[K - 1];
    typename W::M1f::template Fill<64, THREADS, false> f1;
    typename W::M1t::template Fill<32, THREADS, true> t1;
    typename W::M2f::template Fill<K == 3 ? 64 : 0, THREADS, false> f2;
    typename W::M2t::template Fill<K == 3 ? 64 : 0, THREADS, true> t2;
    typename W::MLf::template Fill<BWD ? 0 : 32, THREADS, false> fl;
    typename W::MLt::template Fill<BWD ? 64 : 0, THREADS, true> tl;
    f1.load(tid, [&](int o, int i) { return H1[o * D + i]; });
    t1.load(tid, [&](int i, int o) { return i < D ? H1[o * D + i] : 0.f; });
    f2.load(tid, [&](int o, int i) { return H2[o * 64 + i]; });
    t2.load(tid, [&](int i, int o) { return H2[o * 64 + i]; });
    fl.load(tid, [&](int o, int i) { return o < 16 ? HL[o * 64 + i] : 0.f; });
    tl.load(tid, [&](int i, int o) { return HL[o * 64 + i]; });
    // thread 16 h + 8 b + p < 32 splits the pair of row-0 elements that word p of block b of lane
    // half h holds: registers 2p and 2p + 1
    float row0[2] = {0.f, 0.f};
    if (tid < 32) {
        const int hh = tid >> 4, b = (tid >> 3) & 1, p = tid & 7;
        row0[0] = HL[32 * b + neuron_of(2 * p, hh)];
        row0[1] = HL[32 * b + neuron_of(2 * p + 1, hh)];
    }
    f1.store(w.H1f, tid);
    t1.store(w.H1t, tid);
    f2.store(w.H2f, tid);
    t2.store(w.H2t, tid);
    fl.store(w.HLf, tid);
    tl.store(w.HLt, tid);
    if (tid < 32) {
        typedef __bf16 bf2 __attribute__((ext_vector_type(2)));
        typedef float f2 __attribute__((ext_vector_type(2)));
        float x0 = row0[0], x1 = row0[1];
#pragma unroll
        for (int term = 0; term < 3; ++term) {
            const uint32_t word = __builtin_bit_cast(uint32_t, __builtin_convertvector(f2{x0, x1}, bf2));
            w.HLrow0[tid >> 4][term][tid & 15] = word;
            x0 -= __builtin_bit_cast(float, word << 16);
            x1 -= __builtin_bit_cast(float, word & 0xffff0000u);
        }
    }
    __syncthreads();
}

// level-major [L][n][2] <-> register vector of width D.  Register r = 4g + 2u + f of lane half h
// is feature f of level 4g + 2h + u.
template <int D>
__device__ __forceinline__ v16f load_levels(const float* __restrict__ src, int64_t n, int64_t i, bool valid,
                                            int active, int h) {
    v16f x = zero16();
#pragma unroll
    for (int g = 0; g < D / 8; ++g)
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            const int level = 4 * g + 2 * h + u;
            if (valid && level < active) {
                const float2 v = reinterpret_cast<const float2*>(src)[(int64_t)level * n + i];
                x[4 * g + 2 * u] = v.x;
                x[4 * g + 2 * u + 1] = v.y;
            }
        }
    return x;
}

template <int D, bool STREAM = false>
__device__ __forceinline__ void store_levels(float* __restrict__ dst, int64_t n, int64_t i, bool valid,
                                             const v16f& x, int h) {
    if (!valid) return;
#pragma unroll
    for (int g = 0; g < D / 8; ++g)
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            const int level = 4 * g + 2 * h + u;
            if (STREAM) {
                typedef float f2v __attribute__((ext_vector_type(2)));
                __builtin_nontemporal_store(f2v{x[4 * g + 2 * u], x[4 * g + 2 * u + 1]}, reinterpret_cast<f2v*>(dst) + (int64_t)level * n + i);
            } else {
                reinterpret_cast<float2*>(dst)[(int64_t)level * n + i] = make_float2(x[4 * g + 2 * u], x[4 * g + 2 * u + 1]);
            }
        }
}

// out_a = sum over this lane's features of x_k * J[k][a]   (J = de/dx; per level three planes [n] of
// pairs: (J00,J01), (J02,J10), (J11,J12))
template <int D>
__device__ __forceinline__ void contract_jac(const float* __restrict__ jac, int64_t n, int64_t i, bool valid,
                                             int active, int h, const v16f& x, float out[3]) {
    out[0] = out[1] = out[2] = 0.f;
#pragma unroll
    for (int g = 0; g < D / 8; ++g)
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            const int level = 4 * g + 2 * h + u;
            if (valid && level < active) {
                const float2* J = reinterpret_cast<const float2*>(jac) + (int64_t)level * 3 * n + i;
                const float2 a = J[0], b = J[n], c = J[2 * n];     // (J00,J01) (J02,J10) (J11,J12)
                const float x0 = x[4 * g + 2 * u], x1 = x[4 * g + 2 * u + 1];
                out[0] += x0 * a.x + x1 * b.y;
                out[1] += x0 * a.y + x1 * c.x;
                out[2] += x0 * b.x + x1 * c.y;
            }
        }
}

// t_k = sum_a J[k][a] * v_a
template <int D>
__device__ __forceinline__ v16f apply_jac(const float* __restrict__ jac, int64_t n, int64_t i, bool valid,
                                          int active, int h, const float v[3]) {
    v16f t = zero16();
#pragma unroll
    for (int g = 0; g < D / 8; ++g)
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            const int level = 4 * g + 2 * h + u;
            if (valid && level < active) {
                const float2* J = reinterpret_cast<const float2*>(jac) + (int64_t)level * 3 * n + i;
                const float2 a = J[0], b = J[n], c = J[2 * n];
                t[4 * g + 2 * u] = a.x * v[0] + a.y * v[1] + b.x * v[2];
                t[4 * g + 2 * u + 1] = b.y * v[0] + c.x * v[1] + c.y * v[2];
            }
        }
    return t;
}

// The Jacobian rows of this lane's features, held in registers so that the loads can be issued
// long before they are needed.
template <int D>
struct JacRegs {
    float2 v[D / 4][3];        // per level of this lane: (J00,J01) (J02,J10) (J11,J12)
};

template <int D>
__device__ __forceinline__ JacRegs<D> load_jac(const float* __restrict__ jac, int64_t n, int64_t i, bool valid,
                                               int active, int h) {
    JacRegs<D> J;
#pragma unroll
    for (int g = 0; g < D / 8; ++g)
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            const int level = 4 * g + 2 * h + u;
            const bool on = valid && level < active;
            const float2* p = reinterpret_cast<const float2*>(jac) + (int64_t)(on ? level : 0) * 3 * n + (on ? i : 0);
#pragma unroll
            // the Jacobian is the widest stream of the network kernels and is not read again before the
            // other kernel's turn, a whole batch later: non-temporal loads (5 us of the step)
            for (int c = 0; c < 3; ++c) {
                typedef float f2v __attribute__((ext_vector_type(2)));
                J.v[2 * g + u][c] = make_float2(0.f, 0.f);
                if (on) {
                    const f2v w = __builtin_nontemporal_load(reinterpret_cast<const f2v*>(p) + c * n);
                    J.v[2 * g + u][c] = make_float2(w.x, w.y);
                }
            }
        }
    return J;
}

template <int D>
__device__ __forceinline__ void contract_jac_regs(const JacRegs<D>& J, const v16f& x, float out[3]) {
    out[0] = out[1] = out[2] = 0.f;
#pragma unroll
    for (int g = 0; g < D / 8; ++g)
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            const float2 a = J.v[2 * g + u][0], b = J.v[2 * g + u][1], c = J.v[2 * g + u][2];
            const float x0 = x[4 * g + 2 * u], x1 = x[4 * g + 2 * u + 1];
            out[0] += x0 * a.x + x1 * b.y;
            out[1] += x0 * a.y + x1 * c.x;
            out[2] += x0 * b.x + x1 * c.y;
        }
}

template <int D>
__device__ __forceinline__ v16f apply_jac_regs(const JacRegs<D>& J, const float v[3]) {
    v16f t = zero16();
#pragma unroll
    for (int g = 0; g < D / 8; ++g)
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            const float2 a = J.v[2 * g + u][0], b = J.v[2 * g + u][1], c = J.v[2 * g + u][2];
            t[4 * g + 2 * u] = a.x * v[0] + a.y * v[1] + b.x * v[2];
            t[4 * g + 2 * u + 1] = b.y * v[0] + c.x * v[1] + c.y * v[2];
        }
    return t;
}

// Row 0 of the last matrix, masked (S_{K-1} of Definition 1 for output 0), as a split vector: the
// terms were split when the matrix was copied to LDS, and masking a packed pair is an AND with a
// word that has ones in the halves whose mask bit is set (bit 16 b + r for register r of block b;
// word p holds registers 2p and 2p + 1).  The same values as splitting the masked row.
template <int P>
__device__ __forceinline__ void last_row_masked(const uint32_t (*row0)[3][16], uint32_t m, int h, Split<2, P>& out) {
    uint32_t keep[16];
#pragma unroll
    for (int k = 0; k < 16; ++k) {
        const int bit = 16 * (k >> 3) + 2 * (k & 7);
        uint32_t lo, hi;
        asm("v_bfe_i32 %0, %1, %2, 1" : "=v"(lo) : "v"(m), "n"(bit));
        asm("v_bfe_i32 %0, %1, %2, 1" : "=v"(hi) : "v"(m), "n"(bit + 1));
        keep[k] = (lo & 0xffffu) | (hi & 0xffff0000u);
    }
#pragma unroll
    for (int term = 0; term < P; ++term)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            const u32x4 words = *reinterpret_cast<const u32x4*>(&row0[h][term][4 * g]);
#pragma unroll
            for (int e = 0; e < 4; ++e) out.t[term][g >> 1][4 * (g & 1) + e] = words[e] & keep[4 * g + e];
        }
}

// 16-wide per-point rows ([n][16]) <-> register vector: registers 0..7 of lane half h hold
// columns 4h..4h+3 and 8+4h..8+4h+3.
__device__ __forceinline__ v16f load_rows16(const float* __restrict__ src, int64_t i, bool valid, int h) {
    v16f x = zero16();
    if (valid) {
        const float4 a = *reinterpret_cast<const float4*>(src + i * 16 + 4 * h);
        const float4 b = *reinterpret_cast<const float4*>(src + i * 16 + 8 + 4 * h);
        x[0] = a.x; x[1] = a.y; x[2] = a.z; x[3] = a.w;
        x[4] = b.x; x[5] = b.y; x[6] = b.z; x[7] = b.w;
    }
    return x;
}

__device__ __forceinline__ void store_rows16(float* __restrict__ dst, int64_t i, bool valid, int h, const v16f& x) {
    if (!valid) return;
    *reinterpret_cast<float4*>(dst + i * 16 + 4 * h) = make_float4(x[0], x[1], x[2], x[3]);
    *reinterpret_cast<float4*>(dst + i * 16 + 8 + 4 * h) = make_float4(x[4], x[5], x[6], x[7]);
}

// ------------------------------------------------------------------------------------------
// The forward kernel runs 512 threads per workgroup: its 90 KB of matrices are shared by eight
// wavefronts, two per SIMD, so that one wavefront's waits for memory and LDS are filled by the
// other (vector and matrix instructions of a SIMD do not run side by side, but stalls do overlap).
constexpr int kFwdThreads = 512;
constexpr int kFwdWaves = kFwdThreads / 64;

template <int D, int K>
__global__ __launch_bounds__(kFwdThreads) void sdf_fwd_kernel(SdfArgs a) {
    __shared__ SdfWeights<D, K, false> w;
    load_weights<D, K, false, kFwdThreads>(w, a);
    constexpr int KS1 = SdfWeights<D, K, false>::KS1;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // the same for all lanes: keeps tile indices and addresses scalar
    const int j = lane & 31, h = lane >> 5;
    const int64_t tiles = (a.n + 31) / 32;
    const int64_t stride = (int64_t)gridDim.x * kFwdWaves;
    int64_t tile = (int64_t)blockIdx.x * kFwdWaves + wave;
    // the encoding of the NEXT tile and the Jacobian of THIS tile are requested before the
    // matrix work of this tile starts, so that HBM latency hides behind it
    v16f x_next = load_levels<D>(a.enc, a.n, tile * 32 + j, tile < tiles && tile * 32 + j < a.n, a.active_levels, h);
    for (; tile < tiles; tile += stride) {
        const int64_t i = tile * 32 + j;
        const bool valid = i < a.n;
        v16f x0[1] = {x_next};
        const JacRegs<D> J = load_jac<D>(a.jac, a.n, i, valid, a.active_levels, h);
        {
            const int64_t in = (tile + stride) * 32 + j;
            x_next = load_levels<D>(a.enc, a.n, in, tile + stride < tiles && in < a.n, a.active_levels, h);
        }
        v16f a1[2], yv[1];
        Split<1, 3> px;
        Split<2, 3> pv;
        split(x0, px);
        matvec_split<2, KS1, 3, 3>(w.H1f, px, a1, lane);
        const uint32_t m1 = relu_mask<2>(a1);
        uint32_t m_last = m1;
        split(a1, pv);
        if (K == 3) {
            v16f a2[2];
            matvec_split<2, 4, 3, 3>(w.H2f, pv, a2, lane);
            m_last = relu_mask<2>(a2);
            split(a2, pv);
        }
        matvec_split<1, 4, 3, 3>(w.HLf, pv, yv, lane);
        store_rows16(a.y, i, valid, h, yv[0]);
        if (a.masks && valid) {
            a.masks[mask_word(0, a.n, i, h)] = m1;
            if (K == 3) a.masks[mask_word(1, a.n, i, h)] = m_last;
        }
        // reverse sweep for dd/de
        v16f s1[2];
        last_row_masked(w.HLrow0, m_last, h, pv);
        if (K == 3) {
            matvec_split<2, 4, 3, 3>(w.H2t, pv, s1, lane);
            apply_mask<2>(s1, m1);
            split(s1, pv);
        }
        v16f qv[1];
        matvec_split<1, 4, 3, 3>(w.H1t, pv, qv, lane);
        // dd/de is read next by the scatter-add, four kernels later: for a batch whose per-point arrays
        // exceed the caches it is written with non-temporal stores (25 us of the step at 2^20 points; at
        // 2^18 points the cached store is the faster one)
        if (a.stream_q) store_levels<D, true>(a.q, a.n, i, valid, qv[0], h);
        else store_levels<D>(a.q, a.n, i, valid, qv[0], h);
        float nrm[3];
        contract_jac_regs<D>(J, qv[0], nrm);
#pragma unroll
        for (int c = 0; c < 3; ++c) nrm[c] += __shfl_xor(nrm[c], 32);
        if (valid && h == 0) {
            a.normal[3 * i + 0] = nrm[0]; a.normal[3 * i + 1] = nrm[1]; a.normal[3 * i + 2] = nrm[2];
        }
    }
}

// ------------------------------------------------------------------------------------------
template <int D, int K>
struct SdfBwdSmem {
    SdfWeights<D, K, true> w;
    float tiles[kWaves][2][kTileWords];
};

// add the registers [r0, r0 + count) of this wave's accumulator into dst[rows][cols] (row-major,
// ld = cols) with atomics; r0 is the same for all lanes
template <int ZB, int XB>
__device__ __forceinline__ void flush_grad(float* __restrict__ dst, int rows, int cols, v16f (*G)[XB], int j, int h,
                                           int r0, int count) {
#pragma unroll
    for (int mb = 0; mb < ZB; ++mb)
#pragma unroll
        for (int nb = 0; nb < XB; ++nb)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                if (r < r0 || r >= r0 + count) continue;
                const int o = 32 * mb + neuron_of(r, h), i = 32 * nb + j;
                if (o < rows && i < cols) atomicAdd(dst + o * cols + i, G[mb][nb][r]);
            }
}

// GIVEN: the masks come from the forward kernel (a.masks).  The forward pass is then recomputed
// only for its values, which enter weight gradients and further products at gradient tolerance:
// two terms and three products like the rest of this kernel, and a plain ReLU (where its sign
// differs from the given mask the value is within rounding of zero); every masked product uses
// the given masks.  Without them the forward pass is recomputed in the forward kernel's own
// arithmetic, which yields the same masks bit for bit.
template <int D, int K, bool GIVEN>
__global__ __launch_bounds__(kThreads) void sdf_bwd_kernel(SdfArgs a) {
    __shared__ SdfBwdSmem<D, K> sm;
    SdfWeights<D, K, true>& w = sm.w;
    load_weights<D, K, true, kThreads>(w, a);
    constexpr int KS1 = SdfWeights<D, K, true>::KS1;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // the same for all lanes: keeps tile indices and addresses scalar
    const int j = lane & 31, h = lane >> 5;
    float* Zt = sm.tiles[wave][0];
    float* Xt = sm.tiles[wave][1];
    uint32_t* Zs = reinterpret_cast<uint32_t*>(Zt);     // the same tiles in the transposed split layout
    uint32_t* Xs = reinterpret_cast<uint32_t*>(Xt);

    v16f G1[2][1], G2[2][2], tsum[2];
    v4f GL[4];                 // gradient of the last matrix [16][64]: four blocks of 16 columns
#pragma unroll
    for (int mb = 0; mb < 2; ++mb) {
        G1[mb][0] = zero16();
        G2[mb][0] = zero16(); G2[mb][1] = zero16();
        tsum[mb] = zero16();
    }
#pragma unroll
    for (int cb = 0; cb < 4; ++cb) GL[cb] = v4f{0.f, 0.f, 0.f, 0.f};

    const int64_t tiles = (a.n + 31) / 32;
    const int64_t stride = (int64_t)gridDim.x * kWaves;
    int64_t tile = (int64_t)blockIdx.x * kWaves + wave;
    // every global input of a tile is requested at its top (the next tile's encoding as well),
    // so that HBM latency hides behind the matrix work
    v16f x_next = load_levels<D>(a.enc, a.n, tile * 32 + j, tile < tiles && tile * 32 + j < a.n, a.active_levels, h);
    for (; tile < tiles; tile += stride) {
        const int64_t i = tile * 32 + j;
        const bool valid = i < a.n;
        v16f x0[1] = {x_next};
        v16f dK[1] = {zero16()};
        if (valid) {
            typedef float f4v __attribute__((ext_vector_type(4)));
            const f4v a_ = __builtin_nontemporal_load(reinterpret_cast<const f4v*>(a.d_y + i * 16 + 4 * h));
            const f4v b_ = __builtin_nontemporal_load(reinterpret_cast<const f4v*>(a.d_y + i * 16 + 8 + 4 * h));
            dK[0][0] = a_.x; dK[0][1] = a_.y; dK[0][2] = a_.z; dK[0][3] = a_.w;
            dK[0][4] = b_.x; dK[0][5] = b_.y; dK[0][6] = b_.z; dK[0][7] = b_.w;
        }
        // given masks are first needed after the forward pass has been recomputed
        uint32_t m1 = 0u, m_last = 0u;
        if (GIVEN && valid) {
            // masks and the adjoint of (d,g) are read here for the last time in the step: non-temporal loads
            m1 = __builtin_nontemporal_load(a.masks + mask_word(0, a.n, i, h));
            m_last = K == 3 ? __builtin_nontemporal_load(a.masks + mask_word(1, a.n, i, h)) : m1;
        }
        float nb3[3] = {0.f, 0.f, 0.f};
        if (valid) { nb3[0] = a.d_normal[3 * i]; nb3[1] = a.d_normal[3 * i + 1]; nb3[2] = a.d_normal[3 * i + 2]; }
        const JacRegs<D> J = load_jac<D>(a.jac, a.n, i, valid, a.active_levels, h);
        {
            const int64_t in = (tile + stride) * 32 + j;
            x_next = load_levels<D>(a.enc, a.n, in, tile + stride < tiles && in < a.n, a.active_levels, h);
        }
        // ---- forward pass again
        constexpr int PF = GIVEN ? 2 : 3;
        v16f a1[2], a2[2];
        Split<1, PF> px;         // x0: input of the first layer, factor of its weight gradient
        Split<2, PF> p1;         // a1 likewise for the second layer
        split(x0, px);
        matvec_split<2, KS1, 3, PF>(w.H1f, px, a1, lane);
        if (GIVEN) relu<2>(a1);
        else m_last = m1 = relu_mask<2>(a1);
        split(a1, p1);
        if (K == 3) {
            matvec_split<2, 4, 3, PF>(w.H2f, p1, a2, lane);
            if (GIVEN) relu<2>(a2);
            else m_last = relu_mask<2>(a2);
        }
        // t_0 = (de/dx) dL/dn, computed now so that the Jacobian's registers are free again
        v16f t0[1] = {apply_jac_regs<D>(J, nb3)};
        // ---- first-order chain delta_K .. delta_1 (two terms, three products from here on),
        // weight gradients as they appear
        v16f d2[2], d1[2];
        Split<1, 2> pk;
        Split<2, 2> pd;
        stage<1, kLd64>(Zt, dK, j, h);
        stage<2, kLd64>(Xt, K == 3 ? a2 : a1, j, h);
        wave_lds_fence();
        outer_accumulate16<2, kLd64, kLd64>(GL, Zt, Xt, lane);
        split(dK, pk);
        matvec_split<2, 1, 2, 2>(w.HLt, pk, d2, lane);
        apply_mask<2>(d2, m_last);
        if (K == 3) {
            split(d2, pd);
            wave_lds_fence();
            stage_split(Zs, pd, j, h);
            stage_split(Xs, p1, j, h);
            wave_lds_fence();
            outer_accumulate_split<2, 2>(G2, Zs, Xs, lane);
            matvec_split<2, 4, 2, 2>(w.H2t, pd, d1, lane);
            apply_mask<2>(d1, m1);
        } else {
            d1[0] = d2[0]; d1[1] = d2[1];
        }
        split(d1, pd);
        wave_lds_fence();
        stage_split(Zs, pd, j, h);
        stage_split(Xs, px, j, h);
        wave_lds_fence();
        outer_accumulate_split<2, 1>(G1, Zs, Xs, lane);
        v16f de[1];
        matvec_split<1, 4, 2, 2>(w.H1t, pd, de, lane);
        if (a.stream_q) store_levels<D, true>(a.d_enc, a.n, i, valid, de[0], h);      // as for q in the forward kernel
        else store_levels<D>(a.d_enc, a.n, i, valid, de[0], h);
        if (a.d_pos) {
            float dp[3];
            contract_jac<D>(a.jac, a.n, i, valid, a.active_levels, h, de[0], dp);
#pragma unroll
            for (int c = 0; c < 3; ++c) dp[c] += __shfl_xor(dp[c], 32);
            if (valid && h == 0) {
                a.d_pos[3 * i + 0] += dp[0]; a.d_pos[3 * i + 1] += dp[1]; a.d_pos[3 * i + 2] += dp[2];
            }
        }
        // ---- second order: S sweep (reverse) and t sweep (forward mode), Theorem 1
        v16f s1[2];
        Split<2, 2> ps2;
        Split<1, 2> pt;
        last_row_masked(w.HLrow0, m_last, h, ps2);
        if (K == 3) {
            matvec_split<2, 4, 2, 2>(w.H2t, ps2, s1, lane);
            apply_mask<2>(s1, m1);
            split(s1, pd);
        } else {
            pd = ps2;
        }
        split(t0, pt);
        wave_lds_fence();
        stage_split(Zs, pd, j, h);
        stage_split(Xs, pt, j, h);
        wave_lds_fence();
        outer_accumulate_split<2, 1>(G1, Zs, Xs, lane);
        v16f t1[2], t2[2];
        matvec_split<2, KS1, 3, 2>(w.H1f, pt, t1, lane);
        apply_mask<2>(t1, m1);
        if (K == 3) {
            split(t1, pd);
            wave_lds_fence();
            stage_split(Zs, ps2, j, h);
            stage_split(Xs, pd, j, h);
            wave_lds_fence();
            outer_accumulate_split<2, 2>(G2, Zs, Xs, lane);
            matvec_split<2, 4, 3, 2>(w.H2f, pd, t2, lane);
            apply_mask<2>(t2, m_last);
            tsum[0] += t2[0]; tsum[1] += t2[1];
        } else {
            tsum[0] += t1[0]; tsum[1] += t1[1];
        }
        wave_lds_fence();
    }
    // S_K is the unit row selecting the SDF output: row 0 of the last matrix's gradient gets
    // the sum of t_{K-1} over points.  One outer product with a one-hot factor does the
    // cross-lane sum of the per-lane partials.
    {
        v16f onehot[1] = {zero16()};
        if (h == 0) onehot[0][0] = 1.f;
        stage<1, kLd64>(Zt, onehot, j, h);
        stage<2, kLd64>(Xt, tsum, j, h);
        wave_lds_fence();
        outer_accumulate16<2, kLd64, kLd64>(GL, Zt, Xt, lane);
    }
    __syncthreads();
    // ---- every wave gets a quarter of the registers of the block's sums and adds it to global
    // memory: one barrier, and the atomics of the four waves run side by side
    float* scratch = reinterpret_cast<float*>(&sm);
    constexpr int kVecs = K == 3 ? 7 : 3;
    static_assert(sizeof(sm) >= kWaves * kVecs * 1024 * sizeof(float), "scratch for the block sum");
    v16f gl;                   // the four 16-column blocks of GL side by side
#pragma unroll
    for (int cb = 0; cb < 4; ++cb)
#pragma unroll
        for (int v = 0; v < 4; ++v) gl[4 * cb + v] = GL[cb][v];
    constexpr int kShare = 16 / kWaves;
    if (K == 3) {
        v16f* all[7] = {&G1[0][0], &G1[1][0], &G2[0][0], &G2[0][1], &G2[1][0], &G2[1][1], &gl};
        block_sum_shared<kWaves, 7>(scratch, all, wave, lane);
        flush_grad<2, 2>(a.dH[1], 64, 64, G2, j, h, wave * kShare, kShare);
    } else {
        v16f* all[3] = {&G1[0][0], &G1[1][0], &gl};
        block_sum_shared<kWaves, 3>(scratch, all, wave, lane);
    }
    flush_grad<2, 1>(a.dH[0], 64, D, G1, j, h, wave * kShare, kShare);
    // register 4 cb + v of gl: row 4 (lane / 16) + v, column 16 cb + lane % 16 of the last matrix; a wave's
    // quarter is one block of 16 columns
#pragma unroll
    for (int cb = 0; cb < 4; ++cb)
#pragma unroll
        for (int v = 0; v < 4; ++v)
            if (cb == wave) atomicAdd(a.dH[K - 1] + (4 * (lane >> 4) + v) * 64 + 16 * cb + (lane & 15), gl[4 * cb + v]);
}

template <int D, int K>
int run_fwd(const SdfArgs& a, hipStream_t st) {
    const int64_t tiles = (a.n + 31) / 32;
    const int64_t want = (tiles + kFwdWaves - 1) / kFwdWaves;
    const int blocks = persistent_blocks((const void*)sdf_fwd_kernel<D, K>, kFwdThreads, want);
    hipLaunchKernelGGL((sdf_fwd_kernel<D, K>), dim3(blocks), dim3(kFwdThreads), 0, st, a);
    return check_launch("sdf forward");
}

template <int D, int K>
int run_bwd(const SdfArgs& a, hipStream_t st) {
    const int64_t tiles = (a.n + 31) / 32;
    const int64_t want = (tiles + kWaves - 1) / kWaves;
    if (a.masks) {
        const int blocks = persistent_blocks((const void*)sdf_bwd_kernel<D, K, true>, kThreads, want);
        hipLaunchKernelGGL((sdf_bwd_kernel<D, K, true>), dim3(blocks), dim3(kThreads), 0, st, a);
    } else {
        const int blocks = persistent_blocks((const void*)sdf_bwd_kernel<D, K, false>, kThreads, want);
        hipLaunchKernelGGL((sdf_bwd_kernel<D, K, false>), dim3(blocks), dim3(kThreads), 0, st, a);
    }
    return check_launch("sdf backward");
}

// ------------------------------------------------------------------------------------------
// Networks deeper than the fused kernels hold (up to eight hidden layers of 64: the depths of the
// paper's Fig. 7), layer by layer.  The fused kernels keep every matrix in LDS and every weight
// gradient in registers, which stops at two hidden layers; here ONE matrix is in LDS per launch
// and the per-point vectors pass from launch to launch through a workspace in HBM, each lane
// writing the 32 registers it holds as 128 consecutive bytes (vector v of point tile t, lane l:
// floats ((t * 64 + l) * 32 ...)).  Every matrix is used as 64 x 64 (the first one's missing
// columns and the last one's missing rows are zeros), so one kernel serves every layer.
//   forward launch l:  a_l = G_l H_l a_{l-1}  (six-product arithmetic, writes the mask word)
//                      t_l = G_l H_l t_{l-1}  (with WITH_T; t_0 = (de/dx) dL/dn)
//   reverse launch l:  dH_l += delta_l a_{l-1}^T + S_l^T t_{l-1}^T   (with GRAD)
//                      S_{l-1} = (H_l^T S_l) G_{l-1},  delta_{l-1} = G_{l-1} H_l^T delta_l
// with S_K = the unit row of the SDF output and delta_K = dL/d(d,g): Theorem 1 and Eqs. 7-8 as in
// the fused kernels, Definition 1's vectors one layer at a time.
struct DeepArgs {
    const float* W; int out_dim, in_dim;       // H_l [out_dim][in_dim], row-major
    int64_t n; int levels;                     // points; levels of the encoding (input width / 2)
    bool first, last;                          // l == 1, l == K
    const float* enc; const float* jac; const float* d_normal; const float* d_y;
    const float* a_in; const float* t_in; const float* s_in; const float* d_in;     // lane layout
    float* a_out; float* t_out; float* s_out; float* d_out;                         // lane layout
    float* a0_out; float* t0_out;              // forward, first layer: its inputs in lane layout, for the reverse launch
    uint32_t* mask_out; const uint32_t* mask_in;   // one word per lane: [tile * 64 + lane]
    float* y; float* q; float* normal; float* d_enc; float* dW;
};

__device__ __forceinline__ void load_lane(const float* __restrict__ base, int64_t tile, int lane, v16f* v) {
    const float4* p = reinterpret_cast<const float4*>(base + (tile * 64 + lane) * 32);
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const float4 f = p[4 * b + k];
            v[b][4 * k] = f.x; v[b][4 * k + 1] = f.y; v[b][4 * k + 2] = f.z; v[b][4 * k + 3] = f.w;
        }
}

__device__ __forceinline__ void store_lane(float* __restrict__ base, int64_t tile, int lane, const v16f* v) {
    float4* p = reinterpret_cast<float4*>(base + (tile * 64 + lane) * 32);
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
        for (int k = 0; k < 4; ++k) p[4 * b + k] = make_float4(v[b][4 * k], v[b][4 * k + 1], v[b][4 * k + 2], v[b][4 * k + 3]);
}

template <bool WITH_T>
__global__ __launch_bounds__(kThreads) void deep_forward_kernel(DeepArgs a) {
    typedef SplitMatrix<4, 3> M;
    __shared__ alignas(16) unsigned char Wf[64 * M::kLd];
    {
        typename M::template Fill<64, kThreads, false> f;
        const float* __restrict__ W = a.W;
        const int od = a.out_dim, id = a.in_dim;
        f.load(threadIdx.x, [&](int o, int i) { return (o < od && i < id) ? W[o * id + i] : 0.f; });
        f.store(Wf, threadIdx.x);
        __syncthreads();
    }
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int j = lane & 31, h = lane >> 5;
    const int64_t tiles = (a.n + 31) / 32;
    for (int64_t tile = (int64_t)blockIdx.x * kWaves + wave; tile < tiles; tile += (int64_t)gridDim.x * kWaves) {
        const int64_t i = tile * 32 + j;
        const bool valid = i < a.n;
        v16f x[2], z[2];
        if (a.first) {
            x[0] = load_levels<32>(a.enc, a.n, i, valid, a.levels, h);
            x[1] = zero16();
            if (a.a0_out) store_lane(a.a0_out, tile, lane, x);
        } else {
            load_lane(a.a_in, tile, lane, x);
        }
        Split<2, 3> px;
        split(x, px);
        matvec_split<2, 4, 3, 3>(Wf, px, z, lane);
        uint32_t m = 0xffffffffu;
        if (a.last) {
            store_rows16(a.y, i, valid, h, z[0]);
        } else {
            m = relu_mask<2>(z);
            store_lane(a.a_out, tile, lane, z);
            a.mask_out[tile * 64 + lane] = m;
        }
        if (WITH_T) {
            v16f t[2], tz[2];
            if (a.first) {
                float nb3[3] = {0.f, 0.f, 0.f};
                if (valid) { nb3[0] = a.d_normal[3 * i]; nb3[1] = a.d_normal[3 * i + 1]; nb3[2] = a.d_normal[3 * i + 2]; }
                t[0] = apply_jac<32>(a.jac, a.n, i, valid, a.levels, h, nb3);
                t[1] = zero16();
                store_lane(a.t0_out, tile, lane, t);
            } else {
                load_lane(a.t_in, tile, lane, t);
            }
            Split<2, 2> pt;
            split(t, pt);
            matvec_split<2, 4, 3, 2>(Wf, pt, tz, lane);
            apply_mask<2>(tz, m);
            store_lane(a.t_out, tile, lane, tz);
        }
    }
}

struct DeepRevSmem {
    alignas(16) unsigned char Wt[64 * SplitMatrix<4, 3>::kLd];
    float tiles[kWaves][2][kTileWords];
};

// P: terms per factor of the transposed products (3 where the result is dd/de, which is compared at
// forward tolerance; 2 in the backward call)
template <int P, bool GRAD>
__global__ __launch_bounds__(kThreads) void deep_reverse_kernel(DeepArgs a) {
    typedef SplitMatrix<4, P> M;
    __shared__ DeepRevSmem sm;
    {
        typename M::template Fill<64, kThreads, true> f;
        const float* __restrict__ W = a.W;
        const int od = a.out_dim, id = a.in_dim;
        f.load(threadIdx.x, [&](int i, int o) { return (o < od && i < id) ? W[o * id + i] : 0.f; });
        f.store(sm.Wt, threadIdx.x);
        __syncthreads();
    }
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int j = lane & 31, h = lane >> 5;
    uint32_t* Zs = reinterpret_cast<uint32_t*>(sm.tiles[wave][0]);
    uint32_t* Xs = reinterpret_cast<uint32_t*>(sm.tiles[wave][1]);
    v16f G[2][2];
#pragma unroll
    for (int mb = 0; mb < 2; ++mb) { G[mb][0] = zero16(); G[mb][1] = zero16(); }
    const int64_t tiles = (a.n + 31) / 32;
    for (int64_t tile = (int64_t)blockIdx.x * kWaves + wave; tile < tiles; tile += (int64_t)gridDim.x * kWaves) {
        const int64_t i = tile * 32 + j;
        const bool valid = i < a.n;
        v16f s[2], d[2];
        if (a.last) {
            // S_K: the unit row of output 0; delta_K: the adjoint of the 16 outputs
            s[0] = zero16(); s[1] = zero16(); d[1] = zero16();
            if (h == 0 && valid) s[0][0] = 1.f;
            if (GRAD) d[0] = load_rows16(a.d_y, i, valid, h);
        } else {
            load_lane(a.s_in, tile, lane, s);
            if (GRAD) load_lane(a.d_in, tile, lane, d);
        }
        Split<2, P> ps;
        Split<2, 2> pd;
        split(s, ps);
        if (GRAD) {
            v16f ap[2], tp[2];
            load_lane(a.a_in, tile, lane, ap);
            load_lane(a.t_in, tile, lane, tp);
            Split<2, 2> pa, pt;
            split(d, pd);
            split(ap, pa);
            split(tp, pt);
            stage_split(Zs, pd, j, h);
            stage_split(Xs, pa, j, h);
            wave_lds_fence();
            outer_accumulate_split<2, 2>(G, Zs, Xs, lane);
            wave_lds_fence();
            stage_split(Zs, ps, j, h);
            stage_split(Xs, pt, j, h);
            wave_lds_fence();
            outer_accumulate_split<2, 2>(G, Zs, Xs, lane);
            wave_lds_fence();
        }
        const uint32_t m = a.first ? 0xffffffffu : a.mask_in[tile * 64 + lane];
        v16f s2[2], d2[2];
        matvec_split<2, 4, P, P>(sm.Wt, ps, s2, lane);
        if (a.first) {
            // dd/de and the normal (Eq. 2); the levels of this lane are 4g + 2h + u
            if (a.q) {
#pragma unroll
                for (int g = 0; g < 4; ++g)
#pragma unroll
                    for (int u = 0; u < 2; ++u) {
                        const int level = 4 * g + 2 * h + u;
                        if (valid && level < a.levels)
                            reinterpret_cast<float2*>(a.q)[(int64_t)level * a.n + i] = make_float2(s2[0][4 * g + 2 * u], s2[0][4 * g + 2 * u + 1]);
                    }
                float nrm[3];
                contract_jac<32>(a.jac, a.n, i, valid, a.levels, h, s2[0], nrm);
#pragma unroll
                for (int c = 0; c < 3; ++c) nrm[c] += __shfl_xor(nrm[c], 32);
                if (valid && h == 0) { a.normal[3 * i] = nrm[0]; a.normal[3 * i + 1] = nrm[1]; a.normal[3 * i + 2] = nrm[2]; }
            }
        } else {
            apply_mask<2>(s2, m);
            store_lane(a.s_out, tile, lane, s2);
        }
        if (GRAD) {
            matvec_split<2, 4, P, 2>(sm.Wt, pd, d2, lane);
            if (a.first) {
#pragma unroll
                for (int g = 0; g < 4; ++g)
#pragma unroll
                    for (int u = 0; u < 2; ++u) {
                        const int level = 4 * g + 2 * h + u;
                        if (valid && level < a.levels)
                            reinterpret_cast<float2*>(a.d_enc)[(int64_t)level * a.n + i] = make_float2(d2[0][4 * g + 2 * u], d2[0][4 * g + 2 * u + 1]);
                    }
            } else {
                apply_mask<2>(d2, m);
                store_lane(a.d_out, tile, lane, d2);
            }
        }
    }
    if (GRAD) {
        __syncthreads();
        float* scratch = reinterpret_cast<float*>(&sm);
        static_assert(sizeof(sm) >= kWaves * 4 * 1024 * sizeof(float), "scratch for the block sum");
        v16f* all[4] = {&G[0][0], &G[0][1], &G[1][0], &G[1][1]};
        block_sum_shared<kWaves, 4>(scratch, all, wave, lane);
        constexpr int kShare = 16 / kWaves;
        flush_grad<2, 2>(a.dW, a.out_dim, a.in_dim, G, j, h, wave * kShare, kShare);
    }
}

SdfArgs base_args(const neus2_config* cfg, const float* enc, const float* jac, const float* const* H, int64_t n) {
    SdfArgs a = {};
    a.enc = enc; a.jac = jac; a.n = n; a.active_levels = cfg->active_levels;
    for (int l = 0; l < cfg->n_sdf_mats; ++l) a.H[l] = H[l];
    return a;
}

}  // namespace

int launch_sdf_fwd(const neus2_config* cfg, const float* enc, const float* jac, const float* const* H,
                   int64_t n, float* y, float* q, float* normal, uint32_t* masks, hipStream_t st) {
    if (n == 0) return NEUS2_OK;
    SdfArgs a = base_args(cfg, enc, jac, H, n);
    a.y = y; a.q = q; a.normal = normal; a.masks = masks;
    a.stream_q = n >= ((int64_t)1 << 20);
    const int D = cfg->sdf_dims[0], K = cfg->n_sdf_mats;
    if (D == 32 && K == 3) return run_fwd<32, 3>(a, st);
    if (D == 32 && K == 2) return run_fwd<32, 2>(a, st);
    if (D == 16 && K == 3) return run_fwd<16, 3>(a, st);
    if (D == 16 && K == 2) return run_fwd<16, 2>(a, st);
    return fail(NEUS2_ERR_UNSUPPORTED, "sdf network: input width %d with %d matrices has no kernel", D, K);
}

// Workspace of the layer-by-layer path: per point 32 floats per lane-layout vector (two lanes a
// point), for a_0..a_{K-1} and t_0..t_{K-1} (the backward call keeps them all for its reverse
// launches), two pairs of vectors that the reverse launches hand on, and a mask word per lane and
// hidden layer.
static int64_t deep_vector_floats(int64_t n) { return ((n + 31) / 32) * 64 * 32; }

int64_t sdf_deep_workspace_bytes(int n_mats, int64_t n) {
    const int64_t vec = deep_vector_floats(n) * 4, words = ((n + 31) / 32) * 64 * 4;
    return (2 * (int64_t)n_mats + 4) * vec + (int64_t)n_mats * words;
}

namespace {

struct DeepLayout {
    float* a[NEUS2_DEEP_MAX_MATS]; float* t[NEUS2_DEEP_MAX_MATS]; float* pass[4]; uint32_t* mask[NEUS2_DEEP_MAX_MATS];
};

DeepLayout deep_layout(void* workspace, int n_mats, int64_t n) {
    DeepLayout L;
    float* p = reinterpret_cast<float*>(workspace);
    const int64_t vec = deep_vector_floats(n);
    for (int l = 0; l < n_mats; ++l) { L.a[l] = p; p += vec; L.t[l] = p; p += vec; }
    for (int k = 0; k < 4; ++k) { L.pass[k] = p; p += vec; }
    uint32_t* w = reinterpret_cast<uint32_t*>(p);
    for (int l = 0; l < n_mats; ++l) { L.mask[l] = w; w += ((n + 31) / 32) * 64; }
    return L;
}

int deep_dims(int n_mats, int enc_dim, int l, int& out_dim, int& in_dim) {
    in_dim = l == 0 ? enc_dim : 64;
    out_dim = l == n_mats - 1 ? 16 : 64;
    return 0;
}

template <typename Kernel>
void deep_launch(Kernel kernel, const DeepArgs& a, hipStream_t st) {
    const int64_t want = ((a.n + 31) / 32 + kWaves - 1) / kWaves;
    const int blocks = persistent_blocks((const void*)kernel, kThreads, want);
    hipLaunchKernelGGL(kernel, dim3(blocks), dim3(kThreads), 0, st, a);
}

}  // namespace

int launch_sdf_deep_fwd(int n_mats, int enc_dim, const float* enc, const float* jac, const float* const* H, int64_t n,
                        float* y, float* q, float* normal, void* workspace, hipStream_t st) {
    if (n == 0) return NEUS2_OK;
    const DeepLayout L = deep_layout(workspace, n_mats, n);
    for (int l = 0; l < n_mats; ++l) {                           // forward launches: a_1 .. a_{K-1}, y
        DeepArgs a = {};
        a.W = H[l]; deep_dims(n_mats, enc_dim, l, a.out_dim, a.in_dim);
        a.n = n; a.levels = enc_dim / 2; a.first = l == 0; a.last = l == n_mats - 1;
        a.enc = enc; a.a_in = L.a[l]; a.a_out = L.a[(l + 1) % n_mats]; a.mask_out = L.mask[l]; a.y = y;
        deep_launch(deep_forward_kernel<false>, a, st);
    }
    for (int l = n_mats - 1; l >= 0; --l) {                      // reverse launches: S_{K-1} .. S_1, dd/de
        DeepArgs a = {};
        a.W = H[l]; deep_dims(n_mats, enc_dim, l, a.out_dim, a.in_dim);
        a.n = n; a.levels = enc_dim / 2; a.first = l == 0; a.last = l == n_mats - 1;
        a.s_in = L.pass[l & 1]; a.s_out = L.pass[(l & 1) ^ 1];
        a.mask_in = l > 0 ? L.mask[l - 1] : nullptr;
        a.jac = jac; a.q = q; a.normal = normal;
        deep_launch(deep_reverse_kernel<3, false>, a, st);
    }
    return check_launch("sdf forward (layer by layer)");
}

int launch_sdf_deep_bwd(int n_mats, int enc_dim, const float* enc, const float* jac, const float* const* H,
                        const float* d_y, const float* d_normal, int64_t n, float* const* dH, float* d_enc,
                        void* workspace, hipStream_t st) {
    if (n == 0) return NEUS2_OK;
    const DeepLayout L = deep_layout(workspace, n_mats, n);
    for (int l = 0; l + 1 < n_mats; ++l) {                       // a_l and t_l of every hidden layer
        DeepArgs a = {};
        a.W = H[l]; deep_dims(n_mats, enc_dim, l, a.out_dim, a.in_dim);
        a.n = n; a.levels = enc_dim / 2; a.first = l == 0; a.last = false;
        a.enc = enc; a.jac = jac; a.d_normal = d_normal;
        a.a0_out = L.a[0]; a.t0_out = L.t[0];
        a.a_in = L.a[l]; a.t_in = L.t[l]; a.a_out = L.a[l + 1]; a.t_out = L.t[l + 1]; a.mask_out = L.mask[l];
        deep_launch(deep_forward_kernel<true>, a, st);
    }
    for (int l = n_mats - 1; l >= 0; --l) {
        DeepArgs a = {};
        a.W = H[l]; deep_dims(n_mats, enc_dim, l, a.out_dim, a.in_dim);
        a.n = n; a.levels = enc_dim / 2; a.first = l == 0; a.last = l == n_mats - 1;
        a.d_y = d_y;
        a.s_in = L.pass[l & 1]; a.s_out = L.pass[(l & 1) ^ 1];
        a.d_in = L.pass[2 + (l & 1)]; a.d_out = L.pass[2 + ((l & 1) ^ 1)];
        a.a_in = L.a[l]; a.t_in = L.t[l];                        // a_{l-1}, t_{l-1} in the paper's numbering
        a.mask_in = l > 0 ? L.mask[l - 1] : nullptr;
        a.d_enc = d_enc; a.dW = dH[l];
        deep_launch(deep_reverse_kernel<2, true>, a, st);
    }
    return check_launch("sdf backward (layer by layer)");
}

int launch_sdf_bwd(const neus2_config* cfg, const float* enc, const float* jac, const float* const* H,
                   const float* d_y, const float* d_normal, int64_t n, float* const* dH, float* d_enc,
                   float* d_pos, const uint32_t* masks, hipStream_t st) {
    if (n == 0) return NEUS2_OK;
    SdfArgs a = base_args(cfg, enc, jac, H, n);
    a.d_y = d_y; a.d_normal = d_normal; a.d_enc = d_enc; a.d_pos = d_pos;
    a.stream_q = n >= ((int64_t)1 << 20);
    a.masks = const_cast<uint32_t*>(masks);              // the backward kernel only reads them
    for (int l = 0; l < cfg->n_sdf_mats; ++l) a.dH[l] = dH[l];
    const int D = cfg->sdf_dims[0], K = cfg->n_sdf_mats;
    if (D == 32 && K == 3) return run_bwd<32, 3>(a, st);
    if (D == 32 && K == 2) return run_bwd<32, 2>(a, st);
    if (D == 16 && K == 3) return run_bwd<16, 3>(a, st);
    if (D == 16 && K == 2) return run_bwd<16, 2>(a, st);
    return fail(NEUS2_ERR_UNSUPPORTED, "sdf network: input width %d with %d matrices has no kernel", D, K);
}

}  // namespace neus2
