// Colour network c = c_Upsilon(x, n, v, d, g) (Eq. 3 of the paper): forward and first-order
// backward, fused per 32-point tile on the matrix cores (fp32 values as sums of bf16 terms, see
// mfma_tile.h).  The paper needs no
// second-order term for Upsilon (text after Eq. 6): the normal enters here as a plain input
// and its adjoint dL/dn is handed on to the SDF backward.
//
// Input, as the caller sees it: [x(3), n(3), SH16(v)(16), (d,g)(16)] = 38 columns of W_1.
// Inside the kernel the columns are walked in the order [(d,g), x, n, 0, 0, SH16]: each lane's
// registers map to contiguous loads, and every column whose adjoint is wanted ((d,g), x, n;
// the view direction is not trained) lies in the first block of 32, so the backward pass
// computes only that block of dL/d(input).  W_1 is permuted to match when it is copied into
// LDS.
#include "common.h"
#include "mfma_tile.h"

namespace neus2 {

namespace {

constexpr int kThreads = 256;
constexpr int kWaves = kThreads / 64;

struct ColorArgs {
    const float* pos; const float* normal; const float* dirs; const int32_t* sample_ray; const float* y; const float* W[3];
    const float* d_rgb; const float* d_sdf; const float* rgb_in;
    float* rgb; float* dW[3]; float* d_y; float* d_normal; float* d_pos;
    uint32_t* masks;           // optional [2][n][2]: written by the forward kernel, read by the backward kernel
    int64_t n; int spr;
};

// The ReLU masks of a point as the kernels keep them: one word per hidden layer and lane half h,
// bit 16 b + r for neuron 32 b + neuron_of(r, h); word (layer * n + i) * 2 + h of the buffer.
__device__ __forceinline__ int64_t mask_word(int layer, int64_t n, int64_t i, int h) { return ((int64_t)layer * n + i) * 2 + h; }

// caller's column of W_1 for internal column c (or -1 for padding)
__device__ __forceinline__ int external_column(int c) {
    if (c < 16) return 22 + c;          // (d, g)
    if (c < 22) return c - 16;          // x (0..2), n (3..5)
    if (c < 24) return -1;
    return 6 + (c - 24);                // SH16
}

// The matrices live in LDS split into bf16 terms (see mfma_tile.h).  The forward pass, in the
// forward kernel and where the backward kernel recomputes it, uses three terms per factor and six
// products: as accurate as fp32 arithmetic, and the same arithmetic in both kernels, so the ReLU
// masks agree.  The adjoint sweep of the backward kernel uses two terms and three products.
template <bool BWD>
struct ColorWeights {
    typedef SplitMatrix<3, 3> M1f;     // [64][40 -> 48]
    typedef SplitMatrix<4, 3> M2f;     // [64][64]
    typedef SplitMatrix<4, 2> M1t;     // [first 32 input columns][64]
    typedef SplitMatrix<4, 2> M2t;
    typedef SplitMatrix<1, 2> M3t;     // [64][3 -> 16]
    alignas(16) unsigned char W1f[64 * M1f::kLd];
    alignas(16) unsigned char W2f[64 * M2f::kLd];
    // The last matrix [3][64] in fp32, as a lane holds its point's activations: W3r[h][o][16 b + r] is
    // column 32 b + neuron_of(r, h) of row o (forward kernel only; the backward pass reads rgb).
    alignas(16) float W3r[BWD ? 1 : 2][3][32];
    alignas(16) unsigned char W1t[BWD ? 32 * M1t::kLd : 16];
    alignas(16) unsigned char W2t[BWD ? 64 * M2t::kLd : 16];
    alignas(16) unsigned char W3t[BWD ? 64 * M3t::kLd : 16];
};

// Every matrix is fetched from global memory before the first is written to LDS, so the fetches
// are in flight together; the copies cover every slot a product reads, so nothing is cleared.
template <bool BWD>
__device__ void load_weights(ColorWeights<BWD>& w, const ColorArgs& a) {
    typedef ColorWeights<BWD> W;
    const int tid = threadIdx.x;
    const float* __restrict__ W1 = a.W[0];
    const float* __restrict__ W2 = a.W[1];
    const float* __restrict__ W3 = a.W[2];
    auto first = [&](int o, int c) {
        const int e = c < 40 ? external_column(c) : -1;
        return e >= 0 ? W1[o * 38 + e] : 0.f;
    };
    typename W::M1f::template Fill<64, kThreads, false> f1;
    typename W::M2f::template Fill<64, kThreads, false> f2;
    typename W::M1t::template Fill<BWD ? 32 : 0, kThreads, true> t1;
    typename W::M2t::template Fill<BWD ? 64 : 0, kThreads, true> t2;
    typename W::M3t::template Fill<BWD ? 64 : 0, kThreads, true> t3;
    f1.load(tid, first);
    f2.load(tid, [&](int o, int i) { return W2[o * 64 + i]; });
    float last = 0.f;
    const int lh = tid / 96, lo = (tid / 32) % 3, lk = tid % 32;          // tid < 192: one element of W3r
    if (!BWD && tid < 192) last = W3[lo * 64 + 32 * (lk >> 4) + neuron_of(lk & 15, lh)];
    t1.load(tid, [&](int c, int o) { return first(o, c); });
    t2.load(tid, [&](int i, int o) { return W2[o * 64 + i]; });
    t3.load(tid, [&](int i, int o) { return o < 3 ? W3[o * 64 + i] : 0.f; });
    f1.store(w.W1f, tid);
    f2.store(w.W2f, tid);
    if (!BWD && tid < 192) w.W3r[lh][lo][lk] = last;
    t1.store(w.W1t, tid);
    t2.store(w.W2t, tid);
    t3.store(w.W3t, tid);
    __syncthreads();
}

// real orthonormal spherical harmonics, degree 0..3, index l*l + l + m
__device__ __forceinline__ void sh16(float x, float y, float z, float* sh) {
    const float xx = x * x, yy = y * y, zz = z * z;
    sh[0] = 0.28209479177387814f;
    sh[1] = 0.4886025119029199f * y;
    sh[2] = 0.4886025119029199f * z;
    sh[3] = 0.4886025119029199f * x;
    sh[4] = 1.0925484305920792f * x * y;
    sh[5] = 1.0925484305920792f * y * z;
    sh[6] = 0.31539156525252005f * (3.f * zz - 1.f);
    sh[7] = 1.0925484305920792f * x * z;
    sh[8] = 0.5462742152960396f * (xx - yy);
    sh[9] = 0.5900435899266435f * y * (3.f * xx - yy);
    sh[10] = 2.890611442640554f * x * y * z;
    sh[11] = 0.4570457994644658f * y * (5.f * zz - 1.f);
    sh[12] = 0.3731763325901154f * z * (5.f * zz - 3.f);
    sh[13] = 0.4570457994644658f * x * (5.f * zz - 1.f);
    sh[14] = 1.445305721320277f * z * (xx - yy);
    sh[15] = 0.5900435899266435f * x * (xx - 3.f * yy);
}

// One point's inputs as they sit in memory; loaded one tile ahead so that HBM latency hides
// behind the matrix work of the current tile.
struct ColorRaw {
    float4 ya, yb;
    float dir[3], p[3], nr[3];
    float d_rgb[3], rgb[3], d_sdf;
    float dn[2];               // backward: this lane's part of d_normal as it comes in (h = 0: n0; h = 1: n1, n2)
    uint32_t m1, m2;           // backward with masks from the forward kernel
};

template <bool BWD>
__device__ __forceinline__ ColorRaw load_raw(const ColorArgs& a, int64_t i, bool valid, int h) {
    ColorRaw r = {};
    if (!valid) return r;
    r.ya = *reinterpret_cast<const float4*>(a.y + i * 16 + 4 * h);
    r.yb = *reinterpret_cast<const float4*>(a.y + i * 16 + 8 + 4 * h);
    // n is at most 2^28: a 32-bit division (the 64-bit one costs over a hundred instructions)
    const int64_t ray = a.sample_ray ? (int64_t)a.sample_ray[i] : (int64_t)((uint32_t)i / (uint32_t)a.spr);
#pragma unroll
    for (int c = 0; c < 3; ++c) {
        r.dir[c] = a.dirs[3 * ray + c];
        r.p[c] = a.pos[3 * i + c];
        r.nr[c] = a.normal[3 * i + c];
        if (BWD) { r.d_rgb[c] = a.d_rgb[3 * i + c]; r.rgb[c] = a.rgb_in[3 * i + c]; }
    }
    if (BWD && a.d_sdf) r.d_sdf = a.d_sdf[i];
    if (BWD && a.masks) { r.m1 = __builtin_nontemporal_load(a.masks + mask_word(0, a.n, i, h)); r.m2 = __builtin_nontemporal_load(a.masks + mask_word(1, a.n, i, h)); }
    if (BWD) {
        r.dn[0] = a.d_normal[3 * i + (h ? 1 : 0)];
        if (h) r.dn[1] = a.d_normal[3 * i + 2];
    }
    return r;
}

// Build the register layout from the raw inputs: block 0 = [(d,g), x, n, 0, 0, SH 0..7],
// block 1 = [SH 8..15].
__device__ __forceinline__ void build_input(const ColorRaw& r, bool valid, int h, v16f* cin) {
    cin[0] = zero16();
    cin[1] = zero16();
    if (!valid) return;
    cin[0][0] = r.ya.x; cin[0][1] = r.ya.y; cin[0][2] = r.ya.z; cin[0][3] = r.ya.w;
    cin[0][4] = r.yb.x; cin[0][5] = r.yb.y; cin[0][6] = r.yb.z; cin[0][7] = r.yb.w;
    float sh[16];
    sh16(r.dir[0], r.dir[1], r.dir[2], sh);
    cin[0][8] = h ? r.nr[1] : r.p[0];
    cin[0][9] = h ? r.nr[2] : r.p[1];
    cin[0][10] = h ? 0.f : r.p[2];
    cin[0][11] = h ? 0.f : r.nr[0];
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        cin[0][12 + k] = h ? sh[4 + k] : sh[k];
        cin[1][k] = h ? sh[12 + k] : sh[8 + k];
    }
}

__device__ __forceinline__ float sigmoid(float u) { return 1.f / (1.f + __expf(-u)); }

// Both hidden layers; leaves the split input and first hidden layer behind for the backward
// pass's weight gradients.
template <bool BWD, bool GIVEN>
__device__ __forceinline__ void forward_tile(const ColorWeights<BWD>& w, const v16f* cin, Split<2, GIVEN ? 2 : 3>& pc,
                                             Split<2, GIVEN ? 2 : 3>& p1, v16f* a2, uint32_t& m1, uint32_t& m2, int lane) {
    constexpr int PF = GIVEN ? 2 : 3;
    v16f a1[2];
    split(cin, pc);
    matvec_split<2, 3, 3, PF>(w.W1f, pc, a1, lane);
    if (GIVEN) apply_mask<2>(a1, m1);
    else m1 = relu_mask<2>(a1);
    split(a1, p1);
    matvec_split<2, 4, 3, PF>(w.W2f, p1, a2, lane);
    if (GIVEN) apply_mask<2>(a2, m2);
    else m2 = relu_mask<2>(a2);
}

__global__ __launch_bounds__(kThreads, 2) void color_fwd_kernel(ColorArgs a) {
    __shared__ ColorWeights<false> w;
    load_weights<false>(w, a);
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // the same for all lanes: keeps tile indices and addresses scalar
    const int j = lane & 31, h = lane >> 5;
    const int64_t tiles = (a.n + 31) / 32;
    const int64_t stride = (int64_t)gridDim.x * kWaves;
    int64_t tile = (int64_t)blockIdx.x * kWaves + wave;
    ColorRaw next = load_raw<false>(a, tile * 32 + j, tile < tiles && tile * 32 + j < a.n, h);
    for (; tile < tiles; tile += stride) {
        const int64_t i = tile * 32 + j;
        const bool valid = i < a.n;
        v16f cin[2], a2[2];
        uint32_t m1, m2;
        Split<2, 3> pc, p1;
        build_input(next, valid, h, cin);
        {
            const int64_t in = (tile + stride) * 32 + j;
            next = load_raw<false>(a, in, tile + stride < tiles && in < a.n, h);
        }
        forward_tile<false, false>(w, cin, pc, p1, a2, m1, m2, lane);
        if (a.masks && valid) {
            a.masks[mask_word(0, a.n, i, h)] = m1;
            a.masks[mask_word(1, a.n, i, h)] = m2;
        }
        // Last layer, three outputs: fp32 dot products of this lane's 32 activations with its part
        // of each row, and one cross-lane add for the other half of the point.  As a matrix product
        // it would take the split of a2 and 24 matrix instructions for 3 rows of 32.
        float u[3] = {0.f, 0.f, 0.f};
#pragma unroll
        for (int o = 0; o < 3; ++o)
#pragma unroll
            for (int q4 = 0; q4 < 8; ++q4) {
                const float4 wv = *reinterpret_cast<const float4*>(&w.W3r[h][o][4 * q4]);
                const v16f& act = a2[q4 >> 2];
                const int r = 4 * (q4 & 3);
                u[o] += wv.x * act[r] + wv.y * act[r + 1] + wv.z * act[r + 2] + wv.w * act[r + 3];
            }
#pragma unroll
        for (int o = 0; o < 3; ++o) u[o] += __shfl_xor(u[o], 32);
        if (valid && h == 0) {
            a.rgb[3 * i + 0] = sigmoid(u[0]);
            a.rgb[3 * i + 1] = sigmoid(u[1]);
            a.rgb[3 * i + 2] = sigmoid(u[2]);
        }
    }
}

struct ColorBwdSmem {
    ColorWeights<true> w;
    float tiles[kWaves][2][kTileWords];
};

// GIVEN: the masks come from the forward kernel (a.masks).  The forward pass is then recomputed
// only for its values, which enter weight gradients and further products at gradient tolerance:
// two terms and three products like the rest of this kernel.  Without them it is recomputed in
// the forward kernel's own arithmetic, which yields the same masks bit for bit.
template <bool GIVEN>
__global__ __launch_bounds__(kThreads) void color_bwd_kernel(ColorArgs a) {
    __shared__ ColorBwdSmem sm;
    ColorWeights<true>& w = sm.w;
    load_weights<true>(w, a);
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // the same for all lanes: keeps tile indices and addresses scalar
    const int j = lane & 31, h = lane >> 5;
    float* Zt = sm.tiles[wave][0];
    float* Xt = sm.tiles[wave][1];
    uint32_t* Zs = reinterpret_cast<uint32_t*>(Zt);     // the same tiles in the transposed split layout
    uint32_t* Xs = reinterpret_cast<uint32_t*>(Xt);
    v16f G1[2][2], G2[2][2];
    v4f G3[4];                 // gradient of the last matrix (3 of 16 rows used): four blocks of 16 columns
#pragma unroll
    for (int mb = 0; mb < 2; ++mb)
#pragma unroll
        for (int nb = 0; nb < 2; ++nb) { G1[mb][nb] = zero16(); G2[mb][nb] = zero16(); }
#pragma unroll
    for (int cb = 0; cb < 4; ++cb) G3[cb] = v4f{0.f, 0.f, 0.f, 0.f};

    const int64_t tiles = (a.n + 31) / 32;
    const int64_t stride = (int64_t)gridDim.x * kWaves;
    int64_t tile = (int64_t)blockIdx.x * kWaves + wave;
    ColorRaw next = load_raw<true>(a, tile * 32 + j, tile < tiles && tile * 32 + j < a.n, h);
    for (; tile < tiles; tile += stride) {
        const int64_t i = tile * 32 + j;
        const bool valid = i < a.n;
        v16f cin[2], a2[2];
        const ColorRaw cur = next;
        uint32_t m1 = cur.m1, m2 = cur.m2;
        build_input(cur, valid, h, cin);
        {
            const int64_t in = (tile + stride) * 32 + j;
            next = load_raw<true>(a, in, tile + stride < tiles && in < a.n, h);
        }
        // ---- forward pass again
        Split<2, GIVEN ? 2 : 3> pc, p1;
        forward_tile<true, GIVEN>(w, cin, pc, p1, a2, m1, m2, lane);
        // adjoint of the pre-sigmoid output, from the colour the forward pass stored
        v16f d3[1] = {zero16()};
        if (valid && h == 0) {
#pragma unroll
            for (int c = 0; c < 3; ++c) d3[0][c] = cur.d_rgb[c] * cur.rgb[c] * (1.f - cur.rgb[c]);
        }
        stage<1, kLd64>(Zt, d3, j, h);
        stage<2, kLd64>(Xt, a2, j, h);
        wave_lds_fence();
        outer_accumulate16<2, kLd64, kLd64>(G3, Zt, Xt, lane);
        // ---- adjoint sweep: two terms, three products
        v16f d2[2], d1[2], dcin[1];
        Split<1, 2> p3;
        Split<2, 2> pd;
        split(d3, p3);
        matvec_split<2, 1, 2, 2>(w.W3t, p3, d2, lane);
        apply_mask<2>(d2, m2);
        split(d2, pd);
        wave_lds_fence();
        stage_split(Zs, pd, j, h);
        stage_split(Xs, p1, j, h);
        wave_lds_fence();
        outer_accumulate_split<2, 2>(G2, Zs, Xs, lane);
        matvec_split<2, 4, 2, 2>(w.W2t, pd, d1, lane);
        apply_mask<2>(d1, m1);
        split(d1, pd);
        wave_lds_fence();
        stage_split(Zs, pd, j, h);
        stage_split(Xs, pc, j, h);
        wave_lds_fence();
        outer_accumulate_split<2, 2>(G1, Zs, Xs, lane);
        matvec_split<1, 4, 2, 2>(w.W1t, pd, dcin, lane);
        wave_lds_fence();
        if (valid) {
            // block 0, registers 0..7: dL/d(d,g) columns 4h..4h+3 and 8+4h..8+4h+3
            float4 lo = make_float4(dcin[0][0], dcin[0][1], dcin[0][2], dcin[0][3]);
            const float4 hi = make_float4(dcin[0][4], dcin[0][5], dcin[0][6], dcin[0][7]);
            if (h == 0) lo.x += cur.d_sdf;
            *reinterpret_cast<float4*>(a.d_y + i * 16 + 4 * h) = lo;
            *reinterpret_cast<float4*>(a.d_y + i * 16 + 8 + 4 * h) = hi;
            // registers 8..11: h = 0 -> x0 x1 x2 n0 ; h = 1 -> n1 n2
            if (h == 0) {
                if (a.d_pos) { a.d_pos[3 * i] = dcin[0][8]; a.d_pos[3 * i + 1] = dcin[0][9]; a.d_pos[3 * i + 2] = dcin[0][10]; }
                a.d_normal[3 * i] = cur.dn[0] + dcin[0][11];
            } else {
                a.d_normal[3 * i + 1] = cur.dn[0] + dcin[0][8];
                a.d_normal[3 * i + 2] = cur.dn[1] + dcin[0][9];
            }
        }
    }
    __syncthreads();
    // ---- every wave gets a quarter of the registers of the block's sums and adds it to global
    // memory: one barrier, and the atomics of the four waves run side by side
    float* scratch = reinterpret_cast<float*>(&sm);
    static_assert(sizeof(sm) >= kWaves * 9 * 1024 * sizeof(float), "scratch for the block sum");
    v16f g3;                   // the four 16-column blocks of G3 side by side
#pragma unroll
    for (int cb = 0; cb < 4; ++cb)
#pragma unroll
        for (int v = 0; v < 4; ++v) g3[4 * cb + v] = G3[cb][v];
    v16f* all[9] = {&G1[0][0], &G1[0][1], &G1[1][0], &G1[1][1], &G2[0][0], &G2[0][1], &G2[1][0], &G2[1][1], &g3};
    block_sum_shared<kWaves, 9>(scratch, all, wave, lane);
    constexpr int kShare = 16 / kWaves;
#pragma unroll
    for (int mb = 0; mb < 2; ++mb)
#pragma unroll
        for (int nb = 0; nb < 2; ++nb)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                if (r / kShare != wave) continue;
                const int o = 32 * mb + neuron_of(r, h), c = 32 * nb + j;
                atomicAdd(a.dW[1] + o * 64 + c, G2[mb][nb][r]);
                const int e = external_column(c);
                if (e >= 0) atomicAdd(a.dW[0] + o * 38 + e, G1[mb][nb][r]);
            }
    if (lane < 16) {           // rows 0..3 of a block live in lanes 0..15; three of them are real
#pragma unroll
        for (int cb = 0; cb < 4; ++cb)
#pragma unroll
            for (int v = 0; v < 3; ++v)
                if (cb == wave) atomicAdd(a.dW[2] + v * 64 + 16 * cb + lane, g3[4 * cb + v]);
    }
}

int check_common(const neus2_config* cfg, const float* pos, const float* normal, const float* dirs,
                 const int32_t* sample_ray, const float* y, const float* const* W, int64_t n) {
    NEUS2_TRY(check_config(cfg));
    if (cfg->n_color_mats != 3) return fail(NEUS2_ERR_CONFIG, "the descriptor has no colour network");
    if (n < 0 || n > ((int64_t)1 << 28)) return fail(NEUS2_ERR_SHAPE, "n = %lld out of range", (long long)n);
    if (!sample_ray && n % cfg->samples_per_ray != 0)
        return fail(NEUS2_ERR_SHAPE, "n = %lld is not a multiple of samples_per_ray = %d", (long long)n, cfg->samples_per_ray);
    NEUS2_TRY(check_ptr(pos, "pos"));
    NEUS2_TRY(check_ptr(normal, "normal"));
    NEUS2_TRY(check_ptr(dirs, "dirs"));
    NEUS2_TRY(check_ptr(y, "y"));
    if (!W) return fail(NEUS2_ERR_NULL, "W is NULL");
    for (int l = 0; l < 3; ++l) NEUS2_TRY(check_ptr(W[l], "W[l]"));
    return NEUS2_OK;
}

}  // namespace

}  // namespace neus2

using namespace neus2;

extern "C" {

int neus2_color_fwd(const neus2_config* cfg, const float* pos, const float* normal, const float* dirs,
                    const int32_t* sample_ray, const float* y, const float* const* W, int64_t n, float* rgb,
                    uint32_t* masks, void* stream) {
    NEUS2_TRY(check_common(cfg, pos, normal, dirs, sample_ray, y, W, n));
    NEUS2_TRY(check_ptr(rgb, "rgb"));
    NEUS2_TRY(check_ptr(masks, "masks", false));
    if (n == 0) return NEUS2_OK;
    ColorArgs a = {};
    a.pos = pos; a.normal = normal; a.dirs = dirs; a.sample_ray = sample_ray; a.y = y; a.rgb = rgb; a.n = n; a.masks = masks;
    a.spr = cfg->samples_per_ray;
    for (int l = 0; l < 3; ++l) a.W[l] = W[l];
    const int blocks = persistent_blocks((const void*)color_fwd_kernel, kThreads, ((n + 31) / 32 + kWaves - 1) / kWaves);
    hipLaunchKernelGGL(color_fwd_kernel, dim3(blocks), dim3(kThreads), 0, (hipStream_t)stream, a);
    return check_launch("colour forward");
}

int neus2_color_bwd(const neus2_config* cfg, const float* pos, const float* normal, const float* dirs,
                    const int32_t* sample_ray, const float* y, const float* const* W, const float* rgb, const float* d_rgb, const float* d_sdf, int64_t n,
                    float* const* dW, float* d_y, float* d_normal, float* d_pos, const uint32_t* masks, void* stream) {
    NEUS2_TRY(check_common(cfg, pos, normal, dirs, sample_ray, y, W, n));
    NEUS2_TRY(check_ptr(rgb, "rgb"));
    NEUS2_TRY(check_ptr(d_rgb, "d_rgb"));
    NEUS2_TRY(check_ptr(d_sdf, "d_sdf", false));
    if (!dW) return fail(NEUS2_ERR_NULL, "dW is NULL");
    for (int l = 0; l < 3; ++l) NEUS2_TRY(check_ptr(dW[l], "dW[l]"));
    NEUS2_TRY(check_ptr(d_y, "d_y"));
    NEUS2_TRY(check_ptr(d_normal, "d_normal"));
    NEUS2_TRY(check_ptr(d_pos, "d_pos", false));
    NEUS2_TRY(check_ptr(masks, "masks", false));
    if (n == 0) return NEUS2_OK;
    ColorArgs a = {};
    a.masks = const_cast<uint32_t*>(masks);              // the backward kernel only reads them
    a.pos = pos; a.normal = normal; a.dirs = dirs; a.sample_ray = sample_ray; a.y = y; a.n = n; a.spr = cfg->samples_per_ray;
    a.rgb_in = rgb; a.d_rgb = d_rgb; a.d_sdf = d_sdf; a.d_y = d_y; a.d_normal = d_normal; a.d_pos = d_pos;
    for (int l = 0; l < 3; ++l) { a.W[l] = W[l]; a.dW[l] = dW[l]; }
    const int64_t want = ((n + 31) / 32 + kWaves - 1) / kWaves;
    if (masks) {
        const int blocks = persistent_blocks((const void*)color_bwd_kernel<true>, kThreads, want);
        hipLaunchKernelGGL(color_bwd_kernel<true>, dim3(blocks), dim3(kThreads), 0, (hipStream_t)stream, a);
    } else {
        const int blocks = persistent_blocks((const void*)color_bwd_kernel<false>, kThreads, want);
        hipLaunchKernelGGL(color_bwd_kernel<false>, dim3(blocks), dim3(kThreads), 0, (hipStream_t)stream, a);
    }
    return check_launch("colour backward");
}

}  // extern "C"
