// NeuS compositing along rays as wavefront scans, the loss of Eq. 4, Adam, and the rigid
// transform of Eq. 9.
//
// Paper, supplement Sec. E.3: Phi_s(x) = 1/(1+e^{-sx});
//   alpha_i = max((Phi_s(d_i) - Phi_s(d_{i+1})) / Phi_s(d_i), 0),  T_i = prod_{j<i}(1-alpha_j),
//   C = sum_i T_i alpha_i c_i.
// The quotient is evaluated in the algebraically identical form
//   (1 - Phi_s(d_{i+1})) * (1 - exp(-s (d_i - d_{i+1}))),
// which has no cancellation when both SDF values are close to zero (fp32).
//
// One ray = one wavefront, one sample = one lane (at most 64 samples per ray).
#include <cstring>

#include "common.h"

namespace neus2 {

namespace {

constexpr int kRayThreads = 256;

struct RayLane {
    float alpha, trans, dalpha_di, dalpha_dnext;   // dalpha_i/dd_i and dalpha_i/dd_{i+1}
};

__device__ __forceinline__ float shfl_down1(float v) { return __shfl_down(v, 1); }

// 1 - alpha as a divisor.  In binary32 alpha rounds to exactly 1 once s (d_i - d_{i+1}) and
// -s d_{i+1} both pass about 17; every later transmittance is then 0 and the quotient
// (sum over later samples) / (1 - alpha) would be 0/0.  Both derivatives of alpha are exactly 0 in
// that case (1 - e^{-s delta} = 1 and Phi_s(d_{i+1}) = 0 after rounding), so any finite quotient
// gives the exact adjoint 0; 2^-24 is half the spacing of floats below 1, the smallest 1 - alpha
// that can occur otherwise.
__device__ __forceinline__ float guarded_one_minus(float alpha) { return fmaxf(1.f - alpha, 5.9604645e-8f); }

// inclusive product scan over the wave
__device__ __forceinline__ float wave_scan_mul(float v, int lane) {
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const float o = __shfl_up(v, d);
        if (lane >= d) v *= o;
    }
    return v;
}

// inclusive suffix-sum scan over the wave (lane i gets sum over lanes >= i)
__device__ __forceinline__ float wave_suffix_sum(float v, int lane) {
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const float o = __shfl_down(v, d);
        if (lane + d < 64) v += o;
    }
    return v;
}

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) v += __shfl_xor(v, d);
    return v;
}

__device__ __forceinline__ RayLane ray_lane(float d, int lane, int spr, float s) {
    const float dn = shfl_down1(d);
    RayLane r = {0.f, 1.f, 0.f, 0.f};
    if (lane < spr - 1) {
        const float delta = d - dn;
        if (delta > 0.f) {
            const float one_minus_phi_n = 1.f / (1.f + __expf(s * dn));   // 1 - Phi_s(d_{i+1})
            const float phi_n = 1.f - one_minus_phi_n;
            const float em = -expm1f(-s * delta);                           // 1 - e^{-s delta}
            const float e = 1.f - em;
            r.alpha = one_minus_phi_n * em;
            r.dalpha_di = one_minus_phi_n * s * e;
            r.dalpha_dnext = -s * phi_n * one_minus_phi_n * em - r.dalpha_di;
        }
    }
    const float incl = wave_scan_mul(1.f - r.alpha, lane);
    const float excl = __shfl_up(incl, 1);
    r.trans = lane == 0 ? 1.f : excl;
    return r;
}

__global__ __launch_bounds__(kRayThreads) void render_fwd_kernel(const float* __restrict__ sdf, int64_t stride,
                                                                const float* __restrict__ rgb, int64_t rays, int spr,
                                                                float s, const float* __restrict__ s_dev,
                                                                float* __restrict__ C, float* __restrict__ weights) {
    const int lane = threadIdx.x & 63;
    const int64_t ray = (int64_t)blockIdx.x * (kRayThreads / 64) + (threadIdx.x >> 6);
    if (ray >= rays) return;
    if (s_dev) s = *s_dev;
    const bool live = lane < spr;
    const int64_t i = ray * spr + (live ? lane : 0);
    const float d = live ? sdf[i * stride] : 0.f;
    const RayLane r = ray_lane(d, lane, spr, s);
    const float w = live ? r.trans * r.alpha : 0.f;
    float c0 = 0.f, c1 = 0.f, c2 = 0.f;
    if (live) {
        weights[i] = w;
        c0 = w * rgb[3 * i + 0]; c1 = w * rgb[3 * i + 1]; c2 = w * rgb[3 * i + 2];
    }
    c0 = wave_sum(c0); c1 = wave_sum(c1); c2 = wave_sum(c2);
    if (lane == 0) { C[3 * ray + 0] = c0; C[3 * ray + 1] = c1; C[3 * ray + 2] = c2; }
}

// dC/dalpha_i = T_i (dC.c_i) - (sum_{j>i} T_j alpha_j (dC.c_j)) / (1 - alpha_i)
// The slope s (learnable, supplement Sec. E.3) enters alpha only through the products s d_i, so
// dL/ds = (1/s) sum_i d_i dL/dd_i: one wave sum on top of the SDF gradient.
__global__ __launch_bounds__(kRayThreads) void render_bwd_kernel(const float* __restrict__ sdf, int64_t stride,
                                                                const float* __restrict__ rgb,
                                                                const float* __restrict__ dC, int64_t rays, int spr,
                                                                float s, const float* __restrict__ s_dev,
                                                                float* __restrict__ d_sdf,
                                                                float* __restrict__ d_rgb, float* __restrict__ d_s) {
    const int lane = threadIdx.x & 63;
    const int64_t ray = (int64_t)blockIdx.x * (kRayThreads / 64) + (threadIdx.x >> 6);
    if (ray >= rays) return;
    if (s_dev) s = *s_dev;
    const bool live = lane < spr;
    const int64_t i = ray * spr + (live ? lane : 0);
    const float d = live ? sdf[i * stride] : 0.f;
    const RayLane r = ray_lane(d, lane, spr, s);
    const float w = live ? r.trans * r.alpha : 0.f;
    const float g0 = dC[3 * ray + 0], g1 = dC[3 * ray + 1], g2 = dC[3 * ray + 2];
    float cb = 0.f;
    if (live) {
        cb = g0 * rgb[3 * i + 0] + g1 * rgb[3 * i + 1] + g2 * rgb[3 * i + 2];
        d_rgb[3 * i + 0] = w * g0; d_rgb[3 * i + 1] = w * g1; d_rgb[3 * i + 2] = w * g2;
    }
    const float wc = w * cb;
    const float after = wave_suffix_sum(wc, lane) - wc;          // sum over j > i
    const float d_alpha = r.trans * cb - after / guarded_one_minus(r.alpha);
    const float from_prev = __shfl_up(d_alpha * r.dalpha_dnext, 1);
    float ds = d_alpha * r.dalpha_di;
    if (lane > 0) ds += from_prev;
    if (live) d_sdf[i] = ds;
    if (d_s) {
        const float t = wave_sum(live ? ds * d : 0.f);
        if (lane == 0) atomicAdd(d_s, t / s);
    }
}

// ---- loss ---------------------------------------------------------------------------------
__device__ __forceinline__ void block_add(float v, float* dst, float* red) {
    v = wave_sum(v);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    if (lane == 0) red[wave] = v;
    __syncthreads();
    if (threadIdx.x == 0) {
        float t = 0.f;
        for (int k = 0; k < (int)(blockDim.x >> 6); ++k) t += red[k];
        atomicAdd(dst, t);
    }
    __syncthreads();
}

// N sums per workgroup, added to N neighbouring floats by N lanes of ONE atomic instruction: the
// memory side merges lanes that fall into the same cache line into one request, and requests
// to one line are applied one after the other (about 12 ns each), so this costs a workgroup
// one request where one call of block_add per value costs N.
template <int N>
__device__ __forceinline__ void block_add_n(const float (&v)[N], float* dst, float* red) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, waves = blockDim.x >> 6;
#pragma unroll
    for (int k = 0; k < N; ++k) {
        const float t = wave_sum(v[k]);
        if (lane == 0) red[wave * N + k] = t;
    }
    __syncthreads();
    if (threadIdx.x < N) {
        float t = 0.f;
        for (int w = 0; w < waves; ++w) t += red[w * N + threadIdx.x];
        atomicAdd(dst + threadIdx.x, t);
    }
    __syncthreads();
}

// Grid-stride with few, large workgroups: every workgroup ends in an atomic on one cache line,
// and those are applied one after the other by the memory side (about 12 ns each, which is
// what this kernel's time was made of with a thousand workgroups).
constexpr int kLossThreads = 1024;

__global__ __launch_bounds__(kLossThreads) void loss_kernel(int kind, const float* __restrict__ C, const float* __restrict__ target,
                                                   const float* __restrict__ normal, const float* __restrict__ y,
                                                   int64_t rays, int64_t n, float beta, float huber_delta,
                                                   float* __restrict__ loss,
                                                   float* __restrict__ dC, float* __restrict__ d_normal,
                                                   float* __restrict__ d_y) {
    __shared__ float red[2 * kLossThreads / 64];
    const float inv_n = 1.f / (float)n;
    float first = 0.f, eik = 0.f;
    for (int64_t i = (int64_t)blockIdx.x * kLossThreads + threadIdx.x; i < n; i += (int64_t)gridDim.x * kLossThreads) {
        const float nx = normal[3 * i], ny = normal[3 * i + 1], nz = normal[3 * i + 2];
        const float len = sqrtf(nx * nx + ny * ny + nz * nz);
        const float dev = len - 1.f;
        eik += beta * dev * dev * inv_n;
        const float k = 2.f * beta * inv_n * dev / fmaxf(len, 1e-30f);
        d_normal[3 * i] = k * nx; d_normal[3 * i + 1] = k * ny; d_normal[3 * i + 2] = k * nz;
        if (kind == 0) {
            const float d = y[16 * i];
            first += d * d * inv_n;
            float4* o = reinterpret_cast<float4*>(d_y + 16 * i);
            o[0] = make_float4(2.f * d * inv_n, 0.f, 0.f, 0.f);
            o[1] = o[2] = o[3] = make_float4(0.f, 0.f, 0.f, 0.f);
        }
    }
    if (kind != 0) {
        const float inv_r = 1.f / (float)rays;
        for (int64_t i = (int64_t)blockIdx.x * kLossThreads + threadIdx.x; i < rays; i += (int64_t)gridDim.x * kLossThreads) {
#pragma unroll
            for (int c = 0; c < 3; ++c) {
                const float diff = C[3 * i + c] - target[3 * i + c];
                const float a = fabsf(diff);
                if (kind == 1) {
                    first += a * inv_r;
                    dC[3 * i + c] = diff > 0.f ? inv_r : (diff < 0.f ? -inv_r : 0.f);
                } else {   // Huber: quadratic up to delta, linear beyond
                    first += (a <= huber_delta ? 0.5f * diff * diff : huber_delta * (a - 0.5f * huber_delta)) * inv_r;
                    dC[3 * i + c] = fminf(fmaxf(diff, -huber_delta), huber_delta) * inv_r;
                }
            }
        }
    }
    const float both[2] = {first, eik};
    block_add_n<2>(both, loss, red);
}

// ---- compositing, loss and the backward of both for one ray per wavefront, in one kernel ----
// What render_fwd_kernel, loss_kernel and render_bwd_kernel do one after the other; a ray's
// samples stay in registers in between.  Wavefronts walk the rays with a grid stride and keep
// their share of the two loss terms in registers, so a workgroup ends in two atomics.
constexpr int kFusedThreads = 1024;

__global__ __launch_bounds__(kFusedThreads) void render_loss_kernel(int kind, const float* __restrict__ y,
                                                                   const float* __restrict__ rgb,
                                                                   const float* __restrict__ normal,
                                                                   const float* __restrict__ target, int64_t rays, int spr,
                                                                   float s, const float* __restrict__ s_dev, float beta,
                                                                   float huber_delta, float* __restrict__ C,
                                                                   float* __restrict__ weights, float* __restrict__ loss,
                                                                   float* __restrict__ dC, float* __restrict__ d_sdf,
                                                                   float* __restrict__ d_rgb, float* __restrict__ d_normal,
                                                                   float* __restrict__ d_s) {
    __shared__ float red[2 * kFusedThreads / 64];
    const int lane = threadIdx.x & 63;
    const int64_t waves = (int64_t)gridDim.x * (kFusedThreads / 64);
    if (s_dev) s = *s_dev;
    const float inv_r = 1.f / (float)rays;
    const float inv_n = 1.f / ((float)rays * (float)spr);
    const bool live = lane < spr;
    float first = 0.f, eik = 0.f, ds_total = 0.f;
    // the inputs of a wavefront's next ray are requested before the current one is worked on
    struct In { float d, c0, c1, c2, nx, ny, nz, t0, t1, t2; };
    auto load = [&](int64_t ray) {
        In in = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
        if (ray < rays) {
            const int64_t i = ray * spr + (live ? lane : 0);
            if (live) {
                in.d = y[16 * i];
                in.c0 = rgb[3 * i]; in.c1 = rgb[3 * i + 1]; in.c2 = rgb[3 * i + 2];
                in.nx = normal[3 * i]; in.ny = normal[3 * i + 1]; in.nz = normal[3 * i + 2];
            }
            in.t0 = target[3 * ray]; in.t1 = target[3 * ray + 1]; in.t2 = target[3 * ray + 2];
        }
        return in;
    };
    int64_t ray = (int64_t)blockIdx.x * (kFusedThreads / 64) + (threadIdx.x >> 6);
    In next = load(ray);
    for (; ray < rays; ray += waves) {
        const int64_t i = ray * spr + (live ? lane : 0);
        const In cur = next;
        next = load(ray + waves);
        const float d = cur.d, c0 = cur.c0, c1 = cur.c1, c2 = cur.c2, nx = cur.nx, ny = cur.ny, nz = cur.nz;
        const float t0 = cur.t0, t1 = cur.t1, t2 = cur.t2;
        // eikonal term and its adjoint
        if (live) {
            const float len = sqrtf(nx * nx + ny * ny + nz * nz);
            const float dev = len - 1.f;
            eik += beta * dev * dev * inv_n;
            const float k = 2.f * beta * inv_n * dev / fmaxf(len, 1e-30f);
            d_normal[3 * i] = k * nx; d_normal[3 * i + 1] = k * ny; d_normal[3 * i + 2] = k * nz;
        }
        // compositing
        const RayLane r = ray_lane(d, lane, spr, s);
        const float w = live ? r.trans * r.alpha : 0.f;
        const float C0 = wave_sum(w * c0), C1 = wave_sum(w * c1), C2 = wave_sum(w * c2);
        if (live) weights[i] = w;
        // colour term and dL/dC
        float g[3];
        const float diff[3] = {C0 - t0, C1 - t1, C2 - t2};
#pragma unroll
        for (int c = 0; c < 3; ++c) {
            const float a = fabsf(diff[c]);
            if (kind == 1) {
                if (lane == 0) first += a * inv_r;
                g[c] = diff[c] > 0.f ? inv_r : (diff[c] < 0.f ? -inv_r : 0.f);
            } else {
                if (lane == 0) first += (a <= huber_delta ? 0.5f * diff[c] * diff[c] : huber_delta * (a - 0.5f * huber_delta)) * inv_r;
                g[c] = fminf(fmaxf(diff[c], -huber_delta), huber_delta) * inv_r;
            }
        }
        if (lane == 0) {
            C[3 * ray] = C0; C[3 * ray + 1] = C1; C[3 * ray + 2] = C2;
            dC[3 * ray] = g[0]; dC[3 * ray + 1] = g[1]; dC[3 * ray + 2] = g[2];
        }
        // backward of the compositing
        float cb = 0.f;
        if (live) {
            cb = g[0] * c0 + g[1] * c1 + g[2] * c2;
            d_rgb[3 * i] = w * g[0]; d_rgb[3 * i + 1] = w * g[1]; d_rgb[3 * i + 2] = w * g[2];
        }
        const float wc = w * cb;
        const float after = wave_suffix_sum(wc, lane) - wc;
        const float d_alpha = r.trans * cb - after / guarded_one_minus(r.alpha);
        const float from_prev = __shfl_up(d_alpha * r.dalpha_dnext, 1);
        float ds = d_alpha * r.dalpha_di;
        if (lane > 0) ds += from_prev;
        if (live) { d_sdf[i] = ds; ds_total += ds * d; }
    }
    const float both[2] = {first, eik};
    block_add_n<2>(both, loss, red);
    if (d_s) block_add(ds_total / s, d_s, red);
}

// ---- the same for rays with their own sample counts ------------------------------------------
// Ray r owns samples offsets[r] .. offsets[r+1]-1 (what an occupancy-grid ray marcher produces,
// supplement Sec. E.3).  One wavefront per ray walks the ray in chunks of 64 samples: forwards
// for T, C and the loss (the transmittance at the start of chunk k is kept in lane k of one
// register), then backwards for the adjoints, carrying the sum over later samples.
struct AlphaTerms {
    float alpha, dalpha_di, dalpha_dnext;
};

__device__ __forceinline__ AlphaTerms alpha_terms(float d, float dn, bool has_next, float s) {
    AlphaTerms r = {0.f, 0.f, 0.f};
    const float delta = d - dn;
    if (has_next && delta > 0.f) {
        const float one_minus_phi_n = 1.f / (1.f + __expf(s * dn));
        const float phi_n = 1.f - one_minus_phi_n;
        const float em = -expm1f(-s * delta);
        const float e = 1.f - em;
        r.alpha = one_minus_phi_n * em;
        r.dalpha_di = one_minus_phi_n * s * e;
        r.dalpha_dnext = -s * phi_n * one_minus_phi_n * em - r.dalpha_di;
    }
    return r;
}

// product of (1 - alpha) over the 64 samples from `first` (samples at or beyond `end` count as 1)
__device__ __forceinline__ float chunk_transmittance(const float* __restrict__ y, int64_t first, int64_t end, int lane, float s) {
    const int64_t i = first + lane;
    float one_minus = 1.f;
    if (i + 1 < end) one_minus = 1.f - alpha_terms(y[16 * i], y[16 * (i + 1)], true, s).alpha;
    return __shfl(wave_scan_mul(one_minus, lane), 63);
}

__global__ __launch_bounds__(kFusedThreads) void render_loss_ragged_kernel(
    int kind, const float* __restrict__ y, const float* __restrict__ rgb, const float* __restrict__ normal,
    const float* __restrict__ target, const int32_t* __restrict__ offsets, int64_t rays, int64_t n, float s,
    const float* __restrict__ s_dev, float beta, float huber_delta, float* __restrict__ C, float* __restrict__ weights,
    float* __restrict__ loss, float* __restrict__ dC, float* __restrict__ d_sdf, float* __restrict__ d_rgb,
    float* __restrict__ d_normal, float* __restrict__ d_s) {
    __shared__ float red[2 * kFusedThreads / 64];
    const int lane = threadIdx.x & 63;
    const int64_t waves = (int64_t)gridDim.x * (kFusedThreads / 64);
    if (s_dev) s = *s_dev;
    const float inv_r = 1.f / (float)rays;
    const float inv_n = 1.f / (float)n;
    float first = 0.f, eik = 0.f, ds_total = 0.f;
    for (int64_t ray = (int64_t)blockIdx.x * (kFusedThreads / 64) + (threadIdx.x >> 6); ray < rays; ray += waves) {
        const int64_t begin = offsets[ray], end = offsets[ray + 1];
        const int64_t chunks = (end - begin + 63) / 64;
        // ---- forwards
        float t_carry = 1.f, t_start = 1.f, C0 = 0.f, C1 = 0.f, C2 = 0.f;
        for (int64_t c = 0; c < chunks; ++c) {
            const int64_t i = begin + 64 * c + lane;
            const bool live = i < end, has_next = i + 1 < end;
            float d = 0.f, dn = 0.f, c0 = 0.f, c1 = 0.f, c2 = 0.f;
            if (live) {
                d = y[16 * i];
                c0 = rgb[3 * i]; c1 = rgb[3 * i + 1]; c2 = rgb[3 * i + 2];
                const float nx = normal[3 * i], ny = normal[3 * i + 1], nz = normal[3 * i + 2];
                const float len = sqrtf(nx * nx + ny * ny + nz * nz);
                const float dev = len - 1.f;
                eik += beta * dev * dev * inv_n;
                const float k = 2.f * beta * inv_n * dev / fmaxf(len, 1e-30f);
                d_normal[3 * i] = k * nx; d_normal[3 * i + 1] = k * ny; d_normal[3 * i + 2] = k * nz;
            }
            if (has_next) dn = y[16 * (i + 1)];
            const AlphaTerms a = alpha_terms(d, dn, has_next, s);
            if (c < 64 && lane == (int)c) t_start = t_carry;
            const float incl = wave_scan_mul(1.f - a.alpha, lane);
            const float excl = __shfl_up(incl, 1);
            const float trans = t_carry * (lane == 0 ? 1.f : excl);
            const float w = live ? trans * a.alpha : 0.f;
            if (live) weights[i] = w;
            C0 += wave_sum(w * c0); C1 += wave_sum(w * c1); C2 += wave_sum(w * c2);
            t_carry *= __shfl(incl, 63);
        }
        // ---- colour term and dL/dC
        float g[3];
        const float diff[3] = {C0 - target[3 * ray], C1 - target[3 * ray + 1], C2 - target[3 * ray + 2]};
#pragma unroll
        for (int c = 0; c < 3; ++c) {
            const float a = fabsf(diff[c]);
            if (kind == 1) {
                if (lane == 0) first += a * inv_r;
                g[c] = diff[c] > 0.f ? inv_r : (diff[c] < 0.f ? -inv_r : 0.f);
            } else {
                if (lane == 0) first += (a <= huber_delta ? 0.5f * diff[c] * diff[c] : huber_delta * (a - 0.5f * huber_delta)) * inv_r;
                g[c] = fminf(fmaxf(diff[c], -huber_delta), huber_delta) * inv_r;
            }
        }
        if (lane == 0) {
            C[3 * ray] = C0; C[3 * ray + 1] = C1; C[3 * ray + 2] = C2;
            dC[3 * ray] = g[0]; dC[3 * ray + 1] = g[1]; dC[3 * ray + 2] = g[2];
        }
        // ---- backwards
        float after_carry = 0.f, pending = 0.f;          // pending: dL/dd of the first sample of the chunk after this one,
        for (int64_t c = chunks - 1; c >= 0; --c) {      // still without the term from this chunk's last sample
            const int64_t base = begin + 64 * c;
            const int64_t i = base + lane;
            const bool live = i < end, has_next = i + 1 < end;
            float d = 0.f, dn = 0.f, c0 = 0.f, c1 = 0.f, c2 = 0.f;
            if (live) { d = y[16 * i]; c0 = rgb[3 * i]; c1 = rgb[3 * i + 1]; c2 = rgb[3 * i + 2]; }
            if (has_next) dn = y[16 * (i + 1)];
            const AlphaTerms a = alpha_terms(d, dn, has_next, s);
            float t_chunk;
            if (c < 64) {
                t_chunk = __shfl(t_start, (int)c);
            } else {                                     // rays beyond 4096 samples: walk on from chunk 63
                t_chunk = __shfl(t_start, 63);
                for (int64_t k = 63; k < c; ++k) t_chunk *= chunk_transmittance(y, begin + 64 * k, end, lane, s);
            }
            const float incl = wave_scan_mul(1.f - a.alpha, lane);
            const float excl = __shfl_up(incl, 1);
            const float trans = t_chunk * (lane == 0 ? 1.f : excl);
            const float w = live ? trans * a.alpha : 0.f;
            float cb = 0.f;
            if (live) {
                cb = g[0] * c0 + g[1] * c1 + g[2] * c2;
                d_rgb[3 * i] = w * g[0]; d_rgb[3 * i + 1] = w * g[1]; d_rgb[3 * i + 2] = w * g[2];
            }
            const float wc = w * cb;
            const float after = wave_suffix_sum(wc, lane) - wc + after_carry;
            const float d_alpha = trans * cb - after / guarded_one_minus(a.alpha);
            const float to_next = d_alpha * a.dalpha_dnext;
            float ds = d_alpha * a.dalpha_di;
            const float from_prev = __shfl_up(to_next, 1);
            if (lane > 0) ds += from_prev;
            ds_total += d_alpha * (a.dalpha_di * d + a.dalpha_dnext * dn);
            if (c + 1 < chunks && lane == 63) d_sdf[base + 64] = pending + to_next;
            pending = __shfl(ds, 0);
            if (live && (lane > 0 || c == 0)) d_sdf[i] = ds;
            after_carry += wave_sum(wc);
        }
    }
    const float both[2] = {first, eik};
    block_add_n<2>(both, loss, red);
    if (d_s) block_add(ds_total / s, d_s, red);
}

__global__ void zero_kernel(float* p, int64_t count) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < count) p[i] = 0.f;
}

// ---- Adam ---------------------------------------------------------------------------------
struct AdamArgs {
    float lr, b1, b2, eps, inv_c1, inv_c2;    // inv_c = 1 / (1 - beta^t)
};

// flags: bit 0 clears the gradient, bit 1 skips entries whose gradient is exactly zero (their value
// and moments stay as they are: the "lazy" form for parameters that most steps do not touch)
constexpr int kAdamClear = 1, kAdamLazy = 2, kAdamActiveLevels = 4;

__device__ __forceinline__ float adam_one(float g, float& mi, float& vi, float p, const AdamArgs& a) {
    mi = a.b1 * mi + (1.f - a.b1) * g;
    vi = a.b2 * vi + (1.f - a.b2) * g * g;
    return p - a.lr * (mi * a.inv_c1) / (sqrtf(vi * a.inv_c2) + a.eps);
}

template <bool HALF>
__global__ __launch_bounds__(256) void adam_kernel(void* __restrict__ param, float* __restrict__ master,
                                                   float* __restrict__ grad, float* __restrict__ m,
                                                   float* __restrict__ v, int64_t count, AdamArgs a, int flags) {
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= count) return;
    const float g = grad[i];
    if ((flags & kAdamLazy) && g == 0.f) return;
    float mi = m[i], vi = v[i];
    float* full = HALF ? master : reinterpret_cast<float*>(param);
    const float p = adam_one(g, mi, vi, full[i], a);
    m[i] = mi;
    v[i] = vi;
    full[i] = p;
    if (HALF) reinterpret_cast<__half*>(param)[i] = __float2half_rn(p);
    if (flags & kAdamClear) grad[i] = 0.f;
}

// The same update over the hash tables [L][T][F], restricted to the slots a level can address:
// a dense level uses (res+1)^3 of its T slots, the others never receive a gradient, keep zero
// moments and would be left unchanged by the update, so skipping them changes nothing.  Four
// parameters per thread (16-byte accesses; a level starts on a 16-byte boundary); in the lazy form
// a thread whose four gradients are zero stops after reading them.
struct TableLevels {
    uint32_t used[NEUS2_MAX_LEVELS];     // parameters (slots * F) of each level that can be addressed
};

// A flat fp32 parameter buffer updated by the same launch (count 0: none).
struct AdamExtra {
    float* param; float* grad; float* m; float* v;
    int64_t count;
};

// 16-byte accesses with the non-temporal hint: data that is not read again soon
__device__ __forceinline__ float4 stream_load(const float* p) {
    typedef float f4 __attribute__((ext_vector_type(4)));
    const f4 v = __builtin_nontemporal_load(reinterpret_cast<const f4*>(p));
    return make_float4(v.x, v.y, v.z, v.w);
}
__device__ __forceinline__ void stream_store(float* p, const float4& v) {
    typedef float f4 __attribute__((ext_vector_type(4)));
    __builtin_nontemporal_store(f4{v.x, v.y, v.z, v.w}, reinterpret_cast<f4*>(p));
}

template <bool HALF>
__global__ __launch_bounds__(256) void adam_tables_kernel(void* __restrict__ param, float* __restrict__ master,
                                                          float* __restrict__ grad, float* __restrict__ m,
                                                          float* __restrict__ v, TableLevels lv, uint32_t per_level,
                                                          AdamArgs a, int flags, AdamExtra extra) {
    if (blockIdx.y == gridDim.y - 1 && extra.count > 0) {
        // last row of workgroups: the flat fp32 buffer that rides along (the networks' matrices), dense form
        for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < extra.count; i += (int64_t)gridDim.x * 256) {
            float mi = extra.m[i], vi = extra.v[i];
            extra.param[i] = adam_one(extra.grad[i], mi, vi, extra.param[i], a);
            extra.m[i] = mi;
            extra.v[i] = vi;
            if (flags & kAdamClear) extra.grad[i] = 0.f;
        }
        return;
    }
    const int level = blockIdx.y;
    const uint32_t k = (blockIdx.x * 256u + threadIdx.x) * 4u;
    const uint32_t used = lv.used[level];
    if (k >= used) return;
    const int64_t i = (int64_t)level * per_level + k;
    float* full = HALF ? master : reinterpret_cast<float*>(param);
    const bool lazy = flags & kAdamLazy;
    if (k + 4u <= used) {
        // Gradient, moments and the fp32 values are pure streams (read once, written once, not touched
        // again before the next update): they are moved with non-temporal accesses, which leaves the
        // caches to the fp16 tables this kernel writes and the next encode reads (measured: 73 us of a
        // 2.37 ms step at 2^21 entries a level, 8 us of 0.585 ms at 2^19).
        const float4 g = stream_load(grad + i);
        if (lazy && g.x == 0.f && g.y == 0.f && g.z == 0.f && g.w == 0.f) return;
        float4 mi = stream_load(m + i), vi = stream_load(v + i);
        float4 p = stream_load(full + i);
        if (!(lazy && g.x == 0.f)) p.x = adam_one(g.x, mi.x, vi.x, p.x, a);
        if (!(lazy && g.y == 0.f)) p.y = adam_one(g.y, mi.y, vi.y, p.y, a);
        if (!(lazy && g.z == 0.f)) p.z = adam_one(g.z, mi.z, vi.z, p.z, a);
        if (!(lazy && g.w == 0.f)) p.w = adam_one(g.w, mi.w, vi.w, p.w, a);
        stream_store(m + i, mi);
        stream_store(v + i, vi);
        if (HALF) {
            stream_store(full + i, p);
            __half2* h = reinterpret_cast<__half2*>(reinterpret_cast<__half*>(param) + i);
            const __half2 h0 = __floats2half2_rn(p.x, p.y), h1 = __floats2half2_rn(p.z, p.w);
            *reinterpret_cast<uint2*>(h) = make_uint2(*reinterpret_cast<const uint32_t*>(&h0), *reinterpret_cast<const uint32_t*>(&h1));
        } else {
            *reinterpret_cast<float4*>(full + i) = p;         // fp32 tables: these are what the encode reads
        }
        if (flags & kAdamClear) stream_store(grad + i, make_float4(0.f, 0.f, 0.f, 0.f));
    } else {
        for (uint32_t e = 0; e < used - k; ++e) {            // the last, partial group of a level
            const float g = grad[i + e];
            if (lazy && g == 0.f) continue;
            float mi = m[i + e], vi = v[i + e];
            const float p = adam_one(g, mi, vi, full[i + e], a);
            m[i + e] = mi;
            v[i + e] = vi;
            full[i + e] = p;
            if (HALF) reinterpret_cast<__half*>(param)[i + e] = __float2half_rn(p);
            if (flags & kAdamClear) grad[i + e] = 0.f;
        }
    }
}

// ---- rigid transform (Eq. 9) ---------------------------------------------------------------
struct Rigid {
    float R[9], T[3], scale, offset;
};

// DEV: rotation and translation are read from device memory (pose[0..8] = R row-major,
// pose[9..11] = T), where neus2_pose_update keeps them; otherwise they arrive by value.
template <bool DEV>
__global__ __launch_bounds__(256) void rigid_fwd_kernel(const float* __restrict__ pos, Rigid t, const float* __restrict__ pose,
                                                        int64_t n, float* __restrict__ out) {
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= n) return;
    if (DEV) {
#pragma unroll
        for (int k = 0; k < 9; ++k) t.R[k] = pose[k];
#pragma unroll
        for (int k = 0; k < 3; ++k) t.T[k] = pose[9 + k];
    }
    const float x = pos[3 * i] + t.T[0], y = pos[3 * i + 1] + t.T[1], z = pos[3 * i + 2] + t.T[2];
#pragma unroll
    for (int r = 0; r < 3; ++r) out[3 * i + r] = t.scale * (t.R[3 * r] * x + t.R[3 * r + 1] * y + t.R[3 * r + 2] * z) + t.offset;
}

constexpr int kRigidThreads = 1024;

template <bool DEV>
__global__ __launch_bounds__(kRigidThreads) void rigid_bwd_kernel(const float* __restrict__ pos, Rigid t, const float* __restrict__ pose,
                                                                 const float* __restrict__ d_out, int64_t n,
                                                                 float* __restrict__ Mb) {
    __shared__ float red[12 * kRigidThreads / 64];
    if (DEV) {
#pragma unroll
        for (int k = 0; k < 3; ++k) t.T[k] = pose[9 + k];
    }
    float acc[12];
#pragma unroll
    for (int k = 0; k < 12; ++k) acc[k] = 0.f;
    for (int64_t i = (int64_t)blockIdx.x * kRigidThreads + threadIdx.x; i < n; i += (int64_t)gridDim.x * kRigidThreads) {
        const float x[3] = {pos[3 * i] + t.T[0], pos[3 * i + 1] + t.T[1], pos[3 * i + 2] + t.T[2]};
#pragma unroll
        for (int r = 0; r < 3; ++r) {
            const float g = t.scale * d_out[3 * i + r];
            acc[3 * r + 0] += g * x[0]; acc[3 * r + 1] += g * x[1]; acc[3 * r + 2] += g * x[2];
            acc[9 + r] += g;
        }
    }
    block_add_n<12>(acc, Mb, red);
}

// ---- the six parameters of a frame's transform (Sec. 5, Eqs. 9-10) ----------------------------
// A frame's points reach the canonical space through x_c = R_prev (R(omega) (x + T) + T_prev):
// (R_prev, T_prev) is the transform accumulated over the earlier frames, (omega, T) the frame's
// own, R(omega) = exp([omega]_x).  That is one rigid map x_c = Rc (x + Tc) with Rc = R_prev R and
// Tc = T + R^T T_prev (the accumulation rule of the text after Eq. 10), which is what the
// transform kernels apply.  From their reductions M = sum g (x + Tc)^T and b = sum g:
//   sum g (x + T)^T = M - b (R^T T_prev)^T,   dL/dR = R_prev^T (that),   dL/dT = Rc^T b,
//   dL/domega_k = sum_ij (dR/domega_k)_ij (dL/dR)_ij.
// Twelve numbers in, six parameters out: one thread, in double precision (the derivative of
// Rodrigues' formula cancels badly in binary32 at the small angles of frame-to-frame motion).
struct Mat3 {
    double a[9];
};

__device__ inline Mat3 mat_mul(const Mat3& x, const Mat3& y) {
    Mat3 z;
    for (int i = 0; i < 3; ++i)
        for (int j = 0; j < 3; ++j) z.a[3 * i + j] = x.a[3 * i] * y.a[j] + x.a[3 * i + 1] * y.a[3 + j] + x.a[3 * i + 2] * y.a[6 + j];
    return z;
}

__device__ inline Mat3 skew(const double w[3]) {
    Mat3 k = {{0.0, -w[2], w[1], w[2], 0.0, -w[0], -w[1], w[0], 0.0}};
    return k;
}

// R = I + a K + b K^2, a = sin t / t, b = (1 - cos t) / t^2; da, db = (1/t) d/dt of a and b
__device__ inline void rodrigues_terms(double t2, double& a, double& b, double& da, double& db) {
    if (t2 < 1e-8) {                         // series: the closed forms are 0/0 at t = 0
        a = 1.0 - t2 / 6.0; b = 0.5 - t2 / 24.0; da = -1.0 / 3.0 + t2 / 30.0; db = -1.0 / 12.0 + t2 / 180.0;
    } else {
        const double t = sqrt(t2);
        a = sin(t) / t; b = (1.0 - cos(t)) / t2;
        da = (cos(t) - a) / t2; db = (a - 2.0 * b) / t2;
    }
}

__global__ void pose_update_kernel(float* __restrict__ param, float* __restrict__ m, float* __restrict__ v,
                                   const float* __restrict__ prev, float* __restrict__ Mb, float* __restrict__ pose,
                                   AdamArgs adam, int apply) {
    if (threadIdx.x != 0 || blockIdx.x != 0) return;
    double w[3] = {param[0], param[1], param[2]}, T[3] = {param[3], param[4], param[5]};
    Mat3 Rp;
    double Tp[3];
    for (int k = 0; k < 9; ++k) Rp.a[k] = prev[k];
    for (int k = 0; k < 3; ++k) Tp[k] = prev[9 + k];
    if (apply) {
        double a, b, da, db;
        rodrigues_terms(w[0] * w[0] + w[1] * w[1] + w[2] * w[2], a, b, da, db);
        const Mat3 K = skew(w), K2 = mat_mul(K, K);
        Mat3 R;
        for (int k = 0; k < 9; ++k) R.a[k] = (k % 4 == 0 ? 1.0 : 0.0) + a * K.a[k] + b * K2.a[k];
        double rtp[3], bs[3];                                  // R^T T_prev, b
        for (int j = 0; j < 3; ++j) rtp[j] = R.a[j] * Tp[0] + R.a[3 + j] * Tp[1] + R.a[6 + j] * Tp[2];
        for (int j = 0; j < 3; ++j) bs[j] = Mb[9 + j];
        Mat3 U;                                                // sum g (x + T)^T
        for (int i = 0; i < 3; ++i)
            for (int j = 0; j < 3; ++j) U.a[3 * i + j] = (double)Mb[3 * i + j] - bs[i] * rtp[j];
        Mat3 G;                                                // dL/dR = R_prev^T U
        for (int i = 0; i < 3; ++i)
            for (int j = 0; j < 3; ++j) G.a[3 * i + j] = Rp.a[i] * U.a[j] + Rp.a[3 + i] * U.a[3 + j] + Rp.a[6 + i] * U.a[6 + j];
        const Mat3 Rc = mat_mul(Rp, R);
        double grad[6];
        for (int k = 0; k < 3; ++k) {
            double e[3] = {0.0, 0.0, 0.0};
            e[k] = 1.0;
            const Mat3 E = skew(e), EK = mat_mul(E, K), KE = mat_mul(K, E);
            double acc = 0.0;
            for (int q = 0; q < 9; ++q) acc += (a * E.a[q] + b * (EK.a[q] + KE.a[q]) + w[k] * (da * K.a[q] + db * K2.a[q])) * G.a[q];
            grad[k] = acc;
        }
        for (int j = 0; j < 3; ++j) grad[3 + j] = Rc.a[j] * bs[0] + Rc.a[3 + j] * bs[1] + Rc.a[6 + j] * bs[2];   // Rc^T b
        for (int k = 0; k < 6; ++k) {
            const double mk = (double)adam.b1 * m[k] + (1.0 - (double)adam.b1) * grad[k];
            const double vk = (double)adam.b2 * v[k] + (1.0 - (double)adam.b2) * grad[k] * grad[k];
            const double p = (double)param[k] - (double)adam.lr * (mk * (double)adam.inv_c1) / (sqrt(vk * (double)adam.inv_c2) + (double)adam.eps);
            m[k] = (float)mk; v[k] = (float)vk; param[k] = (float)p;
        }
        for (int k = 0; k < 3; ++k) { w[k] = param[k]; T[k] = param[3 + k]; }      // the binary32 values the next step sees
    }
    // the composed transform the transform kernels apply from now on
    double a, b, da, db;
    rodrigues_terms(w[0] * w[0] + w[1] * w[1] + w[2] * w[2], a, b, da, db);
    const Mat3 K = skew(w), K2 = mat_mul(K, K);
    Mat3 R;
    for (int k = 0; k < 9; ++k) R.a[k] = (k % 4 == 0 ? 1.0 : 0.0) + a * K.a[k] + b * K2.a[k];
    const Mat3 Rc = mat_mul(Rp, R);
    for (int k = 0; k < 9; ++k) pose[k] = (float)Rc.a[k];
    for (int j = 0; j < 3; ++j) pose[9 + j] = (float)(T[j] + R.a[j] * Tp[0] + R.a[3 + j] * Tp[1] + R.a[6 + j] * Tp[2]);
    for (int k = 0; k < 12; ++k) Mb[k] = 0.f;
}

}  // namespace

}  // namespace neus2

using namespace neus2;

extern "C" {

int neus2_render_rays(const neus2_config* cfg, const float* sdf, int64_t sdf_stride, const float* rgb,
                      const float* s_dev, int64_t rays, float* C, float* weights, void* stream) {
    NEUS2_TRY(check_config(cfg));
    if (rays < 0 || rays > ((int64_t)1 << 28) / cfg->samples_per_ray) return fail(NEUS2_ERR_SHAPE, "rays = %lld out of range", (long long)rays);
    if (sdf_stride < 1) return fail(NEUS2_ERR_SHAPE, "sdf_stride = %lld, must be >= 1", (long long)sdf_stride);
    if (!sdf) return fail(NEUS2_ERR_NULL, "sdf is NULL");
    NEUS2_TRY(check_ptr(rgb, "rgb"));
    NEUS2_TRY(check_ptr(C, "C"));
    NEUS2_TRY(check_ptr(weights, "weights"));
    NEUS2_TRY(check_ptr(s_dev, "s_dev", false));
    if (rays == 0) return NEUS2_OK;
    const int per = kRayThreads / 64;
    hipLaunchKernelGGL(render_fwd_kernel, dim3((unsigned)((rays + per - 1) / per)), dim3(kRayThreads), 0,
                       (hipStream_t)stream, sdf, sdf_stride, rgb, rays, cfg->samples_per_ray, cfg->s, s_dev, C, weights);
    return check_launch("render rays");
}

int neus2_render_rays_bwd(const neus2_config* cfg, const float* sdf, int64_t sdf_stride, const float* rgb,
                          const float* dC, const float* s_dev, int64_t rays, float* d_sdf, float* d_rgb, float* d_s,
                          void* stream) {
    NEUS2_TRY(check_config(cfg));
    if (rays < 0 || rays > ((int64_t)1 << 28) / cfg->samples_per_ray) return fail(NEUS2_ERR_SHAPE, "rays = %lld out of range", (long long)rays);
    if (sdf_stride < 1) return fail(NEUS2_ERR_SHAPE, "sdf_stride = %lld, must be >= 1", (long long)sdf_stride);
    if (!sdf) return fail(NEUS2_ERR_NULL, "sdf is NULL");
    NEUS2_TRY(check_ptr(rgb, "rgb"));
    NEUS2_TRY(check_ptr(dC, "dC"));
    NEUS2_TRY(check_ptr(d_sdf, "d_sdf"));
    NEUS2_TRY(check_ptr(d_rgb, "d_rgb"));
    NEUS2_TRY(check_ptr(s_dev, "s_dev", false));
    NEUS2_TRY(check_ptr(d_s, "d_s", false));
    if (rays == 0) return NEUS2_OK;
    const int per = kRayThreads / 64;
    hipLaunchKernelGGL(render_bwd_kernel, dim3((unsigned)((rays + per - 1) / per)), dim3(kRayThreads), 0,
                       (hipStream_t)stream, sdf, sdf_stride, rgb, dC, rays, cfg->samples_per_ray, cfg->s, s_dev, d_sdf, d_rgb, d_s);
    return check_launch("render rays backward");
}

int neus2_loss(const neus2_config* cfg, const float* C, const float* target, const float* normal, const float* y,
               int64_t rays, int64_t n, float* loss, float* dC, float* d_normal, float* d_y, void* stream) {
    NEUS2_TRY(check_config(cfg));
    if (n < 0 || n > ((int64_t)1 << 28)) return fail(NEUS2_ERR_SHAPE, "n = %lld out of range", (long long)n);
    NEUS2_TRY(check_ptr(normal, "normal"));
    NEUS2_TRY(check_ptr(loss, "loss"));
    NEUS2_TRY(check_ptr(d_normal, "d_normal"));
    if (cfg->loss_kind != 0) {
        if (rays < 0 || rays * cfg->samples_per_ray != n)
            return fail(NEUS2_ERR_SHAPE, "rays * samples_per_ray = %lld differs from n = %lld",
                        (long long)(rays * cfg->samples_per_ray), (long long)n);
        NEUS2_TRY(check_ptr(C, "C"));
        NEUS2_TRY(check_ptr(target, "target"));
        NEUS2_TRY(check_ptr(dC, "dC"));
    } else {
        NEUS2_TRY(check_ptr(y, "y"));
        NEUS2_TRY(check_ptr(d_y, "d_y"));
    }
    if (n == 0) return NEUS2_OK;
    const int64_t want = (n + kLossThreads - 1) / kLossThreads;
    const int64_t cap = (int64_t)compute_units() / 2;
    hipLaunchKernelGGL(loss_kernel, dim3((unsigned)(want < cap ? want : cap)), dim3(kLossThreads), 0, (hipStream_t)stream, cfg->loss_kind,
                       C, target, normal, y, cfg->loss_kind != 0 ? rays : 0, n, cfg->beta, cfg->huber_delta, loss, dC, d_normal,
                       d_y);
    return check_launch("loss");
}

int neus2_render_loss_bwd(const neus2_config* cfg, const float* y, const float* rgb, const float* normal,
                          const float* target, const float* s_dev, int64_t rays, float* C, float* weights, float* loss,
                          float* dC, float* d_sdf, float* d_rgb, float* d_normal, float* d_s, void* stream) {
    NEUS2_TRY(check_config(cfg));
    if (cfg->loss_kind == 0) return fail(NEUS2_ERR_CONFIG, "loss_kind 0 has no colour term to composite for");
    if (rays < 0 || rays > ((int64_t)1 << 28) / cfg->samples_per_ray) return fail(NEUS2_ERR_SHAPE, "rays = %lld out of range", (long long)rays);
    NEUS2_TRY(check_ptr(y, "y"));
    NEUS2_TRY(check_ptr(rgb, "rgb"));
    NEUS2_TRY(check_ptr(normal, "normal"));
    NEUS2_TRY(check_ptr(target, "target"));
    NEUS2_TRY(check_ptr(s_dev, "s_dev", false));
    NEUS2_TRY(check_ptr(C, "C"));
    NEUS2_TRY(check_ptr(weights, "weights"));
    NEUS2_TRY(check_ptr(loss, "loss"));
    NEUS2_TRY(check_ptr(dC, "dC"));
    NEUS2_TRY(check_ptr(d_sdf, "d_sdf"));
    NEUS2_TRY(check_ptr(d_rgb, "d_rgb"));
    NEUS2_TRY(check_ptr(d_normal, "d_normal"));
    NEUS2_TRY(check_ptr(d_s, "d_s", false));
    if (rays == 0) return NEUS2_OK;
    const int per = kFusedThreads / 64;
    const int64_t want = (rays + per - 1) / per;
    const int64_t cap = (int64_t)compute_units() / 2;
    hipLaunchKernelGGL(render_loss_kernel, dim3((unsigned)(want < cap ? want : cap)), dim3(kFusedThreads), 0,
                       (hipStream_t)stream, cfg->loss_kind, y, rgb, normal, target, rays, cfg->samples_per_ray, cfg->s, s_dev,
                       cfg->beta, cfg->huber_delta, C, weights, loss, dC, d_sdf, d_rgb, d_normal, d_s);
    return check_launch("render + loss + backward");
}

int neus2_render_loss_bwd_ragged(const neus2_config* cfg, const float* y, const float* rgb, const float* normal,
                                 const float* target, const int32_t* ray_offsets, const float* s_dev, int64_t rays,
                                 int64_t n, float* C, float* weights, float* loss, float* dC, float* d_sdf, float* d_rgb,
                                 float* d_normal, float* d_s, void* stream) {
    NEUS2_TRY(check_config(cfg));
    if (cfg->loss_kind == 0) return fail(NEUS2_ERR_CONFIG, "loss_kind 0 has no colour term to composite for");
    if (rays < 0 || rays > ((int64_t)1 << 28)) return fail(NEUS2_ERR_SHAPE, "rays = %lld out of range", (long long)rays);
    if (n < 0 || n > ((int64_t)1 << 28)) return fail(NEUS2_ERR_SHAPE, "n = %lld out of range", (long long)n);
    if (!ray_offsets) return fail(NEUS2_ERR_NULL, "ray_offsets is NULL");
    NEUS2_TRY(check_ptr(target, "target"));
    NEUS2_TRY(check_ptr(s_dev, "s_dev", false));
    NEUS2_TRY(check_ptr(C, "C"));
    NEUS2_TRY(check_ptr(loss, "loss"));
    NEUS2_TRY(check_ptr(dC, "dC"));
    NEUS2_TRY(check_ptr(d_s, "d_s", false));
    if (n > 0) {
        NEUS2_TRY(check_ptr(y, "y"));
        NEUS2_TRY(check_ptr(rgb, "rgb"));
        NEUS2_TRY(check_ptr(normal, "normal"));
        NEUS2_TRY(check_ptr(weights, "weights"));
        NEUS2_TRY(check_ptr(d_sdf, "d_sdf"));
        NEUS2_TRY(check_ptr(d_rgb, "d_rgb"));
        NEUS2_TRY(check_ptr(d_normal, "d_normal"));
    }
    if (rays == 0) return NEUS2_OK;
    const int per = kFusedThreads / 64;
    const int64_t want = (rays + per - 1) / per;
    const int64_t cap = (int64_t)compute_units() / 2;
    hipLaunchKernelGGL(render_loss_ragged_kernel, dim3((unsigned)(want < cap ? want : cap)), dim3(kFusedThreads), 0,
                       (hipStream_t)stream, cfg->loss_kind, y, rgb, normal, target, ray_offsets, rays, n > 0 ? n : 1, cfg->s,
                       s_dev, cfg->beta, cfg->huber_delta, C, weights, loss, dC, d_sdf, d_rgb, d_normal, d_s);
    return check_launch("render + loss + backward (ragged rays)");
}

int neus2_adam_step(void* param, float* master, float* grad, float* m, float* v, int64_t count, int dtype, float lr,
                    float beta1, float beta2, float eps, int t, int flags, void* stream) {
    if (flags < 0 || flags > 3) return fail(NEUS2_ERR_CONFIG, "flags = %d, must be 0..3 (a flat array has no levels)", flags);
    if (count < 0 || count > ((int64_t)1 << 34)) return fail(NEUS2_ERR_SHAPE, "count = %lld out of range", (long long)count);
    if (dtype != 0 && dtype != 1) return fail(NEUS2_ERR_CONFIG, "dtype = %d, must be 0 (fp32) or 1 (fp16)", dtype);
    if (t < 1) return fail(NEUS2_ERR_CONFIG, "t = %d, the step number starts at 1", t);
    if (!(beta1 >= 0.f && beta1 < 1.f) || !(beta2 >= 0.f && beta2 < 1.f)) return fail(NEUS2_ERR_CONFIG, "beta1, beta2 must be in [0,1)");
    NEUS2_TRY(check_ptr(param, "param"));
    NEUS2_TRY(check_ptr(grad, "grad"));
    NEUS2_TRY(check_ptr(m, "m"));
    NEUS2_TRY(check_ptr(v, "v"));
    if (dtype == 1) NEUS2_TRY(check_ptr(master, "master"));
    if (count == 0) return NEUS2_OK;
    AdamArgs a;
    a.lr = lr; a.b1 = beta1; a.b2 = beta2; a.eps = eps;
    a.inv_c1 = (float)(1.0 / (1.0 - pow((double)beta1, (double)t)));
    a.inv_c2 = (float)(1.0 / (1.0 - pow((double)beta2, (double)t)));
    const dim3 grid((unsigned)((count + 255) / 256));
    if (dtype == 1)
        hipLaunchKernelGGL(adam_kernel<true>, grid, dim3(256), 0, (hipStream_t)stream, param, master, grad, m, v, count, a, flags);
    else
        hipLaunchKernelGGL(adam_kernel<false>, grid, dim3(256), 0, (hipStream_t)stream, param, master, grad, m, v, count, a, flags);
    return check_launch("adam");
}

namespace {

int adam_tables_impl(const neus2_config* cfg, void* tables, float* master, float* grad, float* m, float* v, float lr,
                     float beta1, float beta2, float eps, int t, int flags, const AdamExtra& extra, void* stream) {
    NEUS2_TRY(check_config(cfg));
    if (flags < 0 || flags > 7) return fail(NEUS2_ERR_CONFIG, "flags = %d, must be 0..7", flags);
    if (t < 1) return fail(NEUS2_ERR_CONFIG, "t = %d, the step number starts at 1", t);
    if (!(beta1 >= 0.f && beta1 < 1.f) || !(beta2 >= 0.f && beta2 < 1.f)) return fail(NEUS2_ERR_CONFIG, "beta1, beta2 must be in [0,1)");
    NEUS2_TRY(check_ptr(tables, "tables"));
    NEUS2_TRY(check_ptr(grad, "grad"));
    NEUS2_TRY(check_ptr(m, "m"));
    NEUS2_TRY(check_ptr(v, "v"));
    if (cfg->table_dtype == 1) NEUS2_TRY(check_ptr(master, "master"));
    AdamArgs a;
    a.lr = lr; a.b1 = beta1; a.b2 = beta2; a.eps = eps;
    a.inv_c1 = (float)(1.0 / (1.0 - pow((double)beta1, (double)t)));
    a.inv_c2 = (float)(1.0 / (1.0 - pow((double)beta2, (double)t)));
    const int64_t T = (int64_t)1 << cfg->log2_table_size;
    const int F = cfg->n_features;
    TableLevels lv;
    memset(&lv, 0, sizeof(lv));
    uint32_t most = 0;
    for (int l = 0; l < cfg->n_levels; ++l) {
        const int64_t r1 = (int64_t)cfg->res[l] + 1;
        const int64_t slots = cfg->dense[l] ? r1 * r1 * r1 : T;     // check_config: a dense level fits T
        const bool skipped = l < cfg->frozen_levels || ((flags & kAdamActiveLevels) && l >= cfg->active_levels);
        lv.used[l] = skipped ? 0u : (uint32_t)(slots * F);
        if (lv.used[l] > most) most = lv.used[l];
    }
    // one row of workgroups per level, one more for the buffer that rides along
    const dim3 grid((most + 1023u) / 1024u > 0 ? (most + 1023u) / 1024u : 1u, (unsigned)cfg->n_levels + (extra.count > 0 ? 1u : 0u));
    if (cfg->table_dtype == 1)
        hipLaunchKernelGGL(adam_tables_kernel<true>, grid, dim3(256), 0, (hipStream_t)stream, tables, master, grad, m, v, lv,
                           (uint32_t)(T * F), a, flags, extra);
    else
        hipLaunchKernelGGL(adam_tables_kernel<false>, grid, dim3(256), 0, (hipStream_t)stream, tables, master, grad, m, v, lv,
                           (uint32_t)(T * F), a, flags, extra);
    return check_launch("adam (tables)");
}

}  // namespace

int neus2_adam_tables(const neus2_config* cfg, void* tables, float* master, float* grad, float* m, float* v, float lr,
                      float beta1, float beta2, float eps, int t, int flags, void* stream) {
    const AdamExtra none = {nullptr, nullptr, nullptr, nullptr, 0};
    return adam_tables_impl(cfg, tables, master, grad, m, v, lr, beta1, beta2, eps, t, flags, none, stream);
}

int neus2_adam_all(const neus2_config* cfg, void* tables, float* master, float* grad, float* m, float* v,
                   float* small_param, float* small_grad, float* small_m, float* small_v, int64_t small_count, float lr,
                   float beta1, float beta2, float eps, int t, int flags, void* stream) {
    if (small_count < 0 || small_count > ((int64_t)1 << 28))
        return fail(NEUS2_ERR_SHAPE, "small_count = %lld out of range", (long long)small_count);
    if (small_count > 0) {
        NEUS2_TRY(check_ptr(small_param, "small_param"));
        NEUS2_TRY(check_ptr(small_grad, "small_grad"));
        NEUS2_TRY(check_ptr(small_m, "small_m"));
        NEUS2_TRY(check_ptr(small_v, "small_v"));
    }
    const AdamExtra extra = {small_param, small_grad, small_m, small_v, small_count};
    return adam_tables_impl(cfg, tables, master, grad, m, v, lr, beta1, beta2, eps, t, flags, extra, stream);
}

int neus2_rigid_fwd(const float* pos, const float* R, const float* T, float scale, float offset, int64_t n, float* out,
                    void* stream) {
    if (n < 0 || n > ((int64_t)1 << 28)) return fail(NEUS2_ERR_SHAPE, "n = %lld out of range", (long long)n);
    if (!R || !T) return fail(NEUS2_ERR_NULL, "R or T is NULL");
    NEUS2_TRY(check_ptr(pos, "pos"));
    NEUS2_TRY(check_ptr(out, "out"));
    if (n == 0) return NEUS2_OK;
    Rigid t;
    for (int k = 0; k < 9; ++k) t.R[k] = R[k];
    for (int k = 0; k < 3; ++k) t.T[k] = T[k];
    t.scale = scale; t.offset = offset;
    hipLaunchKernelGGL(rigid_fwd_kernel<false>, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, (hipStream_t)stream, pos, t,
                       nullptr, n, out);
    return check_launch("rigid transform");
}

int neus2_rigid_bwd(const float* pos, const float* T, const float* d_out, float scale, int64_t n, float* Mb, void* stream) {
    if (n < 0 || n > ((int64_t)1 << 28)) return fail(NEUS2_ERR_SHAPE, "n = %lld out of range", (long long)n);
    if (!T) return fail(NEUS2_ERR_NULL, "T is NULL");
    NEUS2_TRY(check_ptr(pos, "pos"));
    NEUS2_TRY(check_ptr(d_out, "d_out"));
    NEUS2_TRY(check_ptr(Mb, "Mb"));
    if (n == 0) return NEUS2_OK;
    Rigid t = {};
    for (int k = 0; k < 3; ++k) t.T[k] = T[k];
    t.scale = scale;
    int64_t blocks = (n + kRigidThreads - 1) / kRigidThreads;
    if (blocks > compute_units()) blocks = compute_units();
    hipLaunchKernelGGL(rigid_bwd_kernel<false>, dim3((unsigned)blocks), dim3(kRigidThreads), 0, (hipStream_t)stream, pos, t, nullptr,
                       d_out, n, Mb);
    return check_launch("rigid transform backward");
}

int neus2_rigid_fwd_dev(const float* pos, const float* pose, float scale, float offset, int64_t n, float* out, void* stream) {
    if (n < 0 || n > ((int64_t)1 << 28)) return fail(NEUS2_ERR_SHAPE, "n = %lld out of range", (long long)n);
    NEUS2_TRY(check_ptr(pose, "pose"));
    NEUS2_TRY(check_ptr(pos, "pos"));
    NEUS2_TRY(check_ptr(out, "out"));
    if (n == 0) return NEUS2_OK;
    Rigid t = {};
    t.scale = scale; t.offset = offset;
    hipLaunchKernelGGL(rigid_fwd_kernel<true>, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, (hipStream_t)stream, pos, t, pose,
                       n, out);
    return check_launch("rigid transform");
}

int neus2_rigid_bwd_dev(const float* pos, const float* pose, const float* d_out, float scale, int64_t n, float* Mb,
                        void* stream) {
    if (n < 0 || n > ((int64_t)1 << 28)) return fail(NEUS2_ERR_SHAPE, "n = %lld out of range", (long long)n);
    NEUS2_TRY(check_ptr(pose, "pose"));
    NEUS2_TRY(check_ptr(pos, "pos"));
    NEUS2_TRY(check_ptr(d_out, "d_out"));
    NEUS2_TRY(check_ptr(Mb, "Mb"));
    if (n == 0) return NEUS2_OK;
    Rigid t = {};
    t.scale = scale;
    int64_t blocks = (n + kRigidThreads - 1) / kRigidThreads;
    if (blocks > compute_units()) blocks = compute_units();
    hipLaunchKernelGGL(rigid_bwd_kernel<true>, dim3((unsigned)blocks), dim3(kRigidThreads), 0, (hipStream_t)stream, pos, t, pose,
                       d_out, n, Mb);
    return check_launch("rigid transform backward");
}

int neus2_pose_update(float* param, float* m, float* v, const float* prev, float* Mb, float* pose, float lr, float beta1,
                      float beta2, float eps, int t, int apply, void* stream) {
    if (apply != 0 && apply != 1) return fail(NEUS2_ERR_CONFIG, "apply = %d, must be 0 or 1", apply);
    if (apply) {
        if (t < 1) return fail(NEUS2_ERR_CONFIG, "t = %d, the step number starts at 1", t);
        if (!(beta1 >= 0.f && beta1 < 1.f) || !(beta2 >= 0.f && beta2 < 1.f)) return fail(NEUS2_ERR_CONFIG, "beta1, beta2 must be in [0,1)");
        NEUS2_TRY(check_ptr(m, "m"));
        NEUS2_TRY(check_ptr(v, "v"));
    }
    NEUS2_TRY(check_ptr(param, "param"));
    NEUS2_TRY(check_ptr(prev, "prev"));
    NEUS2_TRY(check_ptr(Mb, "Mb"));
    NEUS2_TRY(check_ptr(pose, "pose"));
    AdamArgs a = {};
    if (apply) {
        a.lr = lr; a.b1 = beta1; a.b2 = beta2; a.eps = eps;
        a.inv_c1 = (float)(1.0 / (1.0 - pow((double)beta1, (double)t)));
        a.inv_c2 = (float)(1.0 / (1.0 - pow((double)beta2, (double)t)));
    }
    hipLaunchKernelGGL(pose_update_kernel, dim3(1), dim3(64), 0, (hipStream_t)stream, param, m, v, prev, Mb, pose, a, apply);
    return check_launch("pose update");
}

}  // extern "C"

namespace neus2 {
int launch_zero(float* p, int64_t count, hipStream_t st) {
    if (count == 0) return NEUS2_OK;
    hipLaunchKernelGGL(zero_kernel, dim3((unsigned)((count + 255) / 256)), dim3(256), 0, st, p, count);
    return check_launch("zero");
}
}  // namespace neus2
