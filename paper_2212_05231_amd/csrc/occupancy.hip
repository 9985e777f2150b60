// Occupancy grid and ray marcher (arXiv 2212.05231, supplement Sec. E.3 "Ray Marching
// Acceleration"; the grid is kept as in the publication that passage cites: a density value per
// cell, decayed, raised at candidate cells, thresholded into one bit per cell, cells numbered
// along the Morton curve).
//
// Which lattice points of a ray become samples is an integer decision taken from binary32
// arithmetic.  Every operation that feeds it is a single rounded operation in a fixed order
// (no fused multiply-add anywhere in this file), so that the kept set can be reproduced bit for
// bit by any IEEE implementation.
#include "common.h"

#pragma clang fp contract(off)

namespace neus2 {
namespace {

constexpr int kThreads = 256;
constexpr int kScanThreads = 1024;

// 8 coordinate bits -> bits 0, 3, 6, ..., 21
__device__ __forceinline__ uint32_t spread3(uint32_t v) {
    v = (v | (v << 8)) & 0x00F00Fu;
    v = (v | (v << 4)) & 0x0C30C3u;
    v = (v | (v << 2)) & 0x249249u;
    return v;
}

__device__ __forceinline__ uint32_t gather3(uint32_t v) {
    v &= 0x249249u;
    v = (v | (v >> 2)) & 0x0C30C3u;
    v = (v | (v >> 4)) & 0x00F00Fu;
    v = (v | (v >> 8)) & 0xFFu;
    return v;
}

// Sample point of a candidate cell: (cell coordinate + jitter) / G.
__global__ __launch_bounds__(kThreads) void cell_points_kernel(int log2_res, const int32_t* __restrict__ cells,
                                                               const float* __restrict__ jitter, int64_t m,
                                                               float* __restrict__ pos) {
    const int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (i >= m) return;
    const uint32_t mask = (1u << (3 * log2_res)) - 1u;
    const uint32_t code = (uint32_t)cells[i] & mask;
    const float inv = 1.0f / (float)(1 << log2_res);           // a power of two: exact
    pos[3 * i + 0] = ((float)gather3(code) + jitter[3 * i + 0]) * inv;
    pos[3 * i + 1] = ((float)gather3(code >> 1) + jitter[3 * i + 1]) * inv;
    pos[3 * i + 2] = ((float)gather3(code >> 2) + jitter[3 * i + 2]) * inv;
}

__global__ __launch_bounds__(kThreads) void decay_kernel(float* __restrict__ density, int64_t count, float decay) {
    const int64_t i = ((int64_t)blockIdx.x * kThreads + threadIdx.x) * 4;
    if (i + 3 < count) {
        float4 v = *reinterpret_cast<float4*>(density + i);
        v.x *= decay, v.y *= decay, v.z *= decay, v.w *= decay;
        *reinterpret_cast<float4*>(density + i) = v;
    }
}

// density[cell] = max(density[cell], phi_s(sdf)).  Densities are never negative, so their bit
// patterns order like unsigned integers and one integer atomic maximum does it.
__global__ __launch_bounds__(kThreads) void raise_kernel(float* __restrict__ density, int64_t count,
                                                         const int32_t* __restrict__ cells,
                                                         const float* __restrict__ sdf, int64_t stride, int64_t m,
                                                         const float* __restrict__ s_dev, float s_fixed) {
    const int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (i >= m) return;
    const int64_t c = cells[i];
    if (c < 0 || c >= count) return;
    const float s = s_dev ? s_dev[0] : s_fixed;
    const float e = expf(-s * fabsf(sdf[i * stride]));
    const float phi = s * e / ((1.0f + e) * (1.0f + e));
    if (!(phi > 0.0f) || phi > 3.0e38f) return;                 // NaN, zero, overflow: nothing to raise
    atomicMax(reinterpret_cast<unsigned int*>(density) + c, __float_as_uint(phi));
}

// One bit per cell: set where the density exceeds the threshold.  A wavefront covers 64
// consecutive cells, i.e. two words.
__global__ __launch_bounds__(kThreads) void bits_kernel(const float* __restrict__ density, int64_t count,
                                                        float threshold, uint32_t* __restrict__ bitfield) {
    const int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    const bool on = i < count && density[i] > threshold;
    const uint64_t mask = __ballot(on);
    const int lane = threadIdx.x & 63;
    if (i < count && (lane & 31) == 0) bitfield[i >> 5] = (uint32_t)(mask >> lane);
}

// ---- marching ---------------------------------------------------------------------------------

struct Chord {
    float t0, far;     // first lattice parameter, exit parameter
    bool hit;
};

// Slab test against [0,1]^3; every lane of the wavefront computes the same values.
__device__ __forceinline__ Chord clip_ray(const float o[3], const float d[3], float jitter, float dt) {
    float near = 0.0f, far = INFINITY;
    bool hit = true;
#pragma unroll
    for (int a = 0; a < 3; ++a) {
        if (d[a] == 0.0f) {
            hit = hit && (o[a] >= 0.0f && o[a] < 1.0f);
        } else {
            const float inv = 1.0f / d[a];
            const float t1 = (0.0f - o[a]) * inv;
            const float t2 = (1.0f - o[a]) * inv;
            near = fmaxf(near, fminf(t1, t2));
            far = fminf(far, fmaxf(t1, t2));
        }
    }
    Chord c;
    c.hit = hit && near < far;
    c.far = far;
    c.t0 = near + jitter * dt;
    return c;
}

// One wavefront per ray; lane j of pass b looks at lattice point k = 64 b + j:
//   t_k = t0 + k dt, point = o + t_k d, cell = clamp(floor(point G)), kept if t_k < far and the
//   cell's bit is set.
// WRITE = false: ray_offsets[r+1] = number of kept points.  WRITE = true: ray_offsets holds the
// scanned, capacity-clamped offsets and the kept points are written in order.
template <bool WRITE>
__global__ __launch_bounds__(kThreads) void march_kernel(int log2_res, const uint32_t* __restrict__ bitfield,
                                                         const float* __restrict__ origins,
                                                         const float* __restrict__ dirs,
                                                         const float* __restrict__ jitter, int64_t rays, float dt,
                                                         int max_steps, int32_t* __restrict__ ray_offsets,
                                                         float* __restrict__ pos, int32_t* __restrict__ sample_ray,
                                                         float* __restrict__ t_out) {
    const int lane = threadIdx.x & 63;
    const int64_t r = (int64_t)blockIdx.x * (kThreads / 64) + (threadIdx.x >> 6);
    if (r >= rays) return;
    const float o[3] = {origins[3 * r], origins[3 * r + 1], origins[3 * r + 2]};
    const float d[3] = {dirs[3 * r], dirs[3 * r + 1], dirs[3 * r + 2]};
    const Chord ch = clip_ray(o, d, jitter[r], dt);
    const int G = 1 << log2_res;
    const float Gf = (float)G;
    int64_t begin = 0, end = 0;
    if (WRITE) {
        begin = ray_offsets[r];
        end = ray_offsets[r + 1];
    }
    int64_t kept = 0;
    if (ch.hit && (!WRITE || end > begin)) {
        for (int base = 0; base < max_steps; base += 64) {
            if (!(ch.t0 + (float)base * dt < ch.far)) break;            // t_k does not decrease with k
            const int k = base + lane;
            const float t = ch.t0 + (float)k * dt;
            float p[3];
            uint32_t code = 0;
#pragma unroll
            for (int a = 0; a < 3; ++a) {
                p[a] = o[a] + t * d[a];
                int c = (int)floorf(p[a] * Gf);
                c = c < 0 ? 0 : (c > G - 1 ? G - 1 : c);
                code |= spread3((uint32_t)c) << a;
            }
            bool on = k < max_steps && t < ch.far;
            if (on) on = (bitfield[code >> 5] >> (code & 31u)) & 1u;
            const uint64_t mask = __ballot(on);
            if (WRITE) {
                const int64_t dst = begin + kept + __popcll(mask & ((1ull << lane) - 1ull));
                if (on && dst < end) {
                    pos[3 * dst + 0] = p[0];
                    pos[3 * dst + 1] = p[1];
                    pos[3 * dst + 2] = p[2];
                    sample_ray[dst] = (int32_t)r;
                    if (t_out) t_out[dst] = t;
                }
            }
            kept += __popcll(mask);
            if (WRITE && begin + kept >= end) break;
        }
    }
    if (!WRITE && lane == 0) ray_offsets[r + 1] = (int32_t)kept;
}

// In place: ray_offsets[0] = 0, ray_offsets[r+1] = min(count_0 + ... + count_r, capacity).
// One workgroup walks the array in tiles of kScanThreads.
__global__ __launch_bounds__(kScanThreads) void scan_offsets_kernel(int32_t* __restrict__ ray_offsets, int64_t rays,
                                                                    int64_t capacity) {
    __shared__ int64_t wave_total[kScanThreads / 64];
    __shared__ int64_t carry_s;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    if (threadIdx.x == 0) {
        ray_offsets[0] = 0;
        carry_s = 0;
    }
    __syncthreads();
    for (int64_t tile = 0; tile < rays; tile += kScanThreads) {
        const int64_t i = tile + threadIdx.x;
        int64_t v = i < rays ? ray_offsets[i + 1] : 0;
#pragma unroll
        for (int step = 1; step < 64; step <<= 1) {
            const int64_t up = __shfl_up(v, step);
            if (lane >= step) v += up;
        }
        if (lane == 63) wave_total[wave] = v;
        __syncthreads();
        int64_t before = carry_s;
        for (int w = 0; w < wave; ++w) before += wave_total[w];
        v += before;
        if (i < rays) ray_offsets[i + 1] = (int32_t)(v < capacity ? v : capacity);
        __syncthreads();
        if (threadIdx.x == kScanThreads - 1) carry_s = v;
        __syncthreads();
    }
}

int check_grid(int log2_res) {
    if (log2_res < 2 || log2_res > 8) return fail(NEUS2_ERR_SHAPE, "log2_res %d outside 2..8", log2_res);
    return NEUS2_OK;
}

int check_m(int64_t m, const char* name) {
    if (m < 0 || m > ((int64_t)1 << 30)) return fail(NEUS2_ERR_SHAPE, "%s = %lld outside 0..2^30", name, (long long)m);
    return NEUS2_OK;
}

}  // namespace
}  // namespace neus2

using namespace neus2;

extern "C" int neus2_occupancy_points(int log2_res, const int32_t* cells, const float* jitter, int64_t m,
                                      float* pos, void* stream) {
    NEUS2_TRY(check_grid(log2_res));
    NEUS2_TRY(check_m(m, "m"));
    NEUS2_TRY(check_ptr(cells, "cells"));
    NEUS2_TRY(check_ptr(jitter, "jitter"));
    NEUS2_TRY(check_ptr(pos, "pos"));
    if (m == 0) return NEUS2_OK;
    hipStream_t st = static_cast<hipStream_t>(stream);
    cell_points_kernel<<<(unsigned)((m + kThreads - 1) / kThreads), kThreads, 0, st>>>(log2_res, cells, jitter, m, pos);
    return check_launch("cell_points_kernel");
}

extern "C" int neus2_occupancy_update(int log2_res, float* density, const int32_t* cells, const float* sdf,
                                      int64_t sdf_stride, int64_t m, const float* s_dev, float s, float decay,
                                      float threshold, uint32_t* bitfield, void* stream) {
    NEUS2_TRY(check_grid(log2_res));
    NEUS2_TRY(check_m(m, "m"));
    NEUS2_TRY(check_ptr(density, "density"));
    NEUS2_TRY(check_ptr(bitfield, "bitfield"));
    NEUS2_TRY(check_ptr(s_dev, "s_dev", false));
    if (m > 0) {
        NEUS2_TRY(check_ptr(cells, "cells"));
        NEUS2_TRY(check_ptr(sdf, "sdf"));
        if (sdf_stride < 1) return fail(NEUS2_ERR_SHAPE, "sdf_stride %lld < 1", (long long)sdf_stride);
    }
    if (!(decay >= 0.0f && decay <= 1.0f)) return fail(NEUS2_ERR_CONFIG, "decay %g outside [0,1]", (double)decay);
    if (!(threshold >= 0.0f)) return fail(NEUS2_ERR_CONFIG, "threshold %g is negative or NaN", (double)threshold);
    if (!s_dev && !(s > 0.0f)) return fail(NEUS2_ERR_CONFIG, "s %g is not positive", (double)s);
    hipStream_t st = static_cast<hipStream_t>(stream);
    const int64_t count = (int64_t)1 << (3 * log2_res);
    decay_kernel<<<(unsigned)((count / 4 + kThreads - 1) / kThreads), kThreads, 0, st>>>(
        density, count, decay);
    NEUS2_TRY(check_launch("decay_kernel"));
    if (m > 0) {
        raise_kernel<<<(unsigned)((m + kThreads - 1) / kThreads), kThreads, 0, st>>>(density, count, cells, sdf,
                                                                                      sdf_stride, m, s_dev, s);
        NEUS2_TRY(check_launch("raise_kernel"));
    }
    bits_kernel<<<(unsigned)((count + kThreads - 1) / kThreads), kThreads, 0, st>>>(density, count, threshold, bitfield);
    return check_launch("bits_kernel");
}

extern "C" int neus2_march_rays(int log2_res, const uint32_t* bitfield, const float* origins, const float* dirs,
                                const float* jitter, int64_t rays, float dt, int32_t max_steps, int64_t capacity,
                                int32_t* ray_offsets, float* pos, int32_t* sample_ray, float* t, void* stream) {
    NEUS2_TRY(check_grid(log2_res));
    if (rays < 0 || rays > ((int64_t)1 << 24)) return fail(NEUS2_ERR_SHAPE, "rays = %lld outside 0..2^24", (long long)rays);
    if (capacity < 0 || capacity > 0x7fffffffLL)
        return fail(NEUS2_ERR_SHAPE, "capacity = %lld outside 0..2^31-1", (long long)capacity);
    if (max_steps < 1 || max_steps > (1 << 20)) return fail(NEUS2_ERR_SHAPE, "max_steps = %d outside 1..2^20", max_steps);
    if (!(dt > 0.0f) || !(dt < 1e30f)) return fail(NEUS2_ERR_CONFIG, "dt %g is not a positive finite step", (double)dt);
    NEUS2_TRY(check_ptr(bitfield, "bitfield"));
    NEUS2_TRY(check_ptr(ray_offsets, "ray_offsets"));
    NEUS2_TRY(check_ptr(t, "t", false));
    if (rays > 0) {
        NEUS2_TRY(check_ptr(origins, "origins"));
        NEUS2_TRY(check_ptr(dirs, "dirs"));
        NEUS2_TRY(check_ptr(jitter, "jitter"));
    }
    if (capacity > 0) {
        NEUS2_TRY(check_ptr(pos, "pos"));
        NEUS2_TRY(check_ptr(sample_ray, "sample_ray"));
    }
    hipStream_t st = static_cast<hipStream_t>(stream);
    const unsigned blocks = (unsigned)((rays + kThreads / 64 - 1) / (kThreads / 64));
    if (rays > 0) {
        march_kernel<false><<<blocks, kThreads, 0, st>>>(log2_res, bitfield, origins, dirs, jitter, rays, dt, max_steps,
                                                         ray_offsets, nullptr, nullptr, nullptr);
        NEUS2_TRY(check_launch("march_kernel<count>"));
    }
    scan_offsets_kernel<<<1, kScanThreads, 0, st>>>(ray_offsets, rays, capacity);
    NEUS2_TRY(check_launch("scan_offsets_kernel"));
    if (rays > 0 && capacity > 0) {
        march_kernel<true><<<blocks, kThreads, 0, st>>>(log2_res, bitfield, origins, dirs, jitter, rays, dt, max_steps,
                                                        ray_offsets, pos, sample_ray, t);
        NEUS2_TRY(check_launch("march_kernel<write>"));
    }
    return NEUS2_OK;
}
