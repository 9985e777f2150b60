// Multi-resolution hash-grid encoding: forward gather (+ Jacobian) and backward scatter-add.
//
// Paper: Sec. 3 "InstantNGP" (levels of grid vertices mapped into tables of T feature
// vectors, a point's feature is the interpolation of the surrounding vertices), Sec. 4.1,
// Sec. 4.3 (levels above lambda give zeros), Eq. 7 (the term of dL/dOmega that comes through
// the normal).
//
// Launch shape: one thread per (point, level), 256 points of ONE level per workgroup.
// Workgroups are dealt round-robin to the 8 XCDs by the hardware (xcd = bid % 8), in order, so
// every XCD has a queue of its own, and the queues advance together.  A schedule built on the
// host (LevelSchedule) fills the queues with runs of point blocks of one level, such that an
// XCD works on one level at a time - that level's table (2 MiB in fp16 at T = 2^19) stays in its
// private 4 MiB L2 - and every queue holds the same number of blocks of hashed levels (which
// pull about four cache lines per point through the L2) and of dense or inactive levels (which
// mostly hit in L1): with levels dealt out whole, the XCDs that get two hashed levels set the
// pace for all.
#include <cstring>

#include <algorithm>

#include "common.h"

namespace neus2 {

namespace {

constexpr int kBlock = 256;
constexpr int kXcd = 8;
constexpr uint32_t kPrimeY = 2654435761u;
constexpr uint32_t kPrimeZ = 805459861u;

struct Cell {
    uint32_t slot[8];   // table slot of corner c = dx + 2 dy + 4 dz
    float w[3];         // offset inside the cell
};

__device__ __forceinline__ float clamp01(float x) {
    // fmaxf(NaN, 0) = 0, so NaN maps to 0 like the reference definition.
    return fminf(fmaxf(x, 0.0f), 1.0f);
}

// The grid coordinate of a point at one level is ONE binary32 multiply, rounded to nearest.
// The later subtraction of the cell index must see that rounded product, so contraction
// into a fused multiply-add is switched off for this expression (the compiler's default for
// device code would allow it, and then the interpolation weights differ from the definition
// by up to res * 2^-24).
__device__ __forceinline__ float grid_coord(float x, float fres) {
#pragma clang fp contract(off)
    float p = clamp01(x) * fres;
    asm volatile("" : "+v"(p));      // opaque to the optimiser: nothing can be fused across this point
    return p;
}

__device__ __forceinline__ Cell locate(const GridDesc& g, int level, float px, float py, float pz) {
    const int res = g.res[level];
    const float fres = (float)res;
    const float gx = grid_coord(px, fres), gy = grid_coord(py, fres), gz = grid_coord(pz, fres);
    const int cx = min((int)floorf(gx), res - 1);
    const int cy = min((int)floorf(gy), res - 1);
    const int cz = min((int)floorf(gz), res - 1);
    Cell c;
    c.w[0] = gx - (float)cx;
    c.w[1] = gy - (float)cy;
    c.w[2] = gz - (float)cz;
    if ((g.dense_bits >> level) & 1u) {
        const uint32_t s = (uint32_t)(res + 1);
        const uint32_t base = (uint32_t)cx + (uint32_t)cy * s + (uint32_t)cz * s * s;
#pragma unroll
        for (int k = 0; k < 8; ++k)
            c.slot[k] = base + (k & 1) + ((k >> 1) & 1) * s + ((k >> 2) & 1) * s * s;
    } else {
        const uint32_t hx[2] = {(uint32_t)cx, (uint32_t)cx + 1u};
        const uint32_t hy[2] = {(uint32_t)cy * kPrimeY, ((uint32_t)cy + 1u) * kPrimeY};
        const uint32_t hz[2] = {(uint32_t)cz * kPrimeZ, ((uint32_t)cz + 1u) * kPrimeZ};
#pragma unroll
        for (int k = 0; k < 8; ++k)
            c.slot[k] = (hx[k & 1] ^ hy[(k >> 1) & 1] ^ hz[(k >> 2) & 1]) & g.table_mask;
    }
    return c;
}

template <typename T>
__device__ __forceinline__ float2 load_entry(const T* level_table, uint32_t slot);

template <>
__device__ __forceinline__ float2 load_entry<float>(const float* t, uint32_t slot) {
    return reinterpret_cast<const float2*>(t)[slot];
}
template <>
__device__ __forceinline__ float2 load_entry<__half>(const __half* t, uint32_t slot) {
    return __half22float2(reinterpret_cast<const __half2*>(t)[slot]);
}

// The eight corner entries of a cell, as floats.  The coalescing unit in front of the L1
// handles about one cache line per clock, so a gather instruction whose 64 lanes touch 64
// lines costs 64 clocks whatever it returns; the two x corners of a row are therefore fetched
// with ONE load where their slots allow it.
template <typename T>
__device__ __forceinline__ void gather_corners(const GridDesc& g, int level, const T* tab, const Cell& c, float2* v) {
#pragma unroll
    for (int k = 0; k < 8; ++k) v[k] = load_entry<T>(tab, c.slot[k]);
}

struct __attribute__((packed, aligned(4))) EntryPair {
    uint32_t a, b;
};

__device__ __forceinline__ float2 entry_to_float2(uint32_t e) {
    return __half22float2(*reinterpret_cast<const __half2*>(&e));
}

// fp16 tables: an entry is one dword.  Dense level: slot(x+1) = slot(x) + 1, one 8-byte load.
// Hashed level: slot = x ^ (y*P1 ^ z*P2), so slot(x) and slot(x+1) lie in the same aligned
// group of four entries unless x % 4 == 3: one aligned 16-byte load, plus a single-entry load
// for that quarter of the lanes.
__device__ __forceinline__ uint32_t pick4(const uint4& q, uint32_t i) {
    const uint32_t lo = (i & 1u) ? q.y : q.x, hi = (i & 1u) ? q.w : q.z;
    return (i & 2u) ? hi : lo;
}

template <>
__device__ __forceinline__ void gather_corners<__half>(const GridDesc& g, int level, const __half* tab, const Cell& c, float2* v) {
    const uint32_t* t32 = reinterpret_cast<const uint32_t*>(tab);
    if ((g.dense_bits >> level) & 1u) {                       // uniform over the workgroup
        EntryPair p[4];
#pragma unroll
        for (int row = 0; row < 4; ++row) p[row] = *reinterpret_cast<const EntryPair*>(t32 + c.slot[2 * row]);
#pragma unroll
        for (int row = 0; row < 4; ++row) {
            v[2 * row] = entry_to_float2(p[row].a);
            v[2 * row + 1] = entry_to_float2(p[row].b);
        }
    } else {
        // all loads are issued before any of them is used
        uint4 grp[4];
        uint32_t far[4];
#pragma unroll
        for (int row = 0; row < 4; ++row) grp[row] = *reinterpret_cast<const uint4*>(t32 + (c.slot[2 * row] & ~3u));
#pragma unroll
        for (int row = 0; row < 4; ++row) {
            far[row] = 0u;
            if ((c.slot[2 * row] ^ c.slot[2 * row + 1]) >= 4u) far[row] = t32[c.slot[2 * row + 1]];
        }
#pragma unroll
        for (int row = 0; row < 4; ++row) {
            const uint32_t s0 = c.slot[2 * row], s1 = c.slot[2 * row + 1];
            const uint32_t e0 = pick4(grp[row], s0 & 3u);
            const uint32_t near = pick4(grp[row], s1 & 3u);
            const uint32_t e1 = (s0 ^ s1) < 4u ? near : far[row];
            v[2 * row] = entry_to_float2(e0);
            v[2 * row + 1] = entry_to_float2(e1);
        }
    }
}

// Per XCD a queue of runs of consecutive point blocks of one level; positions in a queue are
// j = bid / 8.  Runs of expensive levels come first in every queue and are equally long (+-1).
struct LevelSchedule {
    static constexpr int kMaxRuns = 12;
    int per_xcd;                         // queue length (the grid has 8 * per_xcd workgroups)
    short n_runs[kXcd];
    short level[kXcd][kMaxRuns];
    int start[kXcd][kMaxRuns + 1];       // first queue position of a run; [n_runs] = end of the queue
    int first_pb[kXcd][kMaxRuns];
};

// block index -> (level, point block); returns false for padding blocks.  Every index into the
// schedule is the same for all lanes of the workgroup (indexing a by-value kernel argument with a
// value that differs between lanes is not supported).
__device__ __forceinline__ bool decode_schedule(const LevelSchedule& sch, int& level, int& pb) {
    const int bid = blockIdx.x;
    const int xcd = bid % kXcd;
    const int j = bid / kXcd;
    const int runs = sch.n_runs[xcd];
    if (j >= sch.start[xcd][runs]) return false;
    int r = 0;
    while (r + 1 < runs && j >= sch.start[xcd][r + 1]) ++r;
    level = sch.level[xcd][r];
    pb = sch.first_pb[xcd][r] + (j - sch.start[xcd][r]);
    return true;
}

// block index -> (level, point block) with levels dealt out whole: xcd = bid % 8,
// level = xcd + 8 * slot; returns false for padding blocks
__device__ __forceinline__ bool decode_block(int n_levels, int point_blocks, int& level, int& pb) {
    const int bid = blockIdx.x;
    const int xcd = bid % kXcd;
    const int j = bid / kXcd;
    level = xcd + kXcd * (j / point_blocks);
    pb = j % point_blocks;
    return level < n_levels;
}

// HESS: the mixed second derivatives of the interpolation are written as well (hess [level][3][n][2]:
// the pairs (d2e_f/dxdy), (d2e_f/dxdz), (d2e_f/dydz), f = 0, 1), for a step that wants the gradient with
// respect to the positions: the corners are in registers here, so the backward pass needs no second
// gather for them.  The pure second derivatives of a trilinear interpolation are zero.
template <typename T, bool HESS>
__global__ __launch_bounds__(kBlock) void encode_kernel(GridDesc g, LevelSchedule sch, ZeroRegions zero,
                                                        const float* __restrict__ pos,
                                                        const T* __restrict__ tables, int64_t n,
                                                        float* __restrict__ enc,
                                                        float* __restrict__ jac,
                                                        uint32_t* __restrict__ dbg_idx,
                                                        float* __restrict__ hess) {
    if (blockIdx.x == 0) {
#pragma unroll
        for (int r = 0; r < 2; ++r)
            for (int k = threadIdx.x; k < zero.count[r]; k += kBlock) zero.p[r][k] = 0.f;
    }
    int level, pb;
    if (!decode_schedule(sch, level, pb)) return;
    const int64_t i = (int64_t)pb * kBlock + threadIdx.x;
    if (i >= n) return;
    const float px = pos[3 * i + 0], py = pos[3 * i + 1], pz = pos[3 * i + 2];
    const Cell c = locate(g, level, px, py, pz);
    if (dbg_idx) {
#pragma unroll
        for (int k = 0; k < 8; ++k) dbg_idx[(i * g.n_levels + level) * 8 + k] = c.slot[k];
    }
    float e0 = 0.f, e1 = 0.f;
    float j0[3] = {0.f, 0.f, 0.f}, j1[3] = {0.f, 0.f, 0.f};
    float h0[3] = {0.f, 0.f, 0.f}, h1[3] = {0.f, 0.f, 0.f};       // xy, xz, yz
    if (level < g.active_levels) {
        const T* tab = tables + (size_t)level * g.table_size * 2;
        float2 v[8];
        gather_corners<T>(g, level, tab, c, v);
        const float fres = (float)g.res[level];
#pragma unroll
        for (int k = 0; k < 8; ++k) {
            const float fx = (k & 1) ? c.w[0] : 1.f - c.w[0];
            const float fy = (k & 2) ? c.w[1] : 1.f - c.w[1];
            const float fz = (k & 4) ? c.w[2] : 1.f - c.w[2];
            const float sx = (k & 1) ? fres : -fres;
            const float sy = (k & 2) ? fres : -fres;
            const float sz = (k & 4) ? fres : -fres;
            const float wk = fx * fy * fz;
            const float dx = sx * fy * fz, dy = fx * sy * fz, dz = fx * fy * sz;
            e0 += wk * v[k].x;
            e1 += wk * v[k].y;
            j0[0] += dx * v[k].x; j0[1] += dy * v[k].x; j0[2] += dz * v[k].x;
            j1[0] += dx * v[k].y; j1[1] += dy * v[k].y; j1[2] += dz * v[k].y;
            if (HESS) {
                const float dxy = sx * sy * fz, dxz = sx * fy * sz, dyz = fx * sy * sz;
                h0[0] += dxy * v[k].x; h0[1] += dxz * v[k].x; h0[2] += dyz * v[k].x;
                h1[0] += dxy * v[k].y; h1[1] += dxz * v[k].y; h1[2] += dyz * v[k].y;
            }
        }
    }
    const int64_t o = (int64_t)level * n + i;
    reinterpret_cast<float2*>(enc)[o] = make_float2(e0, e1);
    // three planes per level, each written as consecutive 8-byte words by consecutive lanes.  The Jacobian is
    // the widest array of the step and is read next when the network kernels get to this point, after the rest
    // of the batch has been encoded: non-temporal stores (30 us of the step at 2^20 points, none at 2^18).
    typedef float f2v __attribute__((ext_vector_type(2)));
    f2v* jo = reinterpret_cast<f2v*>(jac) + (int64_t)level * 3 * n + i;
    __builtin_nontemporal_store(f2v{j0[0], j0[1]}, jo);
    __builtin_nontemporal_store(f2v{j0[2], j1[0]}, jo + n);
    __builtin_nontemporal_store(f2v{j1[1], j1[2]}, jo + 2 * n);
    if (HESS && level < g.active_levels) {
        f2v* ho = reinterpret_cast<f2v*>(hess) + (int64_t)level * 3 * n + i;
        ho[0] = f2v{h0[0], h1[0]};
        ho[n] = f2v{h0[1], h1[1]};
        ho[2 * n] = f2v{h0[2], h1[2]};
    }
}

// d_pos += sum over levels and features of q_f (d2e_f/dx dx') dL/dn from the stored second derivatives and,
// with jac and d_enc given, (de/dx)^T dL/de from the stored Jacobian: a stream of 32 (64) bytes per point
// and level.
__global__ __launch_bounds__(kBlock) void pos_from_hessian_kernel(const float* __restrict__ hess, const float* __restrict__ q,
                                                                  const float* __restrict__ d_normal,
                                                                  const float* __restrict__ jac, const float* __restrict__ d_enc,
                                                                  int levels, int first_level,
                                                                  int64_t n, float* __restrict__ d_pos) {
    const int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    if (i >= n) return;
    const float nx = d_normal[3 * i + 0], ny = d_normal[3 * i + 1], nz = d_normal[3 * i + 2];
    float hp[3] = {0.f, 0.f, 0.f};
    for (int l = first_level; l < levels; ++l) {
        const float2* h = reinterpret_cast<const float2*>(hess) + (int64_t)l * 3 * n + i;
        const float2 xy = h[0], xz = h[n], yz = h[2 * n];
        const float2 qq = reinterpret_cast<const float2*>(q)[(int64_t)l * n + i];
        const float qxy = qq.x * xy.x + qq.y * xy.y, qxz = qq.x * xz.x + qq.y * xz.y, qyz = qq.x * yz.x + qq.y * yz.y;
        hp[0] += qxy * ny + qxz * nz;
        hp[1] += qxy * nx + qyz * nz;
        hp[2] += qxz * nx + qyz * ny;
        if (jac) {
            const float2* J = reinterpret_cast<const float2*>(jac) + (int64_t)l * 3 * n + i;
            const float2 a = J[0], b = J[n], c = J[2 * n];          // (J00,J01) (J02,J10) (J11,J12)
            const float2 de = reinterpret_cast<const float2*>(d_enc)[(int64_t)l * n + i];
            hp[0] += de.x * a.x + de.y * b.y;
            hp[1] += de.x * a.y + de.y * c.x;
            hp[2] += de.x * b.x + de.y * c.y;
        }
    }
    d_pos[3 * i + 0] += hp[0]; d_pos[3 * i + 1] += hp[1]; d_pos[3 * i + 2] += hp[2];
}

// Backward.  d_tables[slot_c][f] += w_c * dL/de_f + q_f * res * sum_a dL/dn_a d_a w_c
// (first-order term, and the term Eq. 7 keeps).  With WANT_POS the mixed second derivative
// of the interpolation, contracted with q and dL/dn, is added into d_pos.
//
// The L2 executes float atomics at a fixed rate per (instruction, 64-byte line) request,
// however many lanes of the instruction fall into that line.  So four adjacent lanes share
// one point: lane (dx, f) of the group owns the corners with that x offset and feature f,
// and each of its four atomic instructions (one per (dy, dz)) puts the group's four
// addresses {slot(x), slot(x+1)} x {f0, f1} next to each other: the same 16 bytes on a
// dense level, the same line for 7 of 8 cells on a hashed one.  On coarse levels, where
// consecutive samples of a ray sit in the same cell, runs of equal cells inside the wave are
// summed with a segmented scan first and only the last lane group of a run issues atomics.
constexpr int kScatterPoints = kBlock / 4;     // points per workgroup
constexpr int kMergeMaxRes = 128;              // run-merge only where runs exist

template <typename T, bool WANT_POS>
__global__ __launch_bounds__(kBlock) void scatter_kernel(GridDesc g, const float* __restrict__ pos,
                                                         const T* __restrict__ tables,
                                                         const float* __restrict__ q,
                                                         const float* __restrict__ d_enc,
                                                         const float* __restrict__ d_normal, int64_t n,
                                                         int point_blocks, float* __restrict__ d_tables,
                                                         float* __restrict__ d_pos) {
    int level, pb;
    if (!decode_block(g.active_levels, point_blocks, level, pb)) return;
    if (level < g.frozen_levels && !WANT_POS) return;      // an input level: no table gradient
    const int sub = threadIdx.x & 3;
    const int dxb = sub >> 1, f = sub & 1;
    const int64_t i_raw = (int64_t)pb * kScatterPoints + (threadIdx.x >> 2);
    const bool valid = i_raw < n;
    const int64_t i = valid ? i_raw : n - 1;       // keep every lane in the shuffles below
    const int res = g.res[level];
    const float fres = (float)res;
    const float gx = grid_coord(pos[3 * i + 0], fres), gy = grid_coord(pos[3 * i + 1], fres), gz = grid_coord(pos[3 * i + 2], fres);
    const int cx = min((int)floorf(gx), res - 1);
    const int cy = min((int)floorf(gy), res - 1);
    const int cz = min((int)floorf(gz), res - 1);
    const float w0 = gx - (float)cx, w1 = gy - (float)cy, w2 = gz - (float)cz;
    const bool dense = (g.dense_bits >> level) & 1u;
    uint32_t slot[4];
    if (dense) {
        const uint32_t s = (uint32_t)(res + 1);
        const uint32_t base = (uint32_t)(cx + dxb) + (uint32_t)cy * s + (uint32_t)cz * s * s;
#pragma unroll
        for (int k = 0; k < 4; ++k) slot[k] = base + (k & 1) * s + (k >> 1) * s * s;
    } else {
        const uint32_t hx = (uint32_t)(cx + dxb);
        const uint32_t hy[2] = {(uint32_t)cy * kPrimeY, ((uint32_t)cy + 1u) * kPrimeY};
        const uint32_t hz[2] = {(uint32_t)cz * kPrimeZ, ((uint32_t)cz + 1u) * kPrimeZ};
#pragma unroll
        for (int k = 0; k < 4; ++k) slot[k] = (hx ^ hy[k & 1] ^ hz[k >> 1]) & g.table_mask;
    }
    const int64_t o = ((int64_t)level * n + i) * 2 + f;
    const float de = d_enc[o];
    const float qf = q[o];
    const float nx = d_normal[3 * i + 0] * fres, ny = d_normal[3 * i + 1] * fres, nz = d_normal[3 * i + 2] * fres;
    const float fx = dxb ? w0 : 1.f - w0;
    const float sx = dxb ? 1.f : -1.f;
    float val[4];
    float hp[3] = {0.f, 0.f, 0.f};
    const T* tab = tables + (size_t)level * g.table_size * 2;
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const float fy = (k & 1) ? w1 : 1.f - w1;
        const float fz = (k & 2) ? w2 : 1.f - w2;
        const float sy = (k & 1) ? 1.f : -1.f;
        const float sz = (k & 2) ? 1.f : -1.f;
        const float wk = fx * fy * fz;
        const float dn = nx * (sx * fy * fz) + ny * (fx * sy * fz) + nz * (fx * fy * sz);
        val[k] = valid ? wk * de + qf * dn : 0.f;
        if (WANT_POS) {
            const float2 v2 = load_entry<T>(tab, slot[k]);
            const float qv = qf * (f ? v2.y : v2.x) * fres;
            hp[0] += qv * (ny * (sx * sy * fz) + nz * (sx * fy * sz));
            hp[1] += qv * (nx * (sx * sy * fz) + nz * (fx * sy * sz));
            hp[2] += qv * (nx * (sx * fy * sz) + ny * (fx * sy * sz));
        }
    }
    bool issue = valid;
    if (res <= kMergeMaxRes) {
        // segmented inclusive scan over the wave's 16 lane groups, segments = runs of one cell
        const int lane = threadIdx.x & 63, grp = lane >> 2;
        const uint32_t cell = valid ? (uint32_t)cx + (uint32_t)res * ((uint32_t)cy + (uint32_t)res * (uint32_t)cz) : 0xFFFFFFFFu;
        const uint32_t prev = __shfl_up(cell, 4);
        const uint32_t next = __shfl_down(cell, 4);
        bool head = grp == 0 || prev != cell;
        const bool tail = grp == 15 || next != cell;
#pragma unroll
        for (int d = 1; d < 16; d <<= 1) {
            float up[4];
#pragma unroll
            for (int k = 0; k < 4; ++k) up[k] = __shfl_up(val[k], 4 * d);
            const bool up_head = __shfl_up((int)head, 4 * d) != 0;
            if (grp >= d && !head) {
#pragma unroll
                for (int k = 0; k < 4; ++k) val[k] += up[k];
                head = up_head;
            }
        }
        issue = valid && tail;
    }
    if (issue && level >= g.frozen_levels) {
        float* gt = d_tables + (size_t)level * g.table_size * 2 + f;
#pragma unroll
        for (int k = 0; k < 4; ++k) atomicAdd(gt + 2 * (size_t)slot[k], val[k]);
    }
    if (WANT_POS) {
#pragma unroll
        for (int c = 0; c < 3; ++c) {
            hp[c] += __shfl_xor(hp[c], 1);
            hp[c] += __shfl_xor(hp[c], 2);
        }
        if (valid && sub == 0) {
            atomicAdd(d_pos + 3 * i + 0, hp[0]);
            atomicAdd(d_pos + 3 * i + 1, hp[1]);
            atomicAdd(d_pos + 3 * i + 2, hp[2]);
        }
    }
}

// The position-gradient part of the backward pass on its own, for the path below that does
// not touch the tables' values: per point and level, the mixed second derivative of the
// interpolation contracted with q and dL/dn (three numbers), written to part[level][i][3];
// `sum_levels_kernel` adds the levels into d_pos.  Same gather as the encoder, same
// workgroup -> level mapping (a level's table stays in the L2 of the XCDs that work on it).
template <typename T>
__global__ __launch_bounds__(kBlock) void pos_hessian_kernel(GridDesc g, const float* __restrict__ pos,
                                                             const T* __restrict__ tables,
                                                             const float* __restrict__ q,
                                                             const float* __restrict__ d_normal,
                                                             const float* __restrict__ d_enc, int64_t n,
                                                             LevelSchedule sch, float* __restrict__ part) {
    int level, pb;
    if (!decode_schedule(sch, level, pb)) return;
    const int64_t i = (int64_t)pb * kBlock + threadIdx.x;
    if (i >= n) return;
    const Cell c = locate(g, level, pos[3 * i + 0], pos[3 * i + 1], pos[3 * i + 2]);
    const int64_t o = (int64_t)level * n + i;
    const float2 qq = reinterpret_cast<const float2*>(q)[o];
    const float fres = (float)g.res[level];
    const float nx = d_normal[3 * i + 0] * fres, ny = d_normal[3 * i + 1] * fres, nz = d_normal[3 * i + 2] * fres;
    float2 v[8];
    gather_corners<T>(g, level, tables + (size_t)level * g.table_size * 2, c, v);
    // with d_enc: the first-order part (de/dx)^T dL/de of this level as well (the Jacobian is
    // rebuilt from the corners that are here anyway)
    float2 de = make_float2(0.f, 0.f);
    if (d_enc) de = reinterpret_cast<const float2*>(d_enc)[o];
    float hp[3] = {0.f, 0.f, 0.f};
#pragma unroll
    for (int k = 0; k < 8; ++k) {
        const float fx = (k & 1) ? c.w[0] : 1.f - c.w[0];
        const float fy = (k & 2) ? c.w[1] : 1.f - c.w[1];
        const float fz = (k & 4) ? c.w[2] : 1.f - c.w[2];
        const float sx = (k & 1) ? 1.f : -1.f;
        const float sy = (k & 2) ? 1.f : -1.f;
        const float sz = (k & 4) ? 1.f : -1.f;
        const float ev = (de.x * v[k].x + de.y * v[k].y) * fres;
        hp[0] += ev * (sx * fy * fz);
        hp[1] += ev * (fx * sy * fz);
        hp[2] += ev * (fx * fy * sz);
        const float qv = (qq.x * v[k].x + qq.y * v[k].y) * fres;
        hp[0] += qv * (ny * (sx * sy * fz) + nz * (sx * fy * sz));
        hp[1] += qv * (nx * (sx * sy * fz) + nz * (fx * sy * sz));
        hp[2] += qv * (nx * (sx * fy * sz) + ny * (fx * sy * sz));
    }
    part[3 * o + 0] = hp[0]; part[3 * o + 1] = hp[1]; part[3 * o + 2] = hp[2];
}

__global__ __launch_bounds__(kBlock) void sum_levels_kernel(const float* __restrict__ part, int levels, int64_t n,
                                                            float* __restrict__ d_pos) {
    const int64_t k = (int64_t)blockIdx.x * kBlock + threadIdx.x;      // over the 3 n numbers of d_pos
    if (k >= 3 * n) return;
    float acc = d_pos[k];
    for (int l = 0; l < levels; ++l) acc += part[(int64_t)l * 3 * n + k];
    d_pos[k] = acc;
}

// ---- scatter-add without global atomics: LDS-resident slot ranges ---------------------------
//
// Float atomics leave the L2 as one 32-byte read-modify-write per (instruction, line) and
// the chip retires about 2e10 of them per second, which caps the kernel above at about four
// requests per point and level.  For large batches the table gradient is therefore
// accumulated in LDS instead: a level's T slots are cut into ranges of 8192 slots (128 KiB
// of fp64 pairs, one workgroup's LDS); the workgroup that owns a range adds everything that
// falls into it with LDS atomics and finally adds its LDS image to the global gradient with
// coalesced atomics, one per non-zero accumulator (64 consecutive floats per instruction: a few
// line requests, not one per lane; reading the old values and storing the sums instead held 16
// registers per thread for the length of a task and cost 10 us per step more).  The accumulators are
// DOUBLES on purpose: measured on this chip, ds_add_f64 retires a lane in 0.37 clocks and
// ds_add_f32 in 3.2 (the LDS does float atomics one lane at a time), so fp64 is both the
// faster and the more accurate choice.
//
// Hashed levels (two kernels).  On a hashed level the range of a corner is the top bits of
// slot = x ^ y*P1 ^ z*P2; x is smaller than 2^13, so the range depends on (dy, dz) only and
// both x corners of a row (y+dy, z+dz) share it.  `bin_rows_kernel` computes, per point and
// level, the four row records {two local slots, four values} once and appends each to the
// list of its range in the workspace (position = per-workgroup LDS rank + one global cursor
// reservation per workgroup and range).  `scatter_owner_kernel` then streams the list of its
// range, fully coalesced.  A list that overflows its capacity (only possible when a batch
// concentrates on very few cells) sends the surplus records straight to global atomics, so
// the result never depends on the capacity.
// Dense levels: with one or two ranges they take the in-place path (a filter pass queues the
// points of a chunk whose cell touches the range, then all eight corners are tested) and flush
// with coalesced atomics, several chunks sharing a range; with 3..64 ranges the bin kernel
// appends the point's number to the list of every range one of its corners falls into and an
// owner task takes a segment of such a list; with more ranges they get row records like a hashed
// level.  Workgroups take tasks from a counter, heaviest tasks first.
constexpr int kOwnerThreads = 1024;
constexpr int64_t kOwnerMinPoints = 1 << 16;
constexpr int kOwnerSlotBits = 13;
constexpr int kOwnerSlots = 1 << kOwnerSlotBits;
constexpr int kMaxRanges = 256;
constexpr int kCursorOffset = 256;                                  // bytes: [0,4) task counter
constexpr int kWorkspaceHeader = kCursorOffset + 4 * NEUS2_MAX_LEVELS * kMaxRanges;

struct OwnerPlan {
    int n_entries;
    int n_tasks;
    int n_listed;                           // entries [0, n_listed) are levels with record lists
    int n_indexed;                          // entries [n_listed, n_listed + n_indexed) are levels with point lists
    int seg_points;                         // list entries per task of a level with point lists
    int idx_capacity[NEUS2_MAX_LEVELS];     // points per list of such a level
    int64_t idx_base[NEUS2_MAX_LEVELS + 1]; // first list entry of the level's lists; [n_listed + n_indexed] = total
    int first_task[NEUS2_MAX_LEVELS + 1];   // prefix sums over entries, in the order `order`
    short order[NEUS2_MAX_LEVELS];          // entries by falling time of one task
    int capacity[NEUS2_MAX_LEVELS];         // records per list of a listed entry
    int64_t list_base[NEUS2_MAX_LEVELS + 1];// first record of the entry's lists; [n_listed] = total
    short level[NEUS2_MAX_LEVELS];
    short ranges[NEUS2_MAX_LEVELS];
    int chunks[NEUS2_MAX_LEVELS];           // point chunks of an in-place level, list segments of a level with point lists
    int chunk_points[NEUS2_MAX_LEVELS];     // points per chunk (the last chunk may hold fewer)
};

// A row record: what one point adds to the two x corners of one row (y+dy, z+dz) of its cell, in 12
// bytes.  Four values {x f0, x f1, x+1 f0, x+1 f1} share one exponent and keep 18-bit signed
// mantissas: value = m * 2^(E - 96 - 17), E chosen from the largest magnitude of the four, so each is
// off by at most 2^-17 of that largest one (4e-6 rms) - the gradient is compared at 1e-4, and the
// four products that make up a value already carry binary32 rounding.  The slots: 13 bits for the
// first corner's slot inside its range, 4 bits for how the second follows from it: code t <= 12:
// slot ^ (2^(t+1) - 1) (hashed level: x enters the hash by xor, so the two slots differ in the
// trailing bits in which x and x+1 differ); 15: slot + 1 (dense level); 14: the same slot (dense
// level, second corner beyond the range: its values are zero here and went to the gradient directly).
//   a: slot 0..12 | code 13..16 | E 17..23 | m3 low 8 bits 24..31
//   b: m0 0..17 | m1 low 14 bits 18..31
//   c: m1 high 4 bits 0..3 | m2 4..21 | m3 high 10 bits 22..31
// E = 127 marks a record whose values were not finite (or beyond 2^30): it decodes to NaN, so that a
// broken gradient stays visible.  Magnitudes below 2^-96 are written as zero.
struct __attribute__((packed, aligned(4))) RowRecord {
    uint32_t a, b, c;
};

constexpr int kRecBias = 96;
constexpr int kRecMant = 17;                       // magnitude bits of a mantissa
constexpr uint32_t kCodeNext = 15u, kCodeSame = 14u;

__device__ __forceinline__ int sext(uint32_t x, int off, int len) { return (int32_t)(x << (32 - off - len)) >> (32 - len); }

__device__ __forceinline__ RowRecord pack_row(uint32_t slot, uint32_t code, const float4& v) {
    const float big = fmaxf(fmaxf(fabsf(v.x), fabsf(v.y)), fmaxf(fabsf(v.z), fabsf(v.w)));   // NaN if any is
    int e = __builtin_amdgcn_frexp_expf(big);      // big = f 2^e, 0.5 <= f < 1; 0 for big = 0
    int E = e + kRecBias;
    int m[4] = {0, 0, 0, 0};
    if (!(big <= 1.0e9f)) {
        E = 127;
    } else if (E < 0 || big == 0.f) {
        E = 0;
    } else {
        // in * 2^(17-e) rounded to nearest even, as the low bits of a float: adding 1.5 * 2^23 leaves
        // the integer in the mantissa (two's complement in the low 18 bits); |in| < 2^e, so the only value
        // out of range is +2^17 (a magnitude just below 2^e rounding up), which the unsigned minimum on
        // the bit pattern (positive floats order like their patterns) brings back to 2^17 - 1.
        const float in[4] = {v.x, v.y, v.z, v.w};
        const float scale = __builtin_bit_cast(float, (uint32_t)(127 + kRecMant - e) << 23);
        constexpr float kRound = 12582912.0f;                     // 1.5 * 2^23, pattern 0x4B400000
#pragma unroll
        for (int k = 0; k < 4; ++k)
            m[k] = (int)min(__builtin_bit_cast(uint32_t, fmaf(in[k], scale, kRound)), 0x4B400000u + ((1u << kRecMant) - 1u));
    }
    RowRecord r;
    r.a = slot | (code << 13) | ((uint32_t)E << 17) | (((uint32_t)m[3] & 0xFFu) << 24);
    r.b = ((uint32_t)m[0] & 0x3FFFFu) | (((uint32_t)m[1] & 0x3FFFu) << 18);
    r.c = (((uint32_t)m[1] >> 14) & 0xFu) | (((uint32_t)m[2] & 0x3FFFFu) << 4) | ((((uint32_t)m[3] >> 8) & 0x3FFu) << 22);
    return r;
}

__device__ __forceinline__ void unpack_row(const RowRecord& r, uint32_t& s0, uint32_t& s1, float (&v)[4]) {
    s0 = r.a & (kOwnerSlots - 1);
    const uint32_t code = (r.a >> 13) & 15u;
    s1 = code == kCodeNext ? s0 + 1u : code == kCodeSame ? s0 : s0 ^ ((2u << code) - 1u);
    const int E = (int)((r.a >> 17) & 127u);
    const int m0 = sext(r.b, 0, 18);
    const int m1 = (sext(r.c, 0, 4) << 14) | (int)(r.b >> 18);
    const int m2 = sext(r.c, 4, 18);
    const int m3 = (sext(r.c, 22, 10) << 8) | (int)(r.a >> 24);
    // 2^(E - bias - mant) as a float: the exponent field alone (always a normal number)
    const float scale = E == 127 ? __builtin_nanf("") : __builtin_bit_cast(float, (uint32_t)(E - kRecBias - kRecMant + 127) << 23);
    v[0] = (float)m0 * scale; v[1] = (float)m1 * scale; v[2] = (float)m2 * scale; v[3] = (float)m3 * scale;
}

struct Records {
    int* cursor;            // [n_listed + n_indexed][kMaxRanges]
    uint32_t* index;        // levels with point lists: per entry [ranges][idx_capacity] point numbers
    RowRecord* rows;        // per entry [ranges][capacity]
};

// Records of one workgroup are first put in LDS in list order (range by range), then written
// out by consecutive threads: runs of records of one list leave as whole cache lines instead
// of one 16-byte piece per lane.
constexpr int kBinThreads = 512;
constexpr int kBinRecords = 4 * kBinThreads;
constexpr uint32_t kNoRecord = 0xFFFFFFFFu;

struct BinSmem {
    uint32_t ra[kBinRecords], rb[kBinRecords], rc[kBinRecords];   // the staged records, word by word
    uint32_t dest[kBinRecords];          // record index within the entry's lists, kNoRecord if it went elsewhere
    int cnt[kMaxRanges];                 // records of this workgroup per range
    int base[kMaxRanges];                // first position of this workgroup in the list of the range
    int first[kMaxRanges];               // first staged position of the range
    int total;
};

// What one point adds to the two features of corner cr of its cell: w_c dL/de_f + q_f res sum_a dL/dn_a d_a w_c
// (ax, ay, az = dL/dn times res).
__device__ __forceinline__ float2 corner_value(const Cell& c, int cr, const float2& de, const float2& qq, float ax, float ay, float az) {
    const float fx = (cr & 1) ? c.w[0] : 1.f - c.w[0];
    const float fy = (cr & 2) ? c.w[1] : 1.f - c.w[1];
    const float fz = (cr & 4) ? c.w[2] : 1.f - c.w[2];
    const float sx = (cr & 1) ? 1.f : -1.f;
    const float sy = (cr & 2) ? 1.f : -1.f;
    const float sz = (cr & 4) ? 1.f : -1.f;
    const float wk = fx * fy * fz;
    const float dn = ax * (sx * fy * fz) + ay * (fx * sy * fz) + az * (fx * fy * sz);
    return make_float2(wk * de.x + qq.x * dn, wk * de.y + qq.y * dn);
}

// Dense levels with several ranges get POINT lists instead of row records: a point's eight slots are
// base + {0,1} + {0,s} + {0,s^2}, ascending in the corner number, so the ranges they fall into are
// ascending too; the point's number is appended to the list of every range that holds one of its
// corners (one or two for most points).  4 bytes per entry instead of 48 bytes of row records per
// point, and the owner of a range no longer tests every point of the batch against its range.
// A list that is full sends the point's corners in that range straight to the gradient.
__device__ void bin_points(const GridDesc& g, const OwnerPlan& plan, const Records& rec, const float* __restrict__ pos,
                           const float* __restrict__ q, const float* __restrict__ d_enc,
                           const float* __restrict__ d_normal, int64_t n, int point_blocks, int e,
                           float* __restrict__ d_tables, int* cnt, int* base) {
    const int level = plan.level[e];
    const int n_ranges = plan.ranges[e];
    const int capacity = plan.idx_capacity[e];
    const int64_t i = (int64_t)(blockIdx.x % point_blocks) * kBinThreads + threadIdx.x;
    for (int k = threadIdx.x; k < kMaxRanges; k += kBinThreads) cnt[k] = 0;
    __syncthreads();
    const bool valid = i < n;
    Cell c;
    int rank[8];
    uint32_t fresh = 0;                       // bit k: corner k is the first of the point in its range
    if (valid) {
        c = locate(g, level, pos[3 * i + 0], pos[3 * i + 1], pos[3 * i + 2]);
#pragma unroll
        for (int k = 0; k < 8; ++k) {
            rank[k] = 0;
            if (k == 0 || (c.slot[k] >> kOwnerSlotBits) != (c.slot[k - 1] >> kOwnerSlotBits)) {
                fresh |= 1u << k;
                rank[k] = atomicAdd(&cnt[c.slot[k] >> kOwnerSlotBits], 1);
            }
        }
    }
    __syncthreads();
    for (int k = threadIdx.x; k < n_ranges; k += kBinThreads)
        base[k] = cnt[k] ? atomicAdd(&rec.cursor[e * kMaxRanges + k], cnt[k]) : 0;
    __syncthreads();
    if (!valid) return;
    uint32_t* lists = rec.index + plan.idx_base[e];
#pragma unroll
    for (int k = 0; k < 8; ++k) {
        if (!((fresh >> k) & 1u)) continue;
        const uint32_t r = c.slot[k] >> kOwnerSlotBits;
        const int at = base[r] + rank[k];
        if (at < capacity) {
            lists[(size_t)r * capacity + at] = (uint32_t)i;
        } else {
            const int64_t o = (int64_t)level * n + i;
            const float2 de = reinterpret_cast<const float2*>(d_enc)[o];
            const float2 qq = reinterpret_cast<const float2*>(q)[o];
            const float fres = (float)g.res[level];
            const float ax = d_normal[3 * i + 0] * fres, ay = d_normal[3 * i + 1] * fres, az = d_normal[3 * i + 2] * fres;
            float* gt = d_tables + (size_t)level * g.table_size * 2;
            for (int cr = k; cr < 8 && (c.slot[cr] >> kOwnerSlotBits) == r; ++cr) {
                const float2 v = corner_value(c, cr, de, qq, ax, ay, az);
                atomicAdd(gt + 2 * (size_t)c.slot[cr] + 0, v.x);
                atomicAdd(gt + 2 * (size_t)c.slot[cr] + 1, v.y);
            }
        }
    }
}

// A workgroup takes 512 points and walks over a share of the levels with row records (levels
// grp, grp + level_groups, ...): position and dL/dn are fetched once, and the next level's dL/de and
// dd/de are requested before the current level's records are made, so that only the first level of a
// workgroup waits for memory.  Workgroups beyond the level groups handle the levels with point lists.
__global__ __launch_bounds__(kBinThreads) void bin_rows_kernel(GridDesc g, OwnerPlan plan, Records rec,
                                                              const float* __restrict__ pos,
                                                              const float* __restrict__ q,
                                                              const float* __restrict__ d_enc,
                                                              const float* __restrict__ d_normal, int64_t n,
                                                              int point_blocks, int level_groups,
                                                              float* __restrict__ d_tables) {
    __shared__ BinSmem sm;
    const int grp = blockIdx.x / point_blocks;
    if (grp >= level_groups) {                // uniform over the workgroup
        bin_points(g, plan, rec, pos, q, d_enc, d_normal, n, point_blocks, plan.n_listed + grp - level_groups, d_tables, sm.cnt,
                   sm.base);
        return;
    }
    const int64_t i = (int64_t)(blockIdx.x % point_blocks) * kBinThreads + threadIdx.x;
    const bool valid = i < n;
    float px = 0.f, py = 0.f, pz = 0.f, dnx = 0.f, dny = 0.f, dnz = 0.f;
    float2 de_next = make_float2(0.f, 0.f), q_next = make_float2(0.f, 0.f);
    if (valid) {
        px = pos[3 * i + 0]; py = pos[3 * i + 1]; pz = pos[3 * i + 2];
        dnx = d_normal[3 * i + 0]; dny = d_normal[3 * i + 1]; dnz = d_normal[3 * i + 2];
        const int64_t o = (int64_t)plan.level[grp] * n + i;
        de_next = reinterpret_cast<const float2*>(d_enc)[o];
        q_next = reinterpret_cast<const float2*>(q)[o];
    }
    for (int e = grp; e < plan.n_listed; e += level_groups) {
        const int level = plan.level[e];
        const int n_ranges = plan.ranges[e];
        const int capacity = plan.capacity[e];
        const float2 de = de_next, qq = q_next;
        if (valid && e + level_groups < plan.n_listed) {
            const int64_t o = (int64_t)plan.level[e + level_groups] * n + i;
            // last use of both arrays in the step: non-temporal loads
            typedef float f2v __attribute__((ext_vector_type(2)));
            const f2v a_ = __builtin_nontemporal_load(reinterpret_cast<const f2v*>(d_enc) + o);
            const f2v b_ = __builtin_nontemporal_load(reinterpret_cast<const f2v*>(q) + o);
            de_next = make_float2(a_.x, a_.y);
            q_next = make_float2(b_.x, b_.y);
        }
        for (int k = threadIdx.x; k < kMaxRanges; k += kBinThreads) sm.cnt[k] = 0;
        __syncthreads();

        uint32_t range[4];
        RowRecord row_rec[4];
        int rank[4];
        if (valid) {
            const int res = g.res[level];
            const float fres = (float)res;
            const bool dense = (g.dense_bits >> level) & 1u;
            const uint32_t stride = (uint32_t)res + 1u;
            const float gx = grid_coord(px, fres), gy = grid_coord(py, fres), gz = grid_coord(pz, fres);
            const int cx = min((int)floorf(gx), res - 1);
            const int cy = min((int)floorf(gy), res - 1);
            const int cz = min((int)floorf(gz), res - 1);
            const float w0 = gx - (float)cx, w1 = gy - (float)cy, w2 = gz - (float)cz;
            const float nx = dnx * fres, ny = dny * fres, nz = dnz * fres;
            const uint32_t hy0 = (uint32_t)cy * kPrimeY, hz0 = (uint32_t)cz * kPrimeZ;
            // the trailing bits in which x and x + 1 differ: 2^(t+1) - 1, t = number of trailing ones of x
            const uint32_t code_x = 31u - (uint32_t)__clz((int)((uint32_t)cx ^ ((uint32_t)cx + 1u)));
#pragma unroll
            for (int row = 0; row < 4; ++row) {
                const int dy = row & 1, dz = row >> 1;
                const uint32_t rh = (hy0 + (dy ? kPrimeY : 0u)) ^ (hz0 + (dz ? kPrimeZ : 0u));
                const float fy = dy ? w1 : 1.f - w1, fz = dz ? w2 : 1.f - w2;
                const float sy = dy ? 1.f : -1.f, sz = dz ? 1.f : -1.f;
                const float fyz = fy * fz;
                const float dn_x = nx * fyz;
                const float dn_yz = ny * (sy * fz) + nz * (fy * sz);
                uint32_t s0, s1, code;
                if (dense) {
                    s0 = (uint32_t)cx + ((uint32_t)(cy + dy) + (uint32_t)(cz + dz) * stride) * stride;
                    s1 = s0 + 1u;
                    code = kCodeNext;
                } else {
                    s0 = ((uint32_t)cx ^ rh) & g.table_mask;
                    s1 = ((uint32_t)(cx + 1) ^ rh) & g.table_mask;
                    code = code_x;
                }
                const float f0 = 1.f - w0, f1 = w0;
                const float dn0 = -dn_x + f0 * dn_yz, dn1 = dn_x + f1 * dn_yz;
                const float wk0 = f0 * fyz, wk1 = f1 * fyz;
                float4 val = make_float4(wk0 * de.x + qq.x * dn0, wk0 * de.y + qq.y * dn0, wk1 * de.x + qq.x * dn1, wk1 * de.y + qq.y * dn1);
                range[row] = s0 >> kOwnerSlotBits;
                // On a hashed level both corners share the range.  On a dense level the x+1 corner can be
                // the first slot of the next range (1 row in 8192): it then goes straight to the gradient.
                if ((s1 >> kOwnerSlotBits) != range[row]) {
                    float* gt = d_tables + ((size_t)level * g.table_size + s1) * 2;
                    atomicAdd(gt + 0, val.z);
                    atomicAdd(gt + 1, val.w);
                    val.z = 0.f; val.w = 0.f;
                    code = kCodeSame;
                }
                row_rec[row] = pack_row(s0 & (kOwnerSlots - 1), code, val);
                rank[row] = atomicAdd(&sm.cnt[range[row]], 1);
            }
        }
        __syncthreads();
        // one reservation per range in the global list, and the staged order: ranges one after another
        for (int k = threadIdx.x; k < n_ranges; k += kBinThreads)
            sm.base[k] = sm.cnt[k] ? atomicAdd(&rec.cursor[e * kMaxRanges + k], sm.cnt[k]) : 0;
        if (threadIdx.x >= kBinThreads - 64) {               // the last wavefront: exclusive prefix sums of cnt
            const int lane = threadIdx.x & 63;
            constexpr int kPer = kMaxRanges / 64;
            int c[kPer], sum = 0;
#pragma unroll
            for (int j = 0; j < kPer; ++j) { c[j] = sm.cnt[kPer * lane + j]; sum += c[j]; }
            int incl = sum;
#pragma unroll
            for (int d = 1; d < 64; d <<= 1) {
                const int o = __shfl_up(incl, d);
                if (lane >= d) incl += o;
            }
            int at = incl - sum;
#pragma unroll
            for (int j = 0; j < kPer; ++j) { sm.first[kPer * lane + j] = at; at += c[j]; }
            if (lane == 63) sm.total = incl;
        }
        __syncthreads();
        if (valid) {
#pragma unroll
            for (int row = 0; row < 4; ++row) {
                const int r = (int)range[row];
                const int in_list = sm.base[r] + rank[row];
                const int at = sm.first[r] + rank[row];
                sm.ra[at] = row_rec[row].a; sm.rb[at] = row_rec[row].b; sm.rc[at] = row_rec[row].c;
                if (in_list < capacity) {
                    sm.dest[at] = (uint32_t)r * (uint32_t)capacity + (uint32_t)in_list;
                } else {                                                 // list full: straight to the global gradient
                    sm.dest[at] = kNoRecord;
                    uint32_t s0, s1;
                    float v[4];
                    unpack_row(row_rec[row], s0, s1, v);
                    float* gt = d_tables + ((size_t)level * g.table_size + ((size_t)r << kOwnerSlotBits)) * 2;
                    atomicAdd(gt + 2 * s0 + 0, v[0]);
                    atomicAdd(gt + 2 * s0 + 1, v[1]);
                    atomicAdd(gt + 2 * s1 + 0, v[2]);
                    atomicAdd(gt + 2 * s1 + 1, v[3]);
                }
            }
        }
        __syncthreads();
        const int total = sm.total;
        RowRecord* out = rec.rows + plan.list_base[e];
        for (int at = threadIdx.x; at < total; at += kBinThreads) {
            const uint32_t d = sm.dest[at];
            if (d != kNoRecord) {
                RowRecord r;
                r.a = sm.ra[at]; r.b = sm.rb[at]; r.c = sm.rc[at];
                out[d] = r;            // (a non-temporal store here costs 0.2 ms: measured)
            }
        }
        // the next round writes cnt only after the barrier that follows its clearing, base/first/total
        // after the one behind its ranks, and the staged records after a third: every thread has left
        // this loop by then
    }
}

// In-place path: a filter round tests kFilter points per thread; rounds are added while fewer than
// kOwnerThreads points are queued, so the queue never holds (kFilter + 1) kOwnerThreads or more.
constexpr int kFilter = 4;
constexpr int kQueue = (kFilter + 1) * kOwnerThreads;

struct OwnerSmem {
    double acc[2 * kOwnerSlots];
    uint32_t queue[kQueue];    // in-place path: points of the chunk that touch the range
    int queued;
    int task[2];               // mailbox for the task numbers, see the kernel
};

// The corners of point i that fall into `range`, added to the range's LDS accumulators.
struct PointIn {
    float px, py, pz, ax, ay, az;
    float2 de, qq;
};

__device__ __forceinline__ PointIn load_point(int level, int64_t i, int64_t n, float fres, const float* __restrict__ pos,
                                              const float* __restrict__ q, const float* __restrict__ d_enc,
                                              const float* __restrict__ d_normal) {
    PointIn p;
    const int64_t o = (int64_t)level * n + i;
    p.de = reinterpret_cast<const float2*>(d_enc)[o];
    p.qq = reinterpret_cast<const float2*>(q)[o];
    p.ax = d_normal[3 * i + 0] * fres; p.ay = d_normal[3 * i + 1] * fres; p.az = d_normal[3 * i + 2] * fres;
    p.px = pos[3 * i + 0]; p.py = pos[3 * i + 1]; p.pz = pos[3 * i + 2];
    return p;
}

__device__ __forceinline__ void add_loaded_point(const GridDesc& g, int level, uint32_t range, const PointIn& p, double* acc, int odd) {
    const Cell c = locate(g, level, p.px, p.py, p.pz);
#pragma unroll
    for (int cr = 0; cr < 8; ++cr) {
        if ((c.slot[cr] >> kOwnerSlotBits) != range) continue;
        const float2 v = corner_value(c, cr, p.de, p.qq, p.ax, p.ay, p.az);
        double* a = acc + 2 * (c.slot[cr] & (kOwnerSlots - 1));
        atomicAdd(a + odd, (double)(odd ? v.y : v.x));
        atomicAdd(a + (odd ^ 1), (double)(odd ? v.x : v.y));
    }
}

__device__ __forceinline__ void add_point_to_range(const GridDesc& g, int level, uint32_t range, int64_t i, int64_t n,
                                                   const float* __restrict__ pos, const float* __restrict__ q,
                                                   const float* __restrict__ d_enc, const float* __restrict__ d_normal,
                                                   double* acc, int odd) {
    add_loaded_point(g, level, range, load_point(level, i, n, (float)g.res[level], pos, q, d_enc, d_normal), acc, odd);
}

__global__ __launch_bounds__(kOwnerThreads) void scatter_owner_kernel(GridDesc g, OwnerPlan plan, Records rec,
                                                                     const float* __restrict__ pos,
                                                                     const float* __restrict__ q,
                                                                     const float* __restrict__ d_enc,
                                                                     const float* __restrict__ d_normal,
                                                                     int64_t n, int* __restrict__ counter,
                                                                     float* __restrict__ d_tables) {
    __shared__ OwnerSmem sm;
    double* acc = sm.acc;
    constexpr int kPerThread = 2 * kOwnerSlots / kOwnerThreads;      // accumulators per thread
    // The two features of a slot lie side by side.  Even lanes add feature 0 first, odd lanes
    // feature 1: one instruction then spreads over all LDS banks instead of every other pair.
    const int odd = threadIdx.x & 1;
    // The accumulators are cleared once here and then by every flush as it reads them, and the
    // next task number is requested while the current task runs and handed over through a
    // two-entry mailbox: one barrier separates two tasks.
#pragma unroll
    for (int u = 0; u < kPerThread; ++u) acc[threadIdx.x + u * kOwnerThreads] = 0.0;
    int next_task = 0;
    if (threadIdx.x == 0) { sm.task[0] = atomicAdd(counter, 1); sm.queued = 0; }
    __syncthreads();
    for (int turn = 0;; turn ^= 1) {
        const int task = sm.task[turn];
        if (task >= plan.n_tasks) break;             // uniform: every thread reads the same value
        if (threadIdx.x == 0) next_task = atomicAdd(counter, 1);
        // entry of the task: all prefix sums are compared at once (independent scalar loads with
        // constant offsets, not a dependent chain of them; the index must stay uniform)
        int at_order = 0;
#pragma unroll
        for (int k = 1; k < NEUS2_MAX_LEVELS; ++k) at_order += (k < plan.n_entries && task >= plan.first_task[k]) ? 1 : 0;
        const int e = plan.order[at_order];
        const int local = task - plan.first_task[at_order];
        const int level = plan.level[e];
        const int n_ranges = plan.ranges[e], n_chunks = plan.chunks[e];
        const uint32_t range = (uint32_t)(local % n_ranges);
        const int chunk = local / n_ranges;
        const int64_t begin = (int64_t)chunk * plan.chunk_points[e];
        const int64_t end = min(begin + plan.chunk_points[e], n);
        const uint32_t first_slot = range << kOwnerSlotBits;
        const uint32_t slots_here = min((uint32_t)kOwnerSlots, g.table_size - first_slot);
        float* dst = d_tables + ((size_t)level * g.table_size + first_slot) * 2;
        bool nothing_added = false;

        if (e < plan.n_listed) {
            // A listed task streams the list of its range.
            const int count = min(rec.cursor[e * kMaxRanges + range], plan.capacity[e]);
            const size_t at = (size_t)plan.list_base[e] + (size_t)range * plan.capacity[e];
            const RowRecord* rs = rec.rows + at;
            // this task's stretch of the list (the whole list unless the plan shares lists out)
            const int stretch = ((count + n_chunks - 1) / n_chunks + 63) / 64 * 64;
            const int first = chunk * stretch, stop = min(count, first + stretch);
            nothing_added = first >= stop;
            // four records per thread in flight: the list is streamed from HBM
            constexpr int kAhead = 4;
            for (int j0 = first + threadIdx.x; j0 < stop; j0 += kAhead * kOwnerThreads) {
                RowRecord rr[kAhead];
#pragma unroll
                for (int k = 0; k < kAhead; ++k) {
                    const int j = j0 + k * kOwnerThreads;
                    // a record is read once: non-temporal load, 12 bytes in one instruction
                    if (j < stop) {
                        typedef uint32_t u3 __attribute__((ext_vector_type(3), aligned(4)));
                        const u3 w = __builtin_nontemporal_load(reinterpret_cast<const u3*>(rs + j));
                        rr[k].a = w.x; rr[k].b = w.y; rr[k].c = w.z;
                    }
                }
#pragma unroll
                for (int k = 0; k < kAhead; ++k) {
                    if (j0 + k * kOwnerThreads < stop) {
                        uint32_t s0, s1;
                        float v[4];
                        unpack_row(rr[k], s0, s1, v);
                        double* a0 = acc + 2 * s0;
                        double* a1 = acc + 2 * s1;
                        atomicAdd(a0 + odd, (double)(odd ? v[1] : v[0]));
                        atomicAdd(a0 + (odd ^ 1), (double)(odd ? v[0] : v[1]));
                        atomicAdd(a1 + odd, (double)(odd ? v[3] : v[2]));
                        atomicAdd(a1 + (odd ^ 1), (double)(odd ? v[2] : v[3]));
                    }
                }
            }
        } else if (e < plan.n_listed + plan.n_indexed) {
            // A task of a level with point lists takes one segment of the list of its range: the points
            // whose cell has a corner in the range.  Two points per thread in flight.
            const int count = min(rec.cursor[e * kMaxRanges + range], plan.idx_capacity[e]);
            const uint32_t* list = rec.index + plan.idx_base[e] + (size_t)range * plan.idx_capacity[e];
            // the last segment of a range takes whatever lies beyond the finely cut part of the list
            const int seg_begin = chunk * plan.seg_points;
            const int seg_end = chunk == n_chunks - 1 ? count : min(seg_begin + plan.seg_points, count);
            nothing_added = seg_begin >= seg_end;
            const float fres = (float)g.res[level];
            for (int j = seg_begin + (int)threadIdx.x; j < seg_end; j += 2 * kOwnerThreads) {
                const int j2 = j + kOwnerThreads;
                const bool two = j2 < seg_end;
                const uint32_t i0 = __builtin_nontemporal_load(list + j), i1 = two ? __builtin_nontemporal_load(list + j2) : 0u;
                const PointIn p0 = load_point(level, i0, n, fres, pos, q, d_enc, d_normal);
                PointIn p1 = p0;
                if (two) p1 = load_point(level, i1, n, fres, pos, q, d_enc, d_normal);
                add_loaded_point(g, level, range, p0, acc, odd);
                if (two) add_loaded_point(g, level, range, p1, acc, odd);
            }
        } else {
            // In-place path.  A task tests its chunk of the points against its range and adds the
            // corners that fall into it.  On a dense level with several ranges most points of a
            // wavefront miss, so the test (position only) and the work are separated: points that
            // hit are queued in LDS, and the queue is worked off with every lane busy.
            const float fres = (float)g.res[level];
            const bool filter = n_ranges > 1;              // only dense levels have several ranges here
            int64_t next = begin;
            for (;;) {
                for (;;) {                                 // fill until every thread has work, or the chunk ends
                    float px[kFilter], py[kFilter], pz[kFilter];
#pragma unroll
                    for (int k = 0; k < kFilter; ++k) {
                        const int64_t i = next + threadIdx.x + k * kOwnerThreads;
                        if (filter && i < end) { px[k] = pos[3 * i + 0]; py[k] = pos[3 * i + 1]; pz[k] = pos[3 * i + 2]; }
                    }
#pragma unroll
                    for (int k = 0; k < kFilter; ++k) {
                        const int64_t i = next + threadIdx.x + k * kOwnerThreads;
                        bool hit = i < end;
                        if (hit && filter) {
                            // on a dense level the eight slots lie in [slot[0], slot[7]]
                            const Cell c = locate(g, level, px[k], py[k], pz[k]);
                            hit = (c.slot[7] >> kOwnerSlotBits) >= range && (c.slot[0] >> kOwnerSlotBits) <= range;
                        }
                        const unsigned long long m = __ballot(hit);
                        if (m) {                            // one reservation per wavefront
                            const int lane = threadIdx.x & 63;
                            const int leader = __ffsll((long long)m) - 1;
                            int at = 0;
                            if (lane == leader) at = atomicAdd(&sm.queued, __popcll(m));
                            at = __shfl(at, leader);
                            if (hit) sm.queue[at + __popcll(m & ((1ull << lane) - 1ull))] = (uint32_t)(i - begin);
                        }
                    }
                    next += (int64_t)kFilter * kOwnerThreads;
                    __syncthreads();
                    const int queued = sm.queued;
                    __syncthreads();                        // nobody adds to the counter before all have read it
                    if (queued >= kOwnerThreads || next >= end) break;
                }
                const int queued = sm.queued;
                for (int j = threadIdx.x; j < queued; j += kOwnerThreads)
                    add_point_to_range(g, level, range, begin + sm.queue[j], n, pos, q, d_enc, d_normal, acc, odd);
                __syncthreads();
                if (threadIdx.x == 0) sm.queued = 0;
                __syncthreads();
                if (next >= end) break;
            }
        }
        // flush: the LDS image is added to the gradient (several chunks of the points may share a
        // range of a dense level) and cleared for the next task; a task that found its segment of a
        // point list empty has nothing to flush (the same for every thread)
        __syncthreads();
        if (!nothing_added) {
#pragma unroll
            for (int u = 0; u < kPerThread; ++u) {
                const uint32_t k = threadIdx.x + u * kOwnerThreads;
                const float v = (float)acc[k];
                acc[k] = 0.0;
                if (k < 2 * slots_here && v != 0.f) atomicAdd(dst + k, v);
            }
        }
        if (threadIdx.x == 0) sm.task[turn ^ 1] = next_task;
        __syncthreads();
    }
}

// Which levels get record lists, which point lists, how many ranges and point chunks.  Levels with
// row records (hashed levels with several ranges, dense levels with more than kInPlaceRanges
// ranges) come first, then the dense levels with point lists (kIndexedMinRanges..kInPlaceRanges
// ranges), then the levels of one or two ranges, which take the in-place path.  ok = false if the
// configuration does not fit the scheme (then the atomic kernel is used).
constexpr int kInPlaceRanges = 64;
constexpr int kIndexedMinRanges = 3;
constexpr int kSegPoints = 8192;          // list entries per task of a level with point lists

OwnerPlan make_owner_plan(const neus2_config* cfg, int64_t n, bool& ok) {
    OwnerPlan p;
    memset(&p, 0, sizeof(p));
    ok = true;
    p.seg_points = kSegPoints;
    const int64_t T = (int64_t)1 << cfg->log2_table_size;
    if (T > (int64_t)kMaxRanges * kOwnerSlots) ok = false;          // at most kMaxRanges lists per level
    int e = 0, tasks = 0;
    int64_t records = 0, indices = 0;
    double cost[NEUS2_MAX_LEVELS];
    // lists of row records over all levels (see `chunks` of a listed level below)
    int64_t listed_ranges = 0;
    for (int l = cfg->frozen_levels; l < cfg->active_levels; ++l) {
        const int64_t r1 = (int64_t)cfg->res[l] + 1;
        const int64_t used = cfg->dense[l] ? r1 * r1 * r1 : T;
        const int ranges = (int)((used + kOwnerSlots - 1) / kOwnerSlots);
        if (ranges > (cfg->dense[l] ? kInPlaceRanges : 1)) listed_ranges += ranges;
    }
    int listed_chunks = 1;
    if (listed_ranges > 0) listed_chunks = (int)std::min<int64_t>(4, std::max<int64_t>(1, (2 * compute_units() + listed_ranges - 1) / listed_ranges));

    for (int pass = 0; pass < 3; ++pass) {
        for (int l = cfg->frozen_levels; l < cfg->active_levels; ++l) {
            const int64_t r1 = (int64_t)cfg->res[l] + 1;
            const int64_t used = cfg->dense[l] ? r1 * r1 * r1 : T;
            const int ranges = (int)((used + kOwnerSlots - 1) / kOwnerSlots);
            const bool listed = ranges > (cfg->dense[l] ? kInPlaceRanges : 1);
            const bool indexed = !listed && cfg->dense[l] && ranges >= kIndexedMinRanges;
            if ((listed ? 0 : indexed ? 1 : 2) != pass) continue;
            if (listed && !cfg->dense[l] && cfg->res[l] >= kOwnerSlots) ok = false;   // x must not reach the range bits
            int chunks = 1;
            double task_ns = 4000.0 + 1.25 * (4.0 * (double)n / ranges);   // a list: 1.25 ns per record
            if (listed) {
                // With few lists in all (small tables, few active levels) a list is shared out over several
                // tasks, so that the chip's workgroups get several rounds of them: each task takes a stretch of
                // the list and flushes what it added (atomics, like every flush).
                chunks = listed_chunks;
                task_ns = 4000.0 + 1.25 * (4.0 * (double)n / ranges) / chunks;
                // a list holds 1.5 times its expected share of the 4 n row records of the level;
                // 3 times on a dense level, where the share of a slab of the grid follows the batch
                const int64_t cap = ((4 * n / ranges) * (cfg->dense[l] ? 6 : 3) / 2 + 1023) / 64 * 64;
                if (cap * ranges >= ((int64_t)1 << 32) - 1) ok = false;     // record positions are 32 bits
                p.capacity[e] = (int)cap;
                p.list_base[e] = records;
                records += cap * ranges;
            } else if (indexed) {
                // A point enters the lists of the ranges its eight corners fall into: two on average when
                // a range is thinner than a layer of the grid; the slabs through the middle of the scene
                // hold several times the average.  Eight times the mean share; the surplus, if any, goes
                // through atomics.  A task takes kSegPoints entries of one list; tasks beyond the end of
                // a list find nothing to do.
                const int64_t cap = (8 * n / ranges + 1023) / 64 * 64;
                if (cap >= ((int64_t)1 << 31) - 1 || n >= ((int64_t)1 << 32)) ok = false;
                p.idx_capacity[e] = (int)cap;
                p.idx_base[e] = indices;
                indices += cap * ranges;
                // Tasks: the list is cut finely up to three times its expected length (m n / ranges, where
                // m = 1 + min(1, s^2 / 8192) is about the number of ranges a point's corners fall into, s^2 the
                // slots between two layers of the grid); one more task takes the rest, if there is any.
                const double layers = (double)(r1 * r1) / kOwnerSlots;
                const double expect = (1.0 + (layers < 1.0 ? layers : 1.0)) * (double)n / ranges;
                int64_t fine = (int64_t)(3.0 * expect / kSegPoints) + 1;
                if (fine > (cap + kSegPoints - 1) / kSegPoints) fine = (cap + kSegPoints - 1) / kSegPoints;
                chunks = (int)fine + 1;
                if ((int64_t)chunks * ranges > (1 << 20)) ok = false;
                task_ns = 4000.0 + 7.0 * kSegPoints;
            } else {
                // Every task tests n / chunks points (0.9 ns each; the corner code runs for a whole
                // wavefront as soon as one lane is in the range) and adds those in its range
                // (about 1.5 ranges per point on a dense level, 7 ns each).  Times measured on
                // this kernel.  Tasks of 70 us by this estimate, at least eight chunks: every task
                // ends with a flush of its LDS image, so shorter tasks cost more than they balance
                // (a sweep of 15..300 us and 2..16 chunks on the benchmark workload).
                const double hit = ranges > 1 ? 1.5 / ranges : 1.0;
                const double level_ns = (double)n * ranges * (0.9 + 7.0 * (hit < 1.0 ? hit : 1.0));
                chunks = (int)(level_ns / ranges / 70000.0) + 1;
                if (chunks < 8) chunks = 8;
                if (chunks > 128) chunks = 128;
                task_ns = 4000.0 + level_ns / ranges / chunks;
            }
            p.level[e] = (short)l;
            p.ranges[e] = (short)ranges;
            p.chunks[e] = chunks;
            p.chunk_points[e] = (int)((n + chunks - 1) / chunks);
            cost[e] = task_ns;
            ++e;
        }
        if (pass == 0) { p.n_listed = e; p.list_base[e] = records; }
        if (pass == 1) { p.n_indexed = e - p.n_listed; p.idx_base[e] = indices; }
    }
    p.n_entries = e;
    // Workgroups take tasks in this order: the longest first, so that the kernel does not end
    // on a few workgroups that drew a long task late.
    for (int k = 0; k < e; ++k) p.order[k] = (short)k;
    std::stable_sort(p.order, p.order + e, [&](short a, short b) { return cost[a] > cost[b]; });
    for (int k = 0; k < e; ++k) {
        p.first_task[k] = tasks;
        tasks += p.ranges[p.order[k]] * p.chunks[p.order[k]];
    }
    p.first_task[e] = tasks;
    p.n_tasks = tasks;
    return p;
}

// Queues for levels [0, n_levels): hashed active levels count as expensive, the rest as cheap;
// each class is cut into 8 equal stretches of its level-major block list.
LevelSchedule make_level_schedule(const GridDesc& g, int n_levels, int point_blocks) {
    LevelSchedule sch;
    memset(&sch, 0, sizeof(sch));
    int fill[kXcd] = {0};
    for (int cls = 0; cls < 2; ++cls) {
        int lv[NEUS2_MAX_LEVELS], m = 0;
        for (int l = 0; l < n_levels; ++l) {
            const bool expensive = l < g.active_levels && !((g.dense_bits >> l) & 1u);
            if (expensive == (cls == 0)) lv[m++] = l;
        }
        const int64_t total = (int64_t)m * point_blocks;
        for (int x = 0; x < kXcd; ++x) {
            int64_t a = total * x / kXcd;
            const int64_t b = total * (x + 1) / kXcd;
            while (a < b) {
                const int k = (int)(a / point_blocks), pb = (int)(a % point_blocks);
                const int64_t len = std::min<int64_t>(b - a, point_blocks - pb);
                const int r = sch.n_runs[x]++;
                sch.level[x][r] = (short)lv[k];
                sch.start[x][r] = fill[x];
                sch.first_pb[x][r] = pb;
                fill[x] += (int)len;
                a += len;
            }
        }
    }
    for (int x = 0; x < kXcd; ++x) {
        sch.start[x][sch.n_runs[x]] = fill[x];
        sch.per_xcd = std::max(sch.per_xcd, fill[x]);
    }
    return sch;
}

int grid_blocks(int levels, int point_blocks) {
    const int slots = (levels + kXcd - 1) / kXcd;
    return kXcd * slots * point_blocks;
}

}  // namespace

int launch_encode(const neus2_config* cfg, const float* pos, const void* tables, int64_t n,
                  float* enc, float* jac, uint32_t* dbg_idx, hipStream_t st, const ZeroRegions* zero, float* hess,
                  bool active_only) {
    ZeroRegions zr = {{nullptr, nullptr}, {0, 0}};
    if (zero) zr = *zero;
    if (n == 0) {
        for (int r = 0; r < 2; ++r)
            if (zr.count[r] > 0) NEUS2_TRY(launch_zero(zr.p[r], zr.count[r], st));
        return NEUS2_OK;
    }
    const GridDesc g = make_grid_desc(cfg);
    const int pbs = (int)((n + kBlock - 1) / kBlock);
    // active_only: the levels beyond the active ones are left alone instead of written as zeros (the training
    // step: none of its kernels reads them)
    const int levels = active_only ? std::max(g.active_levels, 1) : g.n_levels;
    const LevelSchedule sch = make_level_schedule(g, levels, pbs);
    const dim3 grid(kXcd * sch.per_xcd);
#define NEUS2_ENCODE(T, HESS)                                                                     \
    hipLaunchKernelGGL((encode_kernel<T, HESS>), grid, dim3(kBlock), 0, st, g, sch, zr, pos, (const T*)tables, n, enc, jac, \
                       dbg_idx, hess)
    if (cfg->table_dtype == 1) {
        if (hess) NEUS2_ENCODE(__half, true); else NEUS2_ENCODE(__half, false);
    } else {
        if (hess) NEUS2_ENCODE(float, true); else NEUS2_ENCODE(float, false);
    }
#undef NEUS2_ENCODE
    return check_launch("hash encode");
}

int64_t owner_workspace_need(const OwnerPlan& plan) {
    return kWorkspaceHeader + plan.list_base[plan.n_listed] * 12 + plan.idx_base[plan.n_listed + plan.n_indexed] * 4 + 256;
}

// scratch of the position-gradient path, behind the records: either part[active levels][n][3] (the gather
// pass) or hess[active levels][3][n][2] (the training step, whose encode kernel writes it)
int64_t pos_scratch_bytes(const neus2_config* cfg, int64_t n) { return (int64_t)cfg->active_levels * n * 24; }

// where the training step's encode kernel puts the second derivatives, or nullptr if the scatter-add will
// not take the path with the workspace (must mirror launch_scatter's condition)
float* scatter_hessian_region(const neus2_config* cfg, int64_t n, void* workspace, int64_t workspace_bytes) {
    if (!scatter_gathers_position(cfg, n, workspace, workspace_bytes)) return nullptr;
    bool ok = false;
    const OwnerPlan plan = make_owner_plan(cfg, n, ok);
    return reinterpret_cast<float*>(reinterpret_cast<char*>(workspace) + (owner_workspace_need(plan) + 255) / 256 * 256);
}

int64_t scatter_workspace_bytes(const neus2_config* cfg, int64_t n) {
    if (n < kOwnerMinPoints) return 0;
    bool ok = false;
    const OwnerPlan plan = make_owner_plan(cfg, n, ok);
    if (!ok) return 0;
    return (owner_workspace_need(plan) + 255) / 256 * 256 + (int64_t)cfg->n_levels * n * 24;
}

int64_t scatter_records_bytes(const neus2_config* cfg, int64_t n) {
    if (n < kOwnerMinPoints || cfg->active_levels == 0) return 0;
    bool ok = false;
    const OwnerPlan plan = make_owner_plan(cfg, n, ok);
    return ok ? owner_workspace_need(plan) : 0;
}

bool scatter_gathers_position(const neus2_config* cfg, int64_t n, const void* workspace, int64_t workspace_bytes) {
    if (n < kOwnerMinPoints || !workspace || cfg->active_levels <= cfg->frozen_levels) return false;
    bool ok = false;
    const OwnerPlan plan = make_owner_plan(cfg, n, ok);
    return ok && workspace_bytes >= (owner_workspace_need(plan) + 255) / 256 * 256 + pos_scratch_bytes(cfg, n);
}

// must mirror the condition under which launch_scatter takes the path with the workspace
void scatter_header(const neus2_config* cfg, int64_t n, bool want_pos, void* workspace, int64_t workspace_bytes,
                    float** p, int* count) {
    *p = nullptr;
    *count = 0;
    if (n == 0 || cfg->active_levels == 0 || n < kOwnerMinPoints || !workspace) return;
    bool ok = false;
    const OwnerPlan plan = make_owner_plan(cfg, n, ok);
    const int64_t records_end = (owner_workspace_need(plan) + 255) / 256 * 256;
    if (ok && workspace_bytes >= (want_pos ? records_end + pos_scratch_bytes(cfg, n) : owner_workspace_need(plan))) {
        *p = reinterpret_cast<float*>(workspace);
        *count = kWorkspaceHeader / 4;
    }
}

int launch_scatter(const neus2_config* cfg, const float* pos, const void* tables, const float* q,
                   const float* d_enc, const float* d_normal, int64_t n, float* d_tables,
                   float* d_pos, void* workspace, int64_t workspace_bytes, bool first_order_pos, hipStream_t st,
                   bool header_cleared, bool hessian_stored, const float* jac) {
    if (n == 0 || cfg->active_levels == 0) return NEUS2_OK;
    const GridDesc g = make_grid_desc(cfg);
    // Large batches with a workspace: LDS-owner kernel (no global atomics on the big levels);
    // the position gradient, if wanted, comes from a gather pass of its own.  Below ~2^16
    // points the atomic kernel is cheaper.
    if (n >= kOwnerMinPoints && workspace) {
        bool ok = false;
        const OwnerPlan plan = make_owner_plan(cfg, n, ok);
        const int64_t records_end = (owner_workspace_need(plan) + 255) / 256 * 256;
        if (ok && workspace_bytes >= (d_pos ? records_end + pos_scratch_bytes(cfg, n) : owner_workspace_need(plan))) {
            char* ws = reinterpret_cast<char*>(workspace);
            int* counter = reinterpret_cast<int*>(ws);
            Records rec;
            rec.cursor = reinterpret_cast<int*>(ws + kCursorOffset);
            rec.rows = reinterpret_cast<RowRecord*>(ws + kWorkspaceHeader);
            rec.index = reinterpret_cast<uint32_t*>(ws + kWorkspaceHeader + plan.list_base[plan.n_listed] * 12);
            if (!header_cleared)                                                                 // task counter and cursors
                NEUS2_TRY(launch_zero(reinterpret_cast<float*>(ws), kWorkspaceHeader / 4, st));
            if (plan.n_listed + plan.n_indexed > 0) {
                const int pbs = (int)((n + kBinThreads - 1) / kBinThreads);
                // enough workgroups to fill the chip several times over; each walks over its share of the levels
                int groups = (8 * compute_units() + pbs - 1) / pbs;
                if (groups > plan.n_listed) groups = plan.n_listed;
                if (groups < 1 && plan.n_listed > 0) groups = 1;
                hipLaunchKernelGGL(bin_rows_kernel, dim3(pbs * (groups + plan.n_indexed)), dim3(kBinThreads), 0, st, g, plan,
                                   rec, pos, q, d_enc, d_normal, n, pbs, groups, d_tables);
            }
            const int wgs = compute_units();
            if (plan.n_tasks > 0)
                hipLaunchKernelGGL(scatter_owner_kernel, dim3(plan.n_tasks < wgs ? plan.n_tasks : wgs), dim3(kOwnerThreads), 0,
                                   st, g, plan, rec, pos, q, d_enc, d_normal, n, counter, d_tables);
            if (d_pos && hessian_stored) {
                // the training step's encode kernel left the second derivatives where `part` would go
                const float* hess = reinterpret_cast<const float*>(ws + records_end);
                hipLaunchKernelGGL(pos_from_hessian_kernel, dim3((unsigned)((n + kBlock - 1) / kBlock)), dim3(kBlock), 0, st, hess, q,
                                   d_normal, first_order_pos ? jac : nullptr, first_order_pos ? d_enc : nullptr, g.active_levels, 0, n,
                                   d_pos);
            } else if (d_pos) {
                float* part = reinterpret_cast<float*>(ws + records_end);
                const int pbs = (int)((n + kBlock - 1) / kBlock);
                const LevelSchedule sch = make_level_schedule(g, g.active_levels, pbs);
                const dim3 grid(kXcd * sch.per_xcd);
                if (cfg->table_dtype == 1)
                    hipLaunchKernelGGL(pos_hessian_kernel<__half>, grid, dim3(kBlock), 0, st, g, pos, (const __half*)tables, q,
                                       d_normal, first_order_pos ? d_enc : nullptr, n, sch, part);
                else
                    hipLaunchKernelGGL(pos_hessian_kernel<float>, grid, dim3(kBlock), 0, st, g, pos, (const float*)tables, q,
                                       d_normal, first_order_pos ? d_enc : nullptr, n, sch, part);
                hipLaunchKernelGGL(sum_levels_kernel, dim3((unsigned)((3 * n + kBlock - 1) / kBlock)), dim3(kBlock), 0, st, part,
                                   g.active_levels, n, d_pos);
            }
            return check_launch("hash scatter (owner)");
        }
    }
    const int pbs = (int)((n + kScatterPoints - 1) / kScatterPoints);
    const dim3 grid(grid_blocks(g.active_levels, pbs));
#define NEUS2_SCATTER(T, WP)                                                                   \
    hipLaunchKernelGGL((scatter_kernel<T, WP>), grid, dim3(kBlock), 0, st, g, pos, (const T*)tables, \
                       q, d_enc, d_normal, n, pbs, d_tables, d_pos)
    if (cfg->table_dtype == 1) {
        if (d_pos) NEUS2_SCATTER(__half, true); else NEUS2_SCATTER(__half, false);
    } else {
        if (d_pos) NEUS2_SCATTER(float, true); else NEUS2_SCATTER(float, false);
    }
#undef NEUS2_SCATTER
    return check_launch("hash scatter");
}

}  // namespace neus2
