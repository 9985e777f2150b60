// Internal declarations shared by the translation units of libneus2 (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>
#include <stdint.h>

#include "../../include/neus2.h"

namespace neus2 {

// ---- host side ---------------------------------------------------------------------------
int fail(int code, const char* fmt, ...);           // records the message, returns code
int check_config(const neus2_config* cfg);
int check_ptr(const void* p, const char* name, bool required = true);
int check_launch(const char* what);                  // hipGetLastError -> NEUS2_ERR_HIP

#define NEUS2_TRY(expr)                 \
    do {                                \
        int _rc = (expr);               \
        if (_rc != NEUS2_OK) return _rc; \
    } while (0)

// ---- kernel-side descriptor of the grid ----------------------------------------------------
struct GridDesc {
    int n_levels;
    int active_levels;
    int frozen_levels;         // levels below this get no table gradient
    uint32_t table_mask;       // T - 1
    uint32_t table_size;       // T
    uint32_t dense_bits;       // bit l set: level l is dense
    int res[NEUS2_MAX_LEVELS];
};

GridDesc make_grid_desc(const neus2_config* cfg);

// Number of compute units, cached per process.
int compute_units();

// Grid size of a persistent kernel: as many workgroups as can be resident at once, but no
// more than `want`.
int persistent_blocks(const void* kernel, int threads, int64_t want);

int launch_zero(float* p, int64_t count, hipStream_t st);

// Up to two small regions that the first kernel of a training step clears on its way, instead
// of a launch of their own each (the loss sums, the header of the scatter's workspace).
struct ZeroRegions {
    float* p[2];
    int count[2];
};

// internal launchers (each validates nothing; the extern "C" wrappers do)
int launch_encode(const neus2_config* cfg, const float* pos, const void* tables, int64_t n,
                  float* enc, float* jac, uint32_t* dbg_idx, hipStream_t st, const ZeroRegions* zero = nullptr,
                  float* hess = nullptr, bool active_only = false);
// first_order_pos: d_pos also gets J^T d_enc (the part the SDF backward kernel adds when it is
// handed d_pos); only honoured on the path scatter_gathers_position() reports.
int launch_scatter(const neus2_config* cfg, const float* pos, const void* tables, const float* q,
                   const float* d_enc, const float* d_normal, int64_t n, float* d_tables,
                   float* d_pos, void* workspace, int64_t workspace_bytes, bool first_order_pos, hipStream_t st,
                   bool header_cleared = false, bool hessian_stored = false, const float* jac = nullptr);
// Where a training step that wants d_pos has its encode kernel write the mixed second derivatives of the
// interpolation (launch_encode's `hess`, [active levels][3][n][2] floats inside the workspace), so that
// launch_scatter(hessian_stored = true) needs no second gather for them; nullptr if the scatter-add will
// not take the path with the workspace.
float* scatter_hessian_region(const neus2_config* cfg, int64_t n, void* workspace, int64_t workspace_bytes);
// The part of the workspace launch_scatter needs cleared before it runs (task counter and list
// cursors) if it will take the path that uses the workspace with these arguments, else count 0.
void scatter_header(const neus2_config* cfg, int64_t n, bool want_pos, void* workspace, int64_t workspace_bytes,
                    float** p, int* count);
bool scatter_gathers_position(const neus2_config* cfg, int64_t n, const void* workspace, int64_t workspace_bytes);
int64_t scatter_workspace_bytes(const neus2_config* cfg, int64_t n);
// Bytes of workspace the scatter-add needs for n points when no position gradient is wanted
// (0 if it would take the path without a workspace).
int64_t scatter_records_bytes(const neus2_config* cfg, int64_t n);
int64_t sdf_deep_workspace_bytes(int n_mats, int64_t n);
int launch_sdf_deep_fwd(int n_mats, int enc_dim, const float* enc, const float* jac, const float* const* H, int64_t n,
                        float* y, float* q, float* normal, void* workspace, hipStream_t st);
int launch_sdf_deep_bwd(int n_mats, int enc_dim, const float* enc, const float* jac, const float* const* H,
                        const float* d_y, const float* d_normal, int64_t n, float* const* dH, float* d_enc,
                        void* workspace, hipStream_t st);
int launch_sdf_fwd(const neus2_config* cfg, const float* enc, const float* jac,
                   const float* const* H, int64_t n, float* y, float* q, float* normal, uint32_t* masks, hipStream_t st);
int launch_sdf_bwd(const neus2_config* cfg, const float* enc, const float* jac,
                   const float* const* H, const float* d_y, const float* d_normal, int64_t n,
                   float* const* dH, float* d_enc, float* d_pos, const uint32_t* masks, hipStream_t st);

}  // namespace neus2
