// Host side of the C ABI: argument validation, error reporting, and the calls that are
// sequences of the kernels in the other translation units.
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <map>
#include <mutex>
#include <utility>

#include "common.h"

namespace neus2 {

namespace {
thread_local char g_error[512] = "";
}

int fail(int code, const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_error, sizeof(g_error), fmt, ap);
    va_end(ap);
    return code;
}

int check_ptr(const void* p, const char* name, bool required) {
    if (!p) return required ? fail(NEUS2_ERR_NULL, "%s is NULL", name) : NEUS2_OK;
    if ((reinterpret_cast<uintptr_t>(p) & 15u) != 0) return fail(NEUS2_ERR_ALIGN, "%s is not 16-byte aligned", name);
    return NEUS2_OK;
}

int check_launch(const char* what) {
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(NEUS2_ERR_HIP, "%s: %s", what, hipGetErrorString(e));
    return NEUS2_OK;
}

int compute_units() {
    static int cus = 0;
    if (cus == 0) {
        int dev = 0, v = 0;
        if (hipGetDevice(&dev) == hipSuccess &&
            hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && v > 0)
            cus = v;
        else
            cus = 256;
    }
    return cus;
}

int persistent_blocks(const void* kernel, int threads, int64_t want) {
    // the occupancy query costs several microseconds of host time; its answer never changes
    static std::mutex mu;
    static std::map<std::pair<const void*, int>, int> cache;
    int per_cu = 0;
    {
        std::lock_guard<std::mutex> lock(mu);
        auto it = cache.find({kernel, threads});
        if (it != cache.end()) per_cu = it->second;
    }
    if (per_cu == 0) {
        per_cu = 1;
        if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, kernel, threads, 0) != hipSuccess || per_cu < 1) {
            (void)hipGetLastError();
            per_cu = 1;
        }
        std::lock_guard<std::mutex> lock(mu);
        cache[{kernel, threads}] = per_cu;
    }
    const int64_t cap = (int64_t)per_cu * compute_units();
    const int64_t b = want < cap ? want : cap;
    return (int)(b < 1 ? 1 : b);
}

int check_config(const neus2_config* c) {
    if (!c) return fail(NEUS2_ERR_NULL, "cfg is NULL");
    if (c->n_levels < 1 || c->n_levels > NEUS2_MAX_LEVELS)
        return fail(NEUS2_ERR_CONFIG, "n_levels = %d, must be 1..%d", c->n_levels, NEUS2_MAX_LEVELS);
    if (c->n_features != 2) return fail(NEUS2_ERR_UNSUPPORTED, "n_features = %d, only 2 is built", c->n_features);
    if (c->log2_table_size < 4 || c->log2_table_size > 24)
        return fail(NEUS2_ERR_CONFIG, "log2_table_size = %d, must be 4..24", c->log2_table_size);
    if (c->active_levels < 0 || c->active_levels > c->n_levels)
        return fail(NEUS2_ERR_CONFIG, "active_levels = %d outside 0..n_levels", c->active_levels);
    if (c->table_dtype != 0 && c->table_dtype != 1)
        return fail(NEUS2_ERR_CONFIG, "table_dtype = %d, must be 0 (fp32) or 1 (fp16)", c->table_dtype);
    const int64_t T = (int64_t)1 << c->log2_table_size;
    for (int l = 0; l < c->n_levels; ++l) {
        const int64_t r = c->res[l];
        if (r < 1 || r > (1 << 20)) return fail(NEUS2_ERR_CONFIG, "res[%d] = %d, must be 1..2^20", l, (int)r);
        if (c->dense[l] != 0 && c->dense[l] != 1) return fail(NEUS2_ERR_CONFIG, "dense[%d] must be 0 or 1", l);
        if (c->dense[l] && (r + 1) * (r + 1) * (r + 1) > T)
            return fail(NEUS2_ERR_CONFIG, "level %d is marked dense but (res+1)^3 = %lld exceeds T = %lld", l,
                        (long long)((r + 1) * (r + 1) * (r + 1)), (long long)T);
    }
    if (c->n_sdf_mats != 2 && c->n_sdf_mats != 3)
        return fail(NEUS2_ERR_UNSUPPORTED, "n_sdf_mats = %d, kernels exist for 2 and 3", c->n_sdf_mats);
    if (c->sdf_dims[0] != c->n_levels * c->n_features)
        return fail(NEUS2_ERR_CONFIG, "sdf_dims[0] = %d must equal n_levels * n_features = %d", c->sdf_dims[0],
                    c->n_levels * c->n_features);
    if (c->sdf_dims[0] != 16 && c->sdf_dims[0] != 32)
        return fail(NEUS2_ERR_UNSUPPORTED, "encoding width %d, kernels exist for 16 and 32", c->sdf_dims[0]);
    for (int l = 1; l < c->n_sdf_mats; ++l)
        if (c->sdf_dims[l] != 64) return fail(NEUS2_ERR_UNSUPPORTED, "sdf hidden width %d, only 64 is built", c->sdf_dims[l]);
    if (c->sdf_dims[c->n_sdf_mats] != 16)
        return fail(NEUS2_ERR_UNSUPPORTED, "sdf output width %d, must be 16 (d and 15 features)", c->sdf_dims[c->n_sdf_mats]);
    if (c->n_color_mats != 0) {
        if (c->n_color_mats != 3 || c->color_dims[0] != 38 || c->color_dims[1] != 64 || c->color_dims[2] != 64 ||
            c->color_dims[3] != 3)
            return fail(NEUS2_ERR_UNSUPPORTED, "colour network must be 38-64-64-3 (or absent)");
    }
    if (c->samples_per_ray < 1 || c->samples_per_ray > 64)
        return fail(NEUS2_ERR_CONFIG, "samples_per_ray = %d, must be 1..64", c->samples_per_ray);
    if (c->loss_kind < 0 || c->loss_kind > 2) return fail(NEUS2_ERR_CONFIG, "loss_kind = %d, must be 0, 1 or 2", c->loss_kind);
    if (c->loss_kind == 2 && !(c->huber_delta > 0.f)) return fail(NEUS2_ERR_CONFIG, "huber_delta must be positive for loss_kind 2");
    if (c->frozen_levels < 0 || c->frozen_levels > c->n_levels)
        return fail(NEUS2_ERR_CONFIG, "frozen_levels = %d outside 0..n_levels", c->frozen_levels);
    if (!(c->s > 0.f)) return fail(NEUS2_ERR_CONFIG, "s must be positive");
    if (!(c->beta >= 0.f)) return fail(NEUS2_ERR_CONFIG, "beta must be non-negative");
    return NEUS2_OK;
}

GridDesc make_grid_desc(const neus2_config* cfg) {
    GridDesc g;
    memset(&g, 0, sizeof(g));
    g.n_levels = cfg->n_levels;
    g.active_levels = cfg->active_levels;
    g.frozen_levels = cfg->frozen_levels;
    g.table_size = 1u << cfg->log2_table_size;
    g.table_mask = g.table_size - 1u;
    for (int l = 0; l < cfg->n_levels; ++l) {
        g.res[l] = cfg->res[l];
        if (cfg->dense[l]) g.dense_bits |= 1u << l;
    }
    return g;
}

int check_count(int64_t n, const char* name) {
    if (n < 0) return fail(NEUS2_ERR_SHAPE, "%s = %lld is negative", name, (long long)n);
    if (n > ((int64_t)1 << 28)) return fail(NEUS2_ERR_SHAPE, "%s = %lld exceeds 2^28", name, (long long)n);
    return NEUS2_OK;
}

int check_mats(const void* const* M, int count, const char* name) {
    if (!M) return fail(NEUS2_ERR_NULL, "%s is NULL", name);
    char buf[32];
    for (int l = 0; l < count; ++l) {
        snprintf(buf, sizeof(buf), "%s[%d]", name, l);
        NEUS2_TRY(check_ptr(M[l], buf));
    }
    return NEUS2_OK;
}

}  // namespace neus2

using namespace neus2;

namespace {

// SDF backward + scatter-add; header_cleared: the caller has had the workspace header cleared
int sdf_bwd_2nd(const neus2_config* cfg, const float* pos, const void* tables, const float* enc,
                const float* jac, const float* const* H, const float* q, const float* d_y,
                const float* d_normal, int64_t n, float* const* dH, float* d_tables, float* d_enc,
                float* d_pos, void* workspace, int64_t workspace_bytes, bool header_cleared, const uint32_t* masks,
                void* stream, bool hessian_stored = false) {
    NEUS2_TRY(check_config(cfg));
    NEUS2_TRY(check_count(n, "n"));
    NEUS2_TRY(check_ptr(workspace, "workspace", false));
    NEUS2_TRY(check_ptr(pos, "pos"));
    NEUS2_TRY(check_ptr(tables, "tables"));
    NEUS2_TRY(check_ptr(enc, "enc"));
    NEUS2_TRY(check_ptr(jac, "jac"));
    NEUS2_TRY(check_mats((const void* const*)H, cfg->n_sdf_mats, "H"));
    NEUS2_TRY(check_ptr(q, "q"));
    NEUS2_TRY(check_ptr(d_y, "d_y"));
    NEUS2_TRY(check_ptr(d_normal, "d_normal"));
    NEUS2_TRY(check_mats((const void* const*)dH, cfg->n_sdf_mats, "dH"));
    NEUS2_TRY(check_ptr(d_tables, "d_tables"));
    NEUS2_TRY(check_ptr(d_enc, "d_enc"));
    NEUS2_TRY(check_ptr(d_pos, "d_pos", false));
    NEUS2_TRY(check_ptr(masks, "masks", false));
    hipStream_t st = (hipStream_t)stream;
    // With a large batch and a workspace the scatter's gather pass has the corners of every level
    // in registers and adds (de/dx)^T dL/de to d_pos on the way; otherwise the network kernel
    // does it from the stored Jacobian.
    // In a training step the encode kernel has stored the second derivatives of the interpolation
    // (hessian_stored): then one streaming kernel adds both parts from the stored arrays.
    const bool gather = d_pos && (hessian_stored || scatter_gathers_position(cfg, n, workspace, workspace_bytes));
    NEUS2_TRY(launch_sdf_bwd(cfg, enc, jac, H, d_y, d_normal, n, dH, d_enc, gather ? nullptr : d_pos, masks, st));
    return launch_scatter(cfg, pos, tables, q, d_enc, d_normal, n, d_tables, d_pos, workspace, workspace_bytes, gather, st,
                          header_cleared, hessian_stored, jac);
}

}  // namespace

extern "C" {

const char* neus2_last_error(void) { return g_error; }
int neus2_version(void) { return 1; }
int neus2_validate_config(const neus2_config* cfg) { return check_config(cfg); }

int64_t neus2_workspace_bytes(const neus2_config* cfg, int64_t n) {
    if (check_config(cfg) != NEUS2_OK || n < 0) return -1;
    return scatter_workspace_bytes(cfg, n);
}

int neus2_hash_encode(const neus2_config* cfg, const float* pos, const void* tables, int64_t n, float* enc,
                      float* jac, uint32_t* dbg_idx, void* stream) {
    NEUS2_TRY(check_config(cfg));
    NEUS2_TRY(check_count(n, "n"));
    NEUS2_TRY(check_ptr(pos, "pos"));
    NEUS2_TRY(check_ptr(tables, "tables"));
    NEUS2_TRY(check_ptr(enc, "enc"));
    NEUS2_TRY(check_ptr(jac, "jac"));
    NEUS2_TRY(check_ptr(dbg_idx, "dbg_idx", false));
    return launch_encode(cfg, pos, tables, n, enc, jac, dbg_idx, (hipStream_t)stream);
}

int neus2_sdf_fwd_grad(const neus2_config* cfg, const float* enc, const float* jac, const float* const* H,
                       int64_t n, float* y, float* q, float* normal, uint32_t* masks, void* stream) {
    NEUS2_TRY(check_config(cfg));
    NEUS2_TRY(check_count(n, "n"));
    NEUS2_TRY(check_ptr(enc, "enc"));
    NEUS2_TRY(check_ptr(jac, "jac"));
    NEUS2_TRY(check_mats((const void* const*)H, cfg->n_sdf_mats, "H"));
    NEUS2_TRY(check_ptr(y, "y"));
    NEUS2_TRY(check_ptr(q, "q"));
    NEUS2_TRY(check_ptr(normal, "normal"));
    NEUS2_TRY(check_ptr(masks, "masks", false));
    return launch_sdf_fwd(cfg, enc, jac, H, n, y, q, normal, masks, (hipStream_t)stream);
}

static int check_deep(int n_mats, int enc_dim, int64_t n, const void* workspace, int64_t workspace_bytes) {
    if (n_mats < 2 || n_mats > NEUS2_DEEP_MAX_MATS)
        return fail(NEUS2_ERR_UNSUPPORTED, "layer-by-layer sdf network: %d matrices (2..%d are built)", n_mats, NEUS2_DEEP_MAX_MATS);
    if (enc_dim != 16 && enc_dim != 32)
        return fail(NEUS2_ERR_UNSUPPORTED, "layer-by-layer sdf network: input width %d (16 and 32 are built)", enc_dim);
    NEUS2_TRY(check_count(n, "n"));
    NEUS2_TRY(check_ptr(workspace, "workspace"));
    if (workspace_bytes < sdf_deep_workspace_bytes(n_mats, n))
        return fail(NEUS2_ERR_SHAPE, "workspace of %lld bytes, neus2_sdf_deep_workspace_bytes asks for %lld", (long long)workspace_bytes,
                    (long long)sdf_deep_workspace_bytes(n_mats, n));
    return NEUS2_OK;
}

int64_t neus2_sdf_deep_workspace_bytes(int32_t n_mats, int64_t n) {
    if (n_mats < 2 || n_mats > NEUS2_DEEP_MAX_MATS || n < 0) return -1;
    return sdf_deep_workspace_bytes(n_mats, n);
}

int neus2_sdf_deep_fwd_grad(int32_t n_mats, int32_t enc_dim, const float* enc, const float* jac, const float* const* H,
                            int64_t n, float* y, float* q, float* normal, void* workspace, int64_t workspace_bytes,
                            void* stream) {
    NEUS2_TRY(check_deep(n_mats, enc_dim, n, workspace, workspace_bytes));
    NEUS2_TRY(check_ptr(enc, "enc"));
    NEUS2_TRY(check_ptr(jac, "jac"));
    NEUS2_TRY(check_mats((const void* const*)H, n_mats, "H"));
    NEUS2_TRY(check_ptr(y, "y"));
    NEUS2_TRY(check_ptr(q, "q"));
    NEUS2_TRY(check_ptr(normal, "normal"));
    return launch_sdf_deep_fwd(n_mats, enc_dim, enc, jac, H, n, y, q, normal, workspace, (hipStream_t)stream);
}

int neus2_sdf_deep_bwd(int32_t n_mats, int32_t enc_dim, const float* enc, const float* jac, const float* const* H,
                       const float* d_y, const float* d_normal, int64_t n, float* const* dH, float* d_enc,
                       void* workspace, int64_t workspace_bytes, void* stream) {
    NEUS2_TRY(check_deep(n_mats, enc_dim, n, workspace, workspace_bytes));
    NEUS2_TRY(check_ptr(enc, "enc"));
    NEUS2_TRY(check_ptr(jac, "jac"));
    NEUS2_TRY(check_mats((const void* const*)H, n_mats, "H"));
    NEUS2_TRY(check_ptr(d_y, "d_y"));
    NEUS2_TRY(check_ptr(d_normal, "d_normal"));
    NEUS2_TRY(check_mats((const void* const*)dH, n_mats, "dH"));
    NEUS2_TRY(check_ptr(d_enc, "d_enc"));
    return launch_sdf_deep_bwd(n_mats, enc_dim, enc, jac, H, d_y, d_normal, n, dH, d_enc, workspace, (hipStream_t)stream);
}

int neus2_sdf_mlp_bwd(const neus2_config* cfg, const float* enc, const float* jac, const float* const* H,
                      const float* d_y, const float* d_normal, int64_t n, float* const* dH, float* d_enc,
                      float* d_pos, const uint32_t* masks, void* stream) {
    NEUS2_TRY(check_config(cfg));
    NEUS2_TRY(check_count(n, "n"));
    NEUS2_TRY(check_ptr(enc, "enc"));
    NEUS2_TRY(check_ptr(jac, "jac"));
    NEUS2_TRY(check_mats((const void* const*)H, cfg->n_sdf_mats, "H"));
    NEUS2_TRY(check_ptr(d_y, "d_y"));
    NEUS2_TRY(check_ptr(d_normal, "d_normal"));
    NEUS2_TRY(check_mats((const void* const*)dH, cfg->n_sdf_mats, "dH"));
    NEUS2_TRY(check_ptr(d_enc, "d_enc"));
    NEUS2_TRY(check_ptr(d_pos, "d_pos", false));
    NEUS2_TRY(check_ptr(masks, "masks", false));
    return launch_sdf_bwd(cfg, enc, jac, H, d_y, d_normal, n, dH, d_enc, d_pos, masks, (hipStream_t)stream);
}

int neus2_hash_scatter_bwd(const neus2_config* cfg, const float* pos, const void* tables, const float* q,
                           const float* d_enc, const float* d_normal, int64_t n, float* d_tables, float* d_pos,
                           void* workspace, int64_t workspace_bytes, void* stream) {
    NEUS2_TRY(check_config(cfg));
    NEUS2_TRY(check_count(n, "n"));
    NEUS2_TRY(check_ptr(pos, "pos"));
    NEUS2_TRY(check_ptr(tables, "tables"));
    NEUS2_TRY(check_ptr(q, "q"));
    NEUS2_TRY(check_ptr(d_enc, "d_enc"));
    NEUS2_TRY(check_ptr(d_normal, "d_normal"));
    NEUS2_TRY(check_ptr(d_tables, "d_tables"));
    NEUS2_TRY(check_ptr(d_pos, "d_pos", false));
    NEUS2_TRY(check_ptr(workspace, "workspace", false));
    return launch_scatter(cfg, pos, tables, q, d_enc, d_normal, n, d_tables, d_pos, workspace, workspace_bytes, false,
                          (hipStream_t)stream);
}

int neus2_sdf_bwd_2nd(const neus2_config* cfg, const float* pos, const void* tables, const float* enc,
                      const float* jac, const float* const* H, const float* q, const float* d_y,
                      const float* d_normal, int64_t n, float* const* dH, float* d_tables, float* d_enc,
                      float* d_pos, void* workspace, int64_t workspace_bytes, const uint32_t* masks, void* stream) {
    return sdf_bwd_2nd(cfg, pos, tables, enc, jac, H, q, d_y, d_normal, n, dH, d_tables, d_enc, d_pos, workspace,
                       workspace_bytes, false, masks, stream);
}

}  // extern "C"

// ---- scatter-add for callers that cannot allocate ----------------------------------------------
// The record lists of the scatter-add live in a file-scope device array instead of a caller's
// workspace.  Each GPU the library runs on holds its own copy of the array until the process
// ends; its address on a device is looked up once, with that device current, and from then on
// host code only ever uses that address (the array's name is not a device address on the host).
static __device__ __align__(256) unsigned char scratch[NEUS2_STATIC_SCRATCH_BYTES];

namespace {

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices] = {};

// the device's copy of `scratch`; nullptr and an error message if the runtime refuses
void* static_scratch() {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) {
        (void)hipGetLastError();
        fail(NEUS2_ERR_HIP, "no current device (or its number is beyond %d)", kMaxDevices - 1);
        return nullptr;
    }
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* ptr = nullptr;
        const hipError_t e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !ptr) {
            (void)hipGetLastError();
            fail(NEUS2_ERR_HIP, "address of the static scratch array on device %d: %s", dev, hipGetErrorString(e));
            return nullptr;
        }
        g_scratch_ptr[dev] = ptr;
    }
    return g_scratch_ptr[dev];
}

}  // namespace

extern "C" int neus2_hash_scatter_bwd_static(const neus2_config* cfg, const float* pos, const void* tables, const float* q,
                                             const float* d_enc, const float* d_normal, int64_t n, float* d_tables,
                                             void* stream) {
    NEUS2_TRY(check_config(cfg));
    NEUS2_TRY(check_count(n, "n"));
    NEUS2_TRY(check_ptr(pos, "pos"));
    NEUS2_TRY(check_ptr(tables, "tables"));
    NEUS2_TRY(check_ptr(q, "q"));
    NEUS2_TRY(check_ptr(d_enc, "d_enc"));
    NEUS2_TRY(check_ptr(d_normal, "d_normal"));
    NEUS2_TRY(check_ptr(d_tables, "d_tables"));
    const int64_t need = scatter_records_bytes(cfg, n);
    if (need > (int64_t)NEUS2_STATIC_SCRATCH_BYTES)
        return fail(NEUS2_ERR_SHAPE, "n = %lld points with this descriptor need %lld bytes of scratch, the static buffer holds %lld",
                    (long long)n, (long long)need, (long long)NEUS2_STATIC_SCRATCH_BYTES);
    void* ws = nullptr;
    if (need > 0) {
        ws = static_scratch();
        if (!ws) return NEUS2_ERR_HIP;
    }
    // the header of the buffer (task counter, list cursors) is cleared by a fill kernel inside; the
    // lists themselves are overwritten up to the cursors, so the last call's contents do not matter
    return launch_scatter(cfg, pos, tables, q, d_enc, d_normal, n, d_tables, nullptr, ws, ws ? (int64_t)NEUS2_STATIC_SCRATCH_BYTES : 0,
                          false, (hipStream_t)stream);
}

namespace {

// Every field of the step's buffers that the chosen path will read or write, checked before the
// first launch: a call that fails here has touched no device memory.
int check_step_buffers(const neus2_config* cfg, const neus2_step_buffers* b, int64_t n, bool ragged) {
    NEUS2_TRY(check_ptr(b->loss, "loss"));
    NEUS2_TRY(check_ptr(b->workspace, "workspace", false));
    if (ragged) {
        NEUS2_TRY(check_ptr(b->target, "target"));
        NEUS2_TRY(check_ptr(b->C, "C"));
        NEUS2_TRY(check_ptr(b->dC, "dC"));
        NEUS2_TRY(check_ptr(b->s_dev, "s_dev", false));
        NEUS2_TRY(check_ptr(b->d_s, "d_s", false));
    }
    if (n == 0) return NEUS2_OK;
    NEUS2_TRY(check_ptr(b->pos, "pos"));
    NEUS2_TRY(check_ptr(b->tables, "tables"));
    NEUS2_TRY(check_ptr(b->enc, "enc"));
    NEUS2_TRY(check_ptr(b->jac, "jac"));
    NEUS2_TRY(check_mats((const void* const*)b->H, cfg->n_sdf_mats, "H"));
    NEUS2_TRY(check_ptr(b->y, "y"));
    NEUS2_TRY(check_ptr(b->q, "q"));
    NEUS2_TRY(check_ptr(b->normal, "normal"));
    NEUS2_TRY(check_ptr(b->sdf_masks, "sdf_masks", false));
    NEUS2_TRY(check_ptr(b->d_y, "d_y"));
    NEUS2_TRY(check_ptr(b->d_normal, "d_normal"));
    NEUS2_TRY(check_ptr(b->d_enc, "d_enc"));
    NEUS2_TRY(check_ptr(b->d_pos, "d_pos", false));
    NEUS2_TRY(check_mats((const void* const*)b->dH, cfg->n_sdf_mats, "dH"));
    NEUS2_TRY(check_ptr(b->d_tables, "d_tables"));
    if (cfg->loss_kind != 0) {
        NEUS2_TRY(check_ptr(b->dirs, "dirs"));
        NEUS2_TRY(check_ptr(b->target, "target"));
        NEUS2_TRY(check_mats((const void* const*)b->W, 3, "W"));
        NEUS2_TRY(check_ptr(b->rgb, "rgb"));
        NEUS2_TRY(check_ptr(b->color_masks, "color_masks", false));
        NEUS2_TRY(check_ptr(b->C, "C"));
        NEUS2_TRY(check_ptr(b->weights, "weights"));
        NEUS2_TRY(check_ptr(b->dC, "dC"));
        NEUS2_TRY(check_ptr(b->d_sdf, "d_sdf"));
        NEUS2_TRY(check_ptr(b->d_rgb, "d_rgb"));
        NEUS2_TRY(check_mats((const void* const*)b->dW, 3, "dW"));
        NEUS2_TRY(check_ptr(b->s_dev, "s_dev", false));
        NEUS2_TRY(check_ptr(b->d_s, "d_s", false));
    }
    return NEUS2_OK;
}

}  // namespace

extern "C" int neus2_train_step(const neus2_config* cfg, const neus2_step_buffers* b, int64_t n, void* stream) {
    NEUS2_TRY(check_config(cfg));
    if (!b) return fail(NEUS2_ERR_NULL, "buf is NULL");
    const bool ragged = b->ray_offsets != nullptr;
    if (ragged != (b->sample_ray != nullptr)) return fail(NEUS2_ERR_NULL, "ray_offsets and sample_ray go together");
    if (ragged && cfg->loss_kind == 0) return fail(NEUS2_ERR_CONFIG, "loss_kind 0 has no rays");
    NEUS2_TRY(check_count(n, "n"));
    if (!ragged && n % cfg->samples_per_ray != 0)
        return fail(NEUS2_ERR_SHAPE, "n = %lld is not a multiple of samples_per_ray = %d", (long long)n, cfg->samples_per_ray);
    if (ragged && (b->n_rays < 0 || b->n_rays > ((int64_t)1 << 28)))
        return fail(NEUS2_ERR_SHAPE, "n_rays = %lld out of range", (long long)b->n_rays);
    if (cfg->loss_kind != 0 && cfg->n_color_mats != 3)
        return fail(NEUS2_ERR_CONFIG, "loss_kind %d needs the colour network", cfg->loss_kind);
    NEUS2_TRY(check_step_buffers(cfg, b, n, ragged));
    hipStream_t st = (hipStream_t)stream;
    const int64_t rays = ragged ? b->n_rays : n / cfg->samples_per_ray;
    if (n == 0) {                  // an empty batch has no sample buffers to look at
        NEUS2_TRY(launch_zero(b->loss, 2, st));
        if (ragged && rays > 0)    // rays without samples still enter the colour term
            return neus2_render_loss_bwd_ragged(cfg, nullptr, nullptr, nullptr, b->target, b->ray_offsets, b->s_dev, rays, 0,
                                                b->C, nullptr, b->loss, b->dC, nullptr, nullptr, nullptr, b->d_s, stream);
        return NEUS2_OK;
    }
    // the encode kernel, first of the step, also clears the loss sums and the header of the scatter's
    // workspace: two launches fewer
    ZeroRegions zero = {{b->loss, nullptr}, {2, 0}};
    scatter_header(cfg, n, b->d_pos != nullptr, b->workspace, b->workspace_bytes, &zero.p[1], &zero.count[1]);
    // a step that wants d_pos: the encode kernel also leaves the second derivatives of the interpolation in
    // the workspace, behind the scatter's records, where the backward pass streams them
    float* hess = b->d_pos ? scatter_hessian_region(cfg, n, b->workspace, b->workspace_bytes) : nullptr;
    NEUS2_TRY(launch_encode(cfg, b->pos, b->tables, n, b->enc, b->jac, nullptr, st, &zero, hess, true));
    NEUS2_TRY(neus2_sdf_fwd_grad(cfg, b->enc, b->jac, b->H, n, b->y, b->q, b->normal, b->sdf_masks, stream));
    if (cfg->loss_kind != 0) {
        NEUS2_TRY(neus2_color_fwd(cfg, b->pos, b->normal, b->dirs, b->sample_ray, b->y, b->W, n, b->rgb, b->color_masks, stream));
        if (ragged)
            NEUS2_TRY(neus2_render_loss_bwd_ragged(cfg, b->y, b->rgb, b->normal, b->target, b->ray_offsets, b->s_dev, rays, n,
                                                   b->C, b->weights, b->loss, b->dC, b->d_sdf, b->d_rgb, b->d_normal, b->d_s,
                                                   stream));
        else
            NEUS2_TRY(neus2_render_loss_bwd(cfg, b->y, b->rgb, b->normal, b->target, b->s_dev, rays, b->C, b->weights, b->loss,
                                            b->dC, b->d_sdf, b->d_rgb, b->d_normal, b->d_s, stream));
        NEUS2_TRY(neus2_color_bwd(cfg, b->pos, b->normal, b->dirs, b->sample_ray, b->y, b->W, b->rgb, b->d_rgb, b->d_sdf, n, b->dW, b->d_y,
                                  b->d_normal, b->d_pos, b->color_masks, stream));
    } else {
        NEUS2_TRY(neus2_loss(cfg, nullptr, nullptr, b->normal, b->y, 0, n, b->loss, nullptr, b->d_normal, b->d_y, stream));
        if (b->d_pos) NEUS2_TRY(launch_zero(b->d_pos, 3 * n, st));
    }
    return sdf_bwd_2nd(cfg, b->pos, b->tables, b->enc, b->jac, b->H, b->q, b->d_y, b->d_normal, n, b->dH,
                       b->d_tables, b->d_enc, b->d_pos, b->workspace, b->workspace_bytes, zero.count[1] > 0, b->sdf_masks,
                       stream, hess != nullptr);
}
