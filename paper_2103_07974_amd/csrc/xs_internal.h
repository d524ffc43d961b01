// Internal declarations shared by the translation units of libxs.so (host side).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "xs.h"

namespace xs {

// ---- error reporting -------------------------------------------------------
int fail(int status, const char *fmt, ...) __attribute__((format(printf, 2, 3)));
int fail_hip(hipError_t e, const char *what);
void clear_error();

#define XS_HIP_TRY(expr)                                                  \
    do {                                                                  \
        hipError_t _e = (expr);                                           \
        if (_e != hipSuccess) return ::xs::fail_hip(_e, #expr);           \
    } while (0)

inline bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// ---- device facts (of the current device; queried once per device) ---------------
int compute_units();   // > 0, or a negative xs_status

// ---- tuning ---------------------------------------------------------------------
struct Tuning {              // indexed by xs_tuning_key
    int reduce_wg_per_cu;     // 0: one vector per lane, no loop
    int copy_wg_per_cu;       // 0: one work item per workgroup (a few for large LDS tables)
    int nt_grads;             // non-temporal loads of gradient replicas
    int nt_state;             // non-temporal loads and stores of parameters and momentum
    int reduce_lds_reserve;   // bytes of LDS reserved per reduce workgroup (-1: per dtype)
    int reduce_max_wg;        // absolute cap on reduce workgroups (0 = none): background pacing
    int copy_max_wg;          // absolute cap on pack/unpack workgroups (0 = none)
    int copy_nt;              // non-temporal loads and stores in pack/unpack
    int gather_lds_reserve;   // as reduce_lds_reserve, for the gathering form
    int copy_lds_reserve;     // LDS reserved per pack/unpack workgroup beyond its table (-1: default)
};
extern Tuning g_tuning;

// ---- plan -------------------------------------------------------------------------
// Copy work is cut into chunks of kChunkBytes of one tensor's bucket segment
// (tensor plus trailing padding).  chunk_prefix[t] = number of chunks that belong
// to tensors before t; a workgroup finds the tensor of a chunk by binary search
// in a copy of this table held in LDS.
constexpr uint32_t kChunkBytes = 16384;
constexpr uint32_t kCopyThreads = 256;
constexpr uint32_t kLdsPrefixCap = 8192;   // table entries that fit the LDS copy
// The gathering reduce kernel works on rows of kRowBytes of gradient data per replica
// (one 16-byte vector per lane of a wavefront).
constexpr uint32_t kRowBytes = 1024;

struct PlanTables {            // device pointers
    const uint64_t *offsets;   // n_tensors + 1
    const uint64_t *numel;     // n_tensors
    const uint32_t *chunk_prefix;  // n_tensors + 1
    const uint32_t *row_first;     // n_rows: tensor whose segment holds the row's first element
};

}  // namespace xs

struct xs_plan {
    uint32_t magic;
    uint32_t n_tensors;
    int dtype;
    uint32_t elem_size;
    uint64_t bucket_elems;
    uint32_t n_chunks;
    uint64_t n_rows;
    void *dev_blob;            // one allocation holding the tables
    xs::PlanTables tables;
};

static_assert(sizeof(xs_tensor_hparams) == 16, "the kernels read per-tensor records as 16-byte vectors");

constexpr uint32_t XS_PLAN_MAGIC = 0x78735031u;  // "xsP1"
constexpr uint32_t XS_APP_MAGIC = 0x78734131u;   // "xsA1"

namespace xs {
// launchers implemented next to their kernels
int launch_pack(const xs_plan *plan, const void *const *tables /* host array of device tables */,
                void *const *buckets /* host array */, uint32_t n_pairs, int32_t *found_inf,
                hipStream_t stream);
int launch_unpack(const xs_plan *plan, const void *bucket, void *const *tensor_ptrs,
                  hipStream_t stream);
int launch_gather_reduce_sgd(const xs_plan *plan, const void *const *grad_ptrs, uint32_t W,
                             const float *x_in, const float *v_in, float *x_out, float *v_out,
                             void *const *param_ptrs, int view_dtype, const xs_sgd_hparams &hp,
                             const xs_tensor_hparams *tensor_hp, int32_t *found_inf, bool detect,
                             hipStream_t stream);
int launch_reduce_sgd(const void *const *replicas, uint32_t W, int dtype, uint64_t n,
                      const float *x_in, const float *v_in, float *x_out, float *v_out,
                      const xs_sgd_hparams &hp, int32_t *found_inf, bool detect,
                      void *model_copy, int model_copy_dtype, const xs_plan *plan,
                      const xs_tensor_hparams *tensor_hp, hipStream_t stream);
// plan + tensor_hp (both or neither): one (lr, momentum, weight decay) record per tensor of
// the plan replaces hp's three; hp.inv_loss_scale always applies.
}  // namespace xs
