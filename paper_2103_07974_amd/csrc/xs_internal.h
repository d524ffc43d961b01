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
// One launch's settings, indexed by xs_tuning_key.  The process-wide defaults live in
// relaxed atomics (xs_tuning_set may run while another thread launches); every entry point
// takes one snapshot and hands it down, and an xs_app may carry its own copy instead.
struct Tuning {
    int v[XS_TUNE_COUNT];
    int reduce_wg_per_cu() const { return v[XS_TUNE_REDUCE_WG_PER_CU]; }      // 0: one vector per lane, no loop
    int copy_wg_per_cu() const { return v[XS_TUNE_COPY_WG_PER_CU]; }          // 0: one work item per workgroup
    bool nt_grads() const { return v[XS_TUNE_NT_GRADS] != 0; }
    bool nt_state() const { return v[XS_TUNE_NT_STATE] != 0; }
    int reduce_lds_reserve() const { return v[XS_TUNE_REDUCE_LDS_RESERVE]; }  // -1: per dtype
    int reduce_max_wg() const { return v[XS_TUNE_REDUCE_MAX_WG]; }
    int copy_max_wg() const { return v[XS_TUNE_COPY_MAX_WG]; }
    bool copy_nt() const { return v[XS_TUNE_COPY_NT] != 0; }
    int gather_lds_reserve() const { return v[XS_TUNE_GATHER_LDS_RESERVE]; }
    int copy_lds_reserve() const { return v[XS_TUNE_COPY_LDS_RESERVE]; }
    int reduce_waves_per_wg() const { return v[XS_TUNE_REDUCE_WAVES_PER_WG]; }
    bool reduce_small() const { return v[XS_TUNE_REDUCE_SMALL] != 0; }
    int copy_waves_per_wg() const { return v[XS_TUNE_COPY_WAVES_PER_WG]; }
};
Tuning tuning_now();                                   // snapshot of the process-wide settings
int tuning_check(const int32_t *values, Tuning *out);  // XS_OK, or which value is out of range

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
int launch_pack(const Tuning &tn, const xs_plan *plan,
                const void *const *tables /* host array of device tables */,
                void *const *buckets /* host array */, uint32_t n_pairs, int32_t *found_inf,
                hipStream_t stream);
int launch_unpack(const Tuning &tn, const xs_plan *plan, const void *bucket, void *const *tensor_ptrs,
                  hipStream_t stream);
int launch_gather_reduce_sgd(const Tuning &tn, const xs_plan *plan, const void *const *grad_ptrs, uint32_t W,
                             const float *x_in, const float *v_in, float *x_out, float *v_out,
                             void *const *param_ptrs, int view_dtype, const xs_sgd_hparams &hp,
                             const xs_tensor_hparams *tensor_hp, int32_t *found_inf, bool detect,
                             hipStream_t stream);
int launch_reduce_sgd(const Tuning &tn, const void *const *replicas, uint32_t W, int dtype, uint64_t n,
                      const float *x_in, const float *v_in, float *x_out, float *v_out,
                      const xs_sgd_hparams &hp, int32_t *found_inf, bool detect,
                      void *model_copy, int model_copy_dtype, const xs_plan *plan,
                      const xs_tensor_hparams *tensor_hp, void *const *param_ptrs, int view_dtype,
                      hipStream_t stream);
// plan + tensor_hp: one (lr, momentum, weight decay) record per tensor of the plan replaces
// hp's three; hp.inv_loss_scale always applies.  plan + param_ptrs: the updated parameters are
// also written to the per-layer views (element type view_dtype) in the same pass.

// The entry points' argument checks + launch under explicit launch settings (the extern "C"
// functions pass tuning_now(); an xs_app passes its own settings if it has any).
int fuse_pack_many_impl(const Tuning &tn, const xs_plan *plan,
                        const void *const *const *tensor_ptr_tables, void *const *buckets, uint32_t n,
                        int32_t *found_inf, hipStream_t stream);
int fuse_unpack_impl(const Tuning &tn, const xs_plan *plan, const void *bucket,
                     void *const *tensor_ptrs, hipStream_t stream);
int reduce_sgd_impl(const Tuning &tn, const xs_plan *plan, const xs_tensor_hparams *tensor_hp,
                    const void *const *replica_buckets, uint32_t W, int grad_dtype, uint64_t n_elems,
                    float *params, float *momentum, float *params_out, float *momentum_out,
                    const xs_sgd_hparams *hp, int32_t *found_inf, const xs_mp_options *mp,
                    void *const *param_tensor_ptrs, hipStream_t stream);
int reduce_sgd_unpack_impl(const Tuning &tn, const xs_plan *gradient_plan,
                           const void *const *replica_buckets, uint32_t W, float *params, float *momentum,
                           void *const *param_tensor_ptrs, const xs_sgd_hparams *hp,
                           const xs_tensor_hparams *tensor_hp, int32_t *found_inf,
                           const xs_mp_options *mp, hipStream_t stream);
int reduce_sgd_pt_impl(const Tuning &tn, const xs_plan *gradient_plan,
                       const void *const *replica_buckets, uint32_t W, float *params, float *momentum,
                       float *params_out, float *momentum_out, const xs_tensor_hparams *tensor_hp,
                       float inv_loss_scale, int32_t *found_inf, const xs_mp_options *mp,
                       hipStream_t stream);
int gather_reduce_sgd_impl(const Tuning &tn, const xs_plan *gradient_plan, const void *const *grad_ptrs,
                           uint32_t W, float *params, float *momentum, float *params_out,
                           float *momentum_out, void *const *param_tensor_ptrs,
                           const xs_sgd_hparams *hp, const xs_tensor_hparams *tensor_hp,
                           int32_t *found_inf, const xs_mp_options *mp, hipStream_t stream);
}  // namespace xs
