// Internal interfaces between the translation units of the library.  Not
// installed; the public surface is include/ps_step.h.
#ifndef PS_INTERNAL_H
#define PS_INTERNAL_H

#include <cstdarg>
#include <cstdint>

#include "ps_step.h"

namespace ps {

void set_error(const char *fmt, ...) __attribute__((format(printf, 1, 2)));
void clear_error();
ps_status_t check_spec(const ps_spec_t *s);
ps_status_t shard_geometry(const ps_spec_t *s, uint64_t *psi_padded, uint64_t *offset,
                           uint64_t *len, uint64_t *valid);

// Scalars of one step, binary32, each rounded once from a binary64 value.
struct StepScalars {
    float gs;   // gradient scale (1/N unless the caller overrides it)
    float cc;   // clip coefficient
    float b1, omb1, b2, omb2;
    float ep;
    float step; // lr / (1 - beta1^t)
    float isb2; // 1 / sqrt(1 - beta2^t)
    float lw;   // lr * weight_decay
    const float *cc_device; // when set: the clip coefficient is read from here at run time
    uint32_t out_f16;       // parameters are written as binary16 instead of bf16
};

struct ContribPtrs {
    const void *p[PS_MAX_CONTRIB];
};

// Doubles of workspace the sum-of-squares pass needs for `count` elements: one
// partial per workgroup of the reduce kernel plus a fixed second level.  A pure
// function of the count, so that the reduction tree never depends on the device.
uint64_t reduce_workspace_doubles(uint64_t count);

// Launchers, defined in ps_kernels.hip.  All pointers are DEVICE pointers that
// already point at the first element to process; `count` elements follow.
// They return the hipError_t of the launch as int (0 = success).
// accum: FP32 values added to the contributions' sum (earlier micro-batches), or NULL.
int launch_update(int dtype, uint32_t n_contrib, const ContribPtrs &g, const float *accum,
                  float *master, float *m, float *v, uint16_t *out, uint64_t count,
                  const StepScalars &s, void *stream);
int launch_clip_coef(const double *sumsq_local, const double *sumsq_others, double max_norm,
                     float *coef_out, void *stream);
int launch_reduce_sumsq(int dtype, uint32_t n_contrib, const ContribPtrs &g, float gs,
                        float *reduced_out, uint64_t count, double *partials,
                        double *sumsq_out, int accumulate, void *stream);
// This device's copy of the library's static partial-sum array (looked up on the first
// call per device) and its capacity in doubles; hipError_t as int.
int static_reduce_scratch(double **out, uint64_t *doubles);
int launch_accumulate(int dtype, uint32_t n_contrib, const ContribPtrs &g, float *accum,
                      int overwrite, uint64_t count, void *stream);
// Verification scans.  `slots` 8-byte slots of workspace as verify_workspace_slots() says.
uint64_t verify_workspace_slots(uint64_t bytes);
int launch_diff_sumsq(int dtype, const void *a, const void *b, uint64_t count, double *out2,
                      int accumulate, void *workspace, uint64_t slots, void *stream);
int launch_checksum(const void *buf, uint64_t n_words, uint64_t first_index, uint64_t *out,
                    int accumulate, void *workspace, void *stream);
void set_update_residency(uint32_t waves_per_cu);
int launch_copy(void *dst, const void *src, uint64_t bytes, void *stream);
// Stage one bucket: for each contribution r copy n_vec 16-byte vectors to
// dst + r * slot_stride_bytes from src.p[r], starting at vector first_vec of the
// periodic source (period_vec vectors long).  `alone` says that no other kernel
// runs beside it (it then caps its own residency).
int launch_stage(uint32_t n_contrib, const ContribPtrs &src, void *dst, uint64_t slot_stride_bytes,
                 uint64_t first_vec, uint64_t period_vec, uint64_t n_vec, bool alone, void *stream);

} // namespace ps

#endif
