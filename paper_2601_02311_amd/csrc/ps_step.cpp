// Device-facing entry points: argument validation (always before the first HIP
// call), derivation of the step's binary32 scalars, and the bucket pipeline.
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstring>
#include <vector>

#include "ps_internal.h"

using namespace ps;

namespace {

bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

ps_status_t hip_fail(hipError_t e, const char *what)
{
    if (e == hipErrorNoDevice || e == hipErrorInvalidDevice || e == hipErrorInsufficientDriver) {
        set_error("%s: %s", what, hipGetErrorString(e));
        return PS_ENODEVICE;
    }
    set_error("%s: %s", what, hipGetErrorString(e));
    return PS_EHIP;
}

ps_status_t need_device()
{
    int n = 0;
    hipError_t e = hipGetDeviceCount(&n);
    if (e != hipSuccess || n <= 0) {
        (void)hipGetLastError();
        set_error("no HIP device (%s)", e == hipSuccess ? "count is 0" : hipGetErrorString(e));
        return PS_ENODEVICE;
    }
    return PS_OK;
}

// beta^t for t up to 2^64-1 through the C library's pow in binary64.
StepScalars derive_scalars(const ps_adamw_t &hp, uint32_t n_devices, int32_t param_dtype)
{
    const double bias1 = 1.0 - std::pow(hp.beta1, (double)hp.step);
    const double bias2 = 1.0 - std::pow(hp.beta2, (double)hp.step);
    StepScalars s;
    s.gs = (float)(hp.grad_scale > 0.0 ? hp.grad_scale : 1.0 / (double)n_devices);
    s.cc = (float)(hp.clip_coef > 0.0 ? hp.clip_coef : 1.0);
    s.b1 = (float)hp.beta1;
    s.omb1 = (float)(1.0 - hp.beta1);
    s.b2 = (float)hp.beta2;
    s.omb2 = (float)(1.0 - hp.beta2);
    s.ep = (float)hp.eps;
    s.step = (float)(hp.lr / bias1);
    s.isb2 = (float)(1.0 / std::sqrt(bias2));
    s.lw = (float)(hp.lr * hp.weight_decay);
    s.cc_device = hp.clip_coef_device;
    s.out_f16 = param_dtype == PS_F16;
    return s;
}

ps_status_t check_hp(const ps_adamw_t *hp)
{
    if (!hp) {
        set_error("hyper-parameters are NULL");
        return PS_EINVAL;
    }
    if (hp->step == 0) {
        set_error("step count t must be >= 1");
        return PS_ERANGE;
    }
    if (!(hp->beta1 >= 0.0 && hp->beta1 < 1.0) || !(hp->beta2 >= 0.0 && hp->beta2 < 1.0)) {
        set_error("beta1 and beta2 must lie in [0, 1)");
        return PS_ERANGE;
    }
    if (!(hp->lr >= 0.0) || !(hp->eps >= 0.0) || !(hp->weight_decay >= 0.0) ||
        !std::isfinite(hp->lr) || !std::isfinite(hp->eps) || !std::isfinite(hp->weight_decay)) {
        set_error("lr, eps and weight_decay must be finite and >= 0");
        return PS_ERANGE;
    }
    if (std::isnan(hp->grad_scale) || std::isnan(hp->clip_coef)) {
        set_error("grad_scale or clip_coef is NaN");
        return PS_ERANGE;
    }
    if (hp->clip_coef_device) {
        if (hp->clip_coef != 0.0) {
            set_error("clip_coef must be 0 when clip_coef_device is set");
            return PS_EINVAL;
        }
        if (reinterpret_cast<uintptr_t>(hp->clip_coef_device) & 3u) {
            set_error("clip_coef_device is not 4-byte aligned");
            return PS_EALIGN;
        }
    }
    return PS_OK;
}

// The placements this path executes: Omega sharded with G sharded and Theta R or S*
// (ZeRO-2, ZeRO-3); Omega sharded with G and Theta replicated (ZeRO-1); everything
// replicated (data parallelism, where the "shard" is the whole tensor).
bool is_zero1(const ps_spec_t *spec)
{
    return spec->omega == PS_S && spec->grad == PS_R && spec->theta == PS_R;
}

bool is_dp(const ps_spec_t *spec)
{
    return spec->omega == PS_R && spec->grad == PS_R && spec->theta == PS_R;
}

// Under pi_G = R the gradient is a single all-reduced, full-length buffer.
bool replicated_grad(const ps_spec_t *spec) { return is_zero1(spec) || is_dp(spec); }

ps_status_t check_path(const ps_spec_t *spec)
{
    ps_status_t st = check_spec(spec);
    if (st != PS_OK)
        return st;
    const bool sharded_g = spec->omega == PS_S && spec->grad == PS_S &&
                           (spec->theta == PS_R || spec->theta == PS_SG);
    if (!sharded_g && !replicated_grad(spec)) {
        set_error("step needs pi_Omega = S with (pi_G = S, pi_Theta in {R, S*}) or "
                  "(pi_G = R, pi_Theta = R), or all of them R");
        return PS_EUNSUPPORTED;
    }
    return PS_OK;
}

// The index range of the flat tensors this device updates: its shard (Eq. 2), or
// under full replication the whole tensor.
ps_status_t step_geometry(const ps_spec_t *spec, uint64_t *padded, uint64_t *off, uint64_t *len,
                          uint64_t *valid)
{
    ps_status_t st = shard_geometry(spec, padded, off, len, valid);
    if (st == PS_OK && is_dp(spec)) {
        *off = 0;
        *len = *padded;
        *valid = spec->psi;
    }
    return st;
}

ps_status_t check_contribs(const void *const *ptrs, uint32_t n_contrib, int32_t dtype,
                           uint32_t n_devices, const char *what, bool replicated_grad = false)
{
    if (!ptrs) {
        set_error("%s pointer array is NULL", what);
        return PS_EINVAL;
    }
    if (dtype != PS_BF16 && dtype != PS_F32 && dtype != PS_F16) {
        set_error("%s dtype must be PS_BF16, PS_F16 or PS_F32", what);
        return PS_EINVAL;
    }
    if (n_contrib == 0 || n_contrib > PS_MAX_CONTRIB) {
        set_error("%s count %u outside [1, %u]", what, n_contrib, PS_MAX_CONTRIB);
        return PS_ERANGE;
    }
    if (replicated_grad) {
        if (n_contrib != 1) {
            set_error("%s count %u: under pi_G = R the gradient is one all-reduced buffer", what,
                      n_contrib);
            return PS_EINVAL;
        }
    } else if (!(n_contrib == n_devices || (n_contrib == 1 && dtype == PS_F32))) {
        set_error("%s count %u: want n_devices = %u contributions (a missing or extra one "
                  "breaks gradient integrity), or one pre-reduced PS_F32 gradient",
                  what, n_contrib, n_devices);
        return PS_EINVAL;
    }
    for (uint32_t r = 0; r < n_contrib; ++r) {
        if (!ptrs[r]) {
            set_error("%s %u is NULL", what, r);
            return PS_EINVAL;
        }
        if (!aligned16(ptrs[r])) {
            set_error("%s %u is not 16-byte aligned", what, r);
            return PS_EALIGN;
        }
    }
    return PS_OK;
}

ps_status_t check_shard(const ps_spec_t *spec, const ps_shard_t *sh, uint64_t *out_offset)
{
    if (!sh) {
        set_error("shard is NULL");
        return PS_EINVAL;
    }
    if (!sh->master || !sh->m || !sh->v || !sh->gather_out) {
        set_error("shard has a NULL buffer");
        return PS_EINVAL;
    }
    if (!aligned16(sh->master) || !aligned16(sh->m) || !aligned16(sh->v) ||
        !aligned16(sh->gather_out)) {
        set_error("shard buffer not 16-byte aligned");
        return PS_EALIGN;
    }
    uint64_t padded, off, len, valid;
    ps_status_t st = step_geometry(spec, &padded, &off, &len, &valid);
    if (st != PS_OK)
        return st;
    if (sh->len != len) {
        set_error("shard.len %llu differs from %llu (psi_padded/N, or psi_padded under full "
                  "replication)", (unsigned long long)sh->len, (unsigned long long)len);
        return PS_ERANGE;
    }
    if (sh->valid_len > sh->len) {
        set_error("shard.valid_len exceeds shard.len");
        return PS_ERANGE;
    }
    // Under R the output buffer is the full replicated parameter tensor.
    *out_offset = spec->theta == PS_R ? off : 0;
    if (*out_offset % 8 != 0) {
        set_error("shard offset %llu into the replicated parameters is not a multiple of 8",
                  (unsigned long long)*out_offset);
        return PS_EALIGN;
    }
    return PS_OK;
}

ps_status_t check_range(uint64_t elem_offset, uint64_t elem_count, uint64_t len)
{
    if (elem_offset % 8 != 0) {
        set_error("elem_offset %llu is not a multiple of 8", (unsigned long long)elem_offset);
        return PS_EALIGN;
    }
    if (elem_offset > len || elem_count > len - elem_offset) {
        set_error("range [%llu, +%llu) leaves the shard of %llu elements",
                  (unsigned long long)elem_offset, (unsigned long long)elem_count,
                  (unsigned long long)len);
        return PS_ERANGE;
    }
    return PS_OK;
}

// Elements of [off, off+count) that lie below valid.
uint64_t clamp_count(uint64_t off, uint64_t count, uint64_t valid)
{
    if (off >= valid)
        return 0;
    return count < valid - off ? count : valid - off;
}

uint64_t elem_bytes(int32_t dtype) { return dtype == PS_F32 ? 4 : 2; }

// The parameters' 16-bit format, and that 16-bit gradients come in the same one.
ps_status_t check_param_dtype(int32_t param_dtype, int32_t reserved, int32_t grad_dtype)
{
    if ((param_dtype != PS_BF16 && param_dtype != PS_F16) || reserved != 0) {
        set_error("param_dtype must be PS_BF16 or PS_F16, reserved 0");
        return PS_EINVAL;
    }
    if (grad_dtype != PS_F32 && grad_dtype != param_dtype) {
        set_error("16-bit gradients (dtype %d) and parameters (dtype %d) must share one format",
                  grad_dtype, param_dtype);
        return PS_EUNSUPPORTED;
    }
    return PS_OK;
}

// Entry points other than ps_step_update take no accumulator beside the contributions.
ps_status_t no_accum(const ps_grads_t *grads, const char *call)
{
    if (grads && grads->accum) {
        set_error("%s takes no grads->accum: only ps_step_update adds an accumulator to the "
                  "contributions", call);
        return PS_EUNSUPPORTED;
    }
    return PS_OK;
}

// Both reduce entry points: `workspace` is the caller's, or NULL for the library's
// static per-device array (then workspace_bytes is ignored and nothing is allocated).
ps_status_t reduce_sumsq_checked(const ps_spec_t *spec, const ps_grads_t *grads, double grad_scale,
                                 float *reduced_out, double *sumsq_out, int32_t accumulate,
                                 void *workspace, uint64_t workspace_bytes, uint64_t elem_offset,
                                 uint64_t elem_count, uint64_t valid_len, void *stream)
{
    ps_status_t st;
    if ((st = check_path(spec)) != PS_OK)
        return st;
    if (replicated_grad(spec) && grads && grads->n_contrib != 1) {
        set_error("under pi_G = R the gradient is one all-reduced buffer");
        return PS_EINVAL;
    }
    if (!grads || !sumsq_out) {
        set_error("grads or sumsq_out is NULL");
        return PS_EINVAL;
    }
    if ((st = no_accum(grads, "the reduce phase")) != PS_OK)
        return st;
    if (std::isnan(grad_scale)) {
        set_error("grad_scale is NaN");
        return PS_ERANGE;
    }
    if (workspace && workspace_bytes < ps_workspace_bytes(elem_count)) {
        set_error("workspace of %llu bytes is smaller than ps_workspace_bytes(%llu) = %llu",
                  (unsigned long long)workspace_bytes, (unsigned long long)elem_count,
                  (unsigned long long)ps_workspace_bytes(elem_count));
        return PS_ERANGE;
    }
    if ((workspace && !aligned16(workspace)) || (reinterpret_cast<uintptr_t>(sumsq_out) & 7u) ||
        (reduced_out && !aligned16(reduced_out))) {
        set_error("workspace, sumsq_out or reduced_out is misaligned");
        return PS_EALIGN;
    }
    const bool z1 = replicated_grad(spec);
    if ((st = check_contribs(grads->contrib, grads->n_contrib, grads->dtype, spec->n_devices,
                             "contribution", z1)) != PS_OK)
        return st;
    uint64_t padded, off, len, valid;
    if ((st = step_geometry(spec, &padded, &off, &len, &valid)) != PS_OK ||
        (st = check_range(elem_offset, elem_count, len)) != PS_OK)
        return st;
    if (valid_len > len) {
        set_error("valid_len exceeds the shard length");
        return PS_ERANGE;
    }
    if (z1 && off % 8 != 0) {
        set_error("shard offset %llu into the replicated gradient is not a multiple of 8",
                  (unsigned long long)off);
        return PS_EALIGN;
    }
    if ((st = need_device()) != PS_OK)
        return st;
    if (!workspace) {
        double *own = nullptr;
        uint64_t doubles = 0;
        int se = static_reduce_scratch(&own, &doubles);
        if (se != 0)
            return hip_fail((hipError_t)se, "looking up the static partial-sum array");
        if (doubles < reduce_workspace_doubles(elem_count)) {
            set_error("static partial-sum array too small for %llu elements",
                      (unsigned long long)elem_count);
            return PS_ERANGE;
        }
        workspace = own;
    }

    const uint64_t count = clamp_count(elem_offset, elem_count, valid_len);
    const float gs = (float)(grad_scale > 0.0 ? grad_scale : 1.0 / (double)spec->n_devices);
    ContribPtrs g;
    std::memset(&g, 0, sizeof g);
    for (uint32_t r = 0; r < grads->n_contrib; ++r)
        g.p[r] = grads->contrib[r];
    if (z1)
        g.p[0] = reinterpret_cast<const char *>(g.p[0]) +
                 (off + elem_offset) * elem_bytes(grads->dtype);
    int e = launch_reduce_sumsq(grads->dtype, grads->n_contrib, g, gs,
                                reduced_out ? reduced_out + elem_offset : nullptr, count,
                                reinterpret_cast<double *>(workspace), sumsq_out, accumulate,
                                stream);
    if (e != 0)
        return hip_fail((hipError_t)e, "reduce kernel launch");
    return PS_OK;
}

// The bucket loop of ps_step_update_bucketed after validation.  Every HIP call goes
// through PS_ATTEMPT: after the first failure nothing more is enqueued, and finish()
// reports that failure once the events have been released.
#define PS_ATTEMPT(call)                                                                          \
    do {                                                                                          \
        if (ok())                                                                                 \
            note((call), #call);                                                                  \
    } while (0)

class BucketRun {
  public:
    BucketRun(const ps_shard_t *shard, const ps_bucket_plan_t *plan, const StepScalars &s,
              uint64_t out_off, uint64_t n_buckets)
        : shard_(shard), plan_(plan), s_(s), out_off_(out_off), n_buckets_(n_buckets),
          eb_(elem_bytes(plan->dtype)), slot_stride_(plan->bucket_elems * elem_bytes(plan->dtype)),
          copy_(reinterpret_cast<hipStream_t>(plan->copy_stream)),
          comp_(reinterpret_cast<hipStream_t>(plan->compute_stream)),
          timed_(plan->kernel_ms != nullptr),
          // A copy kernel and the update kernel both live on HBM bandwidth: run side by
          // side they only widen each other's request windows, so they take turns.  A
          // DMA copy (host or peer source) is bound by its link and overlaps.
          alternate_(plan->schedule == PS_SCHED_ALTERNATE ||
                     (plan->schedule == PS_SCHED_AUTO && plan->copy_engine != PS_COPY_MEMCPY)),
          reduce_(plan->copy_engine == PS_COPY_REDUCE)
    {
    }

    void create_events(bool in_place)
    {
        for (int k = 0; k < 2 && !in_place; ++k) {
            PS_ATTEMPT(hipEventCreateWithFlags(&staged_[k], hipEventDisableTiming));
            PS_ATTEMPT(hipEventCreateWithFlags(&freed_[k], hipEventDisableTiming));
        }
        if (timed_) {
            t0_.assign(n_buckets_, nullptr);
            t1_.assign(n_buckets_, nullptr);
            for (uint64_t b = 0; b < n_buckets_; ++b) {
                PS_ATTEMPT(hipEventCreate(&t0_[b]));
                PS_ATTEMPT(hipEventCreate(&t1_[b]));
            }
        }
    }

    // A source in this device's memory is read where it lies: one kernel per bucket on the
    // compute stream (one per contiguous piece where a repeating source wraps inside a
    // bucket), no staging slot, no second stream, no events unless timings are asked for.
    void in_place()
    {
        for (uint64_t b = 0; b < n_buckets_ && ok(); ++b) {
            const uint64_t lo = b * plan_->bucket_elems;
            const uint64_t cnt = clamp_count(lo, plan_->bucket_elems, shard_->valid_len);
            mark(t0_, b);
            for (uint64_t cur = lo; cur < lo + cnt && ok();) {
                const uint64_t pos = cur % plan_->source_elems;
                const uint64_t room = plan_->source_elems - pos;
                const uint64_t take = lo + cnt - cur < room ? lo + cnt - cur : room;
                ContribPtrs g;
                std::memset(&g, 0, sizeof g);
                for (uint32_t r = 0; r < plan_->n_contrib; ++r)
                    g.p[r] = reinterpret_cast<const char *>(plan_->source[r]) + pos * eb_;
                update(g, cur, take, plan_->dtype, plan_->n_contrib);
                cur += take;
            }
            mark(t1_, b);
        }
    }

    // A source that has to be moved first: bucket b+1 is staged on the copy stream into the
    // slot the update of bucket b-1 has released, while (or, taking turns, after) bucket b is
    // updated on the compute stream.  staged_[k]: slot k holds a complete bucket; freed_[k]:
    // the kernel reading slot k is done.
    void staged()
    {
        stage(0);
        for (uint64_t b = 0; b < n_buckets_ && ok(); ++b) {
            const int k = (int)(b & 1);
            if (b + 1 < n_buckets_ && !alternate_)
                stage(b + 1);
            const uint64_t lo = b * plan_->bucket_elems;
            const uint64_t cnt = clamp_count(lo, plan_->bucket_elems, shard_->valid_len);
            PS_ATTEMPT(hipStreamWaitEvent(comp_, staged_[k], 0));
            mark(t0_, b);
            if (cnt && ok()) {
                ContribPtrs g;
                std::memset(&g, 0, sizeof g);
                if (reduce_) { // the slot holds the contributions' FP32 sum
                    g.p[0] = plan_->staging[k];
                    update(g, lo, cnt, PS_F32, 1);
                } else {
                    for (uint32_t r = 0; r < plan_->n_contrib; ++r)
                        g.p[r] = reinterpret_cast<const char *>(plan_->staging[k]) + r * slot_stride_;
                    update(g, lo, cnt, plan_->dtype, plan_->n_contrib);
                }
            }
            mark(t1_, b);
            PS_ATTEMPT(hipEventRecord(freed_[k], comp_));
            if (b + 1 < n_buckets_ && alternate_)
                stage(b + 1);
        }
        // Later work on the copy stream must not overtake the last kernels.
        if (ok())
            PS_ATTEMPT(hipStreamWaitEvent(copy_, freed_[(n_buckets_ - 1) & 1], 0));
    }

    // Timings asked for: wait for the streams and read the per-bucket durations.
    void collect_timings(bool in_place)
    {
        if (!timed_)
            return;
        PS_ATTEMPT(hipStreamSynchronize(comp_));
        if (!in_place)
            PS_ATTEMPT(hipStreamSynchronize(copy_));
        for (uint64_t b = 0; b < n_buckets_ && ok(); ++b)
            PS_ATTEMPT(hipEventElapsedTime(&plan_->kernel_ms[b], t0_[b], t1_[b]));
    }

    // Destroying an event that is still pending is allowed: its resources are released
    // once the recorded work has completed.
    ps_status_t finish()
    {
        for (int k = 0; k < 2; ++k) {
            if (staged_[k])
                (void)hipEventDestroy(staged_[k]);
            if (freed_[k])
                (void)hipEventDestroy(freed_[k]);
        }
        for (hipEvent_t ev : t0_)
            if (ev)
                (void)hipEventDestroy(ev);
        for (hipEvent_t ev : t1_)
            if (ev)
                (void)hipEventDestroy(ev);
        return e_ == hipSuccess ? PS_OK : hip_fail(e_, what_);
    }

  private:
    bool ok() const { return e_ == hipSuccess; }

    // Records the first failure; PS_ATTEMPT makes no further HIP call after one.
    void note(hipError_t e, const char *what)
    {
        if (e_ == hipSuccess && e != hipSuccess) {
            e_ = e;
            what_ = what;
        }
    }

    void mark(std::vector<hipEvent_t> &ev, uint64_t b)
    {
        if (timed_ && ok())
            PS_ATTEMPT(hipEventRecord(ev[b], comp_));
    }

    // The update kernel over shard elements [lo, lo + count) from the contributions at g.
    void update(const ContribPtrs &g, uint64_t lo, uint64_t count, int dtype, uint32_t n_contrib)
    {
        uint16_t *out = reinterpret_cast<uint16_t *>(shard_->gather_out) + out_off_ + lo;
        int le = launch_update(dtype, n_contrib, g, nullptr, shard_->master + lo, shard_->m + lo,
                               shard_->v + lo, out, count, s_, comp_);
        if (le != 0)
            note((hipError_t)le, "update kernel launch");
    }

    void stage(uint64_t b)
    {
        if (!ok())
            return;
        const int k = (int)(b & 1);
        const uint64_t lo = b * plan_->bucket_elems;
        const uint64_t cnt = clamp_count(lo, plan_->bucket_elems, shard_->len);
        if (b >= 2) // the slot is reused: wait for the kernel that read it
            PS_ATTEMPT(hipStreamWaitEvent(copy_, freed_[k], 0));
        if (alternate_ && b >= 1) // take turns: start after the update of bucket b-1 has finished
            PS_ATTEMPT(hipStreamWaitEvent(copy_, freed_[k ^ 1], 0));
        if (plan_->copy_engine == PS_COPY_MEMCPY) {
            const uint64_t src_off = (lo % plan_->source_elems) * eb_;
            for (uint32_t r = 0; r < plan_->n_contrib && ok(); ++r)
                PS_ATTEMPT(hipMemcpyAsync(reinterpret_cast<char *>(plan_->staging[k]) + r * slot_stride_,
                                       reinterpret_cast<const char *>(plan_->source[r]) + src_off,
                                       cnt * eb_, hipMemcpyDefault, copy_));
        } else if (reduce_) {
            // one reduce launch per contiguous piece of the (possibly repeating) source
            for (uint64_t cur = lo; cur < lo + cnt && ok();) {
                const uint64_t pos = cur % plan_->source_elems;
                const uint64_t room = plan_->source_elems - pos;
                const uint64_t take = lo + cnt - cur < room ? lo + cnt - cur : room;
                ContribPtrs src;
                std::memset(&src, 0, sizeof src);
                for (uint32_t r = 0; r < plan_->n_contrib; ++r)
                    src.p[r] = reinterpret_cast<const char *>(plan_->source[r]) + pos * eb_;
                int le = launch_accumulate(plan_->dtype, plan_->n_contrib, src,
                                           reinterpret_cast<float *>(plan_->staging[k]) + (cur - lo), 1,
                                           take, copy_);
                if (le != 0)
                    note((hipError_t)le, "reduce kernel launch");
                cur += take;
            }
        } else if (ok()) {
            ContribPtrs src;
            std::memset(&src, 0, sizeof src);
            for (uint32_t r = 0; r < plan_->n_contrib; ++r)
                src.p[r] = plan_->source[r];
            int le = launch_stage(plan_->n_contrib, src, plan_->staging[k], slot_stride_, lo * eb_ / 16,
                                  plan_->source_elems * eb_ / 16, (cnt * eb_ + 15) / 16, alternate_,
                                  copy_);
            if (le != 0)
                note((hipError_t)le, "staging kernel launch");
        }
        if (ok())
            PS_ATTEMPT(hipEventRecord(staged_[k], copy_));
    }

    const ps_shard_t *shard_;
    const ps_bucket_plan_t *plan_;
    const StepScalars s_;
    const uint64_t out_off_, n_buckets_, eb_, slot_stride_;
    hipStream_t copy_, comp_;
    const bool timed_, alternate_, reduce_;
    hipEvent_t staged_[2] = {nullptr, nullptr}, freed_[2] = {nullptr, nullptr};
    std::vector<hipEvent_t> t0_, t1_;
    hipError_t e_ = hipSuccess;
    const char *what_ = "";
};

#undef PS_ATTEMPT

} // namespace

extern "C" {

ps_status_t ps_device_info(ps_device_info_t *info)
{
    clear_error();
    if (!info) {
        set_error("info is NULL");
        return PS_EINVAL;
    }
    ps_status_t st = need_device();
    if (st != PS_OK)
        return st;
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess)
        return hip_fail(e, "hipGetDevice");
    hipDeviceProp_t p;
    e = hipGetDeviceProperties(&p, dev);
    if (e != hipSuccess)
        return hip_fail(e, "hipGetDeviceProperties");
    std::memset(info, 0, sizeof *info);
    std::strncpy(info->name, p.name, sizeof info->name - 1);
    std::strncpy(info->arch, p.gcnArchName, sizeof info->arch - 1);
    info->compute_units = p.multiProcessorCount;
    info->wavefront_size = p.warpSize;
    info->clock_khz = p.clockRate;
    info->memory_clock_khz = p.memoryClockRate;
    info->memory_bus_bits = p.memoryBusWidth;
    info->l2_bytes = p.l2CacheSize;
    size_t fr = 0, tot = 0;
    e = hipMemGetInfo(&fr, &tot);
    if (e != hipSuccess)
        return hip_fail(e, "hipMemGetInfo");
    info->total_bytes = tot;
    info->free_bytes = fr;
    return PS_OK;
}

ps_status_t ps_step_update(const ps_spec_t *spec, const ps_adamw_t *hp, const ps_shard_t *shard,
                           const ps_grads_t *grads, uint64_t elem_offset, uint64_t elem_count,
                           void *stream)
{
    clear_error();
    ps_status_t st;
    if ((st = check_path(spec)) != PS_OK || (st = check_hp(hp)) != PS_OK)
        return st;
    uint64_t out_off = 0;
    if ((st = check_shard(spec, shard, &out_off)) != PS_OK)
        return st;
    if (!grads) {
        set_error("grads is NULL");
        return PS_EINVAL;
    }
    const bool z1 = replicated_grad(spec);
    if ((st = check_contribs(grads->contrib, grads->n_contrib, grads->dtype, spec->n_devices,
                             "contribution", z1)) != PS_OK ||
        (st = check_param_dtype(shard->param_dtype, shard->reserved, grads->dtype)) != PS_OK ||
        (st = check_range(elem_offset, elem_count, shard->len)) != PS_OK)
        return st;
    if (grads->accum) {
        if (z1) {
            set_error("grads->accum goes with pi_G = S contributions; under pi_G = R the "
                      "all-reduce has already summed the micro-batch");
            return PS_EUNSUPPORTED;
        }
        if (!aligned16(grads->accum)) {
            set_error("grads->accum is not 16-byte aligned");
            return PS_EALIGN;
        }
    }
    const uint64_t count = clamp_count(elem_offset, elem_count, shard->valid_len);
    if (count == 0)
        return PS_OK;
    if ((st = need_device()) != PS_OK)
        return st;

    const StepScalars s = derive_scalars(*hp, spec->n_devices, shard->param_dtype);
    ContribPtrs g;
    std::memset(&g, 0, sizeof g);
    for (uint32_t r = 0; r < grads->n_contrib; ++r)
        g.p[r] = grads->contrib[r];
    if (z1) // the replicated gradient is full length: this shard's slice starts at its offset
        g.p[0] = reinterpret_cast<const char *>(g.p[0]) +
                 (out_off + elem_offset) * elem_bytes(grads->dtype);
    uint16_t *out = reinterpret_cast<uint16_t *>(shard->gather_out) + out_off + elem_offset;
    int e = launch_update(grads->dtype, grads->n_contrib, g,
                          grads->accum ? grads->accum + elem_offset : nullptr,
                          shard->master + elem_offset, shard->m + elem_offset,
                          shard->v + elem_offset, out, count, s, stream);
    if (e != 0)
        return hip_fail((hipError_t)e, "update kernel launch");
    return PS_OK;
}

ps_status_t ps_step_accumulate(const ps_spec_t *spec, const ps_grads_t *grads, float *accum,
                               int32_t overwrite, uint64_t elem_offset, uint64_t elem_count,
                               uint64_t valid_len, void *stream)
{
    clear_error();
    ps_status_t st;
    if ((st = check_path(spec)) != PS_OK)
        return st;
    if (replicated_grad(spec)) {
        set_error("accumulation reduces pi_G = S contributions; under pi_G = R the "
                  "all-reduce has already done it");
        return PS_EUNSUPPORTED;
    }
    if (!grads || !accum) {
        set_error("grads or accum is NULL");
        return PS_EINVAL;
    }
    if ((st = no_accum(grads, "ps_step_accumulate (its accumulator is the accum argument)")) != PS_OK)
        return st;
    if (!aligned16(accum)) {
        set_error("accum is not 16-byte aligned");
        return PS_EALIGN;
    }
    if ((st = check_contribs(grads->contrib, grads->n_contrib, grads->dtype, spec->n_devices,
                             "contribution")) != PS_OK)
        return st;
    uint64_t padded, off, len, valid;
    if ((st = shard_geometry(spec, &padded, &off, &len, &valid)) != PS_OK ||
        (st = check_range(elem_offset, elem_count, len)) != PS_OK)
        return st;
    if (valid_len > len) {
        set_error("valid_len exceeds the shard length");
        return PS_ERANGE;
    }
    const uint64_t count = clamp_count(elem_offset, elem_count, valid_len);
    if (count == 0)
        return PS_OK;
    if ((st = need_device()) != PS_OK)
        return st;
    ContribPtrs g;
    std::memset(&g, 0, sizeof g);
    for (uint32_t r = 0; r < grads->n_contrib; ++r)
        g.p[r] = grads->contrib[r];
    int e = launch_accumulate(grads->dtype, grads->n_contrib, g, accum + elem_offset, overwrite,
                              count, stream);
    if (e != 0)
        return hip_fail((hipError_t)e, "accumulate kernel launch");
    return PS_OK;
}

uint64_t ps_workspace_bytes(uint64_t elem_count)
{
    return reduce_workspace_doubles(elem_count) * sizeof(double);
}

ps_status_t ps_step_reduce_sumsq(const ps_spec_t *spec, const ps_grads_t *grads,
                                 double grad_scale, float *reduced_out, double *sumsq_out,
                                 int32_t accumulate, void *workspace, uint64_t workspace_bytes,
                                 uint64_t elem_offset, uint64_t elem_count, uint64_t valid_len,
                                 void *stream)
{
    clear_error();
    if (!workspace) {
        set_error("workspace is NULL");
        return PS_EINVAL;
    }
    return reduce_sumsq_checked(spec, grads, grad_scale, reduced_out, sumsq_out, accumulate,
                                workspace, workspace_bytes, elem_offset, elem_count, valid_len,
                                stream);
}

ps_status_t ps_step_reduce_sumsq_static(const ps_spec_t *spec, const ps_grads_t *grads,
                                        double grad_scale, float *reduced_out, double *sumsq_out,
                                        int32_t accumulate, uint64_t elem_offset,
                                        uint64_t elem_count, uint64_t valid_len, void *stream)
{
    clear_error();
    if (elem_count > PS_STATIC_MAX_ELEMS) {
        set_error("elem_count %llu exceeds PS_STATIC_MAX_ELEMS = %llu: call once per range of at "
                  "most that many elements, with accumulate set from the second on",
                  (unsigned long long)elem_count, (unsigned long long)PS_STATIC_MAX_ELEMS);
        return PS_ERANGE;
    }
    return reduce_sumsq_checked(spec, grads, grad_scale, reduced_out, sumsq_out, accumulate,
                                nullptr, 0, elem_offset, elem_count, valid_len, stream);
}

ps_status_t ps_step_clip_coef(const double *sumsq_local, const double *sumsq_others,
                              double max_norm, float *coef_out, void *stream)
{
    clear_error();
    if (!sumsq_local || !coef_out) {
        set_error("sumsq_local or coef_out is NULL");
        return PS_EINVAL;
    }
    if ((reinterpret_cast<uintptr_t>(sumsq_local) & 7u) ||
        (reinterpret_cast<uintptr_t>(sumsq_others) & 7u) ||
        (reinterpret_cast<uintptr_t>(coef_out) & 3u)) {
        set_error("sumsq pointers need 8-byte and coef_out 4-byte alignment");
        return PS_EALIGN;
    }
    ps_status_t st = need_device();
    if (st != PS_OK)
        return st;
    int e = launch_clip_coef(sumsq_local, sumsq_others, max_norm, coef_out, stream);
    if (e != 0)
        return hip_fail((hipError_t)e, "clip coefficient kernel launch");
    return PS_OK;
}

ps_status_t ps_step_update_bucketed(const ps_spec_t *spec, const ps_adamw_t *hp,
                                    const ps_shard_t *shard, const ps_bucket_plan_t *plan)
{
    clear_error();
    ps_status_t st;
    if ((st = check_path(spec)) != PS_OK || (st = check_hp(hp)) != PS_OK)
        return st;
    uint64_t out_off = 0;
    if ((st = check_shard(spec, shard, &out_off)) != PS_OK)
        return st;
    if (!plan) {
        set_error("plan is NULL");
        return PS_EINVAL;
    }
    if (replicated_grad(spec)) {
        set_error("the bucket pipeline stages pi_G = S contributions");
        return PS_EUNSUPPORTED;
    }
    if ((st = check_contribs(plan->source, plan->n_contrib, plan->dtype, spec->n_devices,
                             "bucket source")) != PS_OK ||
        (st = check_param_dtype(shard->param_dtype, shard->reserved, plan->dtype)) != PS_OK)
        return st;
    if (plan->bucket_elems == 0 || plan->bucket_elems % 8 != 0) {
        set_error("bucket_elems must be a positive multiple of 8");
        return PS_EALIGN;
    }
    if (plan->source_elems == 0) {
        set_error("source_elems must be >= 1");
        return PS_ERANGE;
    }
    if (plan->source_elems % 512 != 0) {
        set_error("source_elems must be a multiple of 512");
        return PS_EALIGN;
    }
    if (plan->copy_engine != PS_COPY_KERNEL && plan->copy_engine != PS_COPY_MEMCPY &&
        plan->copy_engine != PS_COPY_NONE && plan->copy_engine != PS_COPY_REDUCE) {
        set_error("copy_engine must be PS_COPY_KERNEL, PS_COPY_MEMCPY, PS_COPY_REDUCE or "
                  "PS_COPY_NONE");
        return PS_EINVAL;
    }
    const bool in_place = plan->copy_engine == PS_COPY_NONE;
    if (plan->schedule != PS_SCHED_AUTO && plan->schedule != PS_SCHED_OVERLAP &&
        plan->schedule != PS_SCHED_ALTERNATE) {
        set_error("schedule must be PS_SCHED_AUTO, PS_SCHED_OVERLAP or PS_SCHED_ALTERNATE");
        return PS_EINVAL;
    }
    if (plan->copy_engine == PS_COPY_MEMCPY && plan->source_elems % plan->bucket_elems != 0) {
        set_error("PS_COPY_MEMCPY needs source_elems to be a multiple of bucket_elems");
        return PS_EUNSUPPORTED;
    }
    if (!in_place) {
        if (!plan->staging[0] || !plan->staging[1] || plan->staging[0] == plan->staging[1]) {
            set_error("two distinct staging buffers are required");
            return PS_EINVAL;
        }
        if (!aligned16(plan->staging[0]) || !aligned16(plan->staging[1])) {
            set_error("staging buffer not 16-byte aligned");
            return PS_EALIGN;
        }
        if (plan->copy_stream == plan->compute_stream) {
            set_error("copy_stream and compute_stream must differ");
            return PS_EINVAL;
        }
    }
    const uint64_t n_buckets = (shard->len + plan->bucket_elems - 1) / plan->bucket_elems;
    if (plan->kernel_ms && plan->kernel_ms_len < n_buckets) {
        set_error("kernel_ms holds %llu entries, %llu buckets", (unsigned long long)plan->kernel_ms_len,
                  (unsigned long long)n_buckets);
        return PS_ERANGE;
    }
    if (n_buckets == 0)
        return PS_OK;
    if ((st = need_device()) != PS_OK)
        return st;

    BucketRun run(shard, plan, derive_scalars(*hp, spec->n_devices, shard->param_dtype), out_off,
                  n_buckets);
    run.create_events(in_place);
    if (in_place)
        run.in_place();
    else
        run.staged();
    run.collect_timings(in_place);
    return run.finish();
}

uint64_t ps_verify_workspace_bytes(uint64_t buffer_bytes)
{
    return verify_workspace_slots(buffer_bytes) * 8;
}

ps_status_t ps_verify_diff_sumsq(const void *a, const void *b, int32_t dtype, uint64_t elem_count,
                                 double *out2, int32_t accumulate, void *workspace,
                                 uint64_t workspace_bytes, void *stream)
{
    clear_error();
    if (!a || !b || !out2 || !workspace) {
        set_error("a, b, out2 or workspace is NULL");
        return PS_EINVAL;
    }
    if (dtype != PS_BF16 && dtype != PS_F32 && dtype != PS_F16) {
        set_error("dtype must be PS_BF16, PS_F16 or PS_F32");
        return PS_EINVAL;
    }
    if (!aligned16(a) || !aligned16(b) || !aligned16(workspace) ||
        (reinterpret_cast<uintptr_t>(out2) & 7u)) {
        set_error("a, b, workspace need 16-byte and out2 8-byte alignment");
        return PS_EALIGN;
    }
    if (elem_count > UINT64_MAX / 4 ||
        workspace_bytes < ps_verify_workspace_bytes(elem_count * elem_bytes(dtype))) {
        set_error("workspace smaller than ps_verify_workspace_bytes()");
        return PS_ERANGE;
    }
    ps_status_t st = need_device();
    if (st != PS_OK)
        return st;
    int e = launch_diff_sumsq(dtype, a, b, elem_count, out2, accumulate, workspace,
                              verify_workspace_slots(elem_count * elem_bytes(dtype)), stream);
    if (e != 0)
        return hip_fail((hipError_t)e, "difference kernel launch");
    return PS_OK;
}

ps_status_t ps_verify_checksum(const void *buf, uint64_t bytes, uint64_t first_word_index,
                               uint64_t *out, int32_t accumulate, void *workspace,
                               uint64_t workspace_bytes, void *stream)
{
    clear_error();
    if (!buf || !out || !workspace) {
        set_error("buf, out or workspace is NULL");
        return PS_EINVAL;
    }
    if (!aligned16(buf) || !aligned16(workspace) || (reinterpret_cast<uintptr_t>(out) & 7u) ||
        bytes % 8 != 0) {
        set_error("buf, workspace need 16-byte alignment, out 8-byte, bytes a multiple of 8");
        return PS_EALIGN;
    }
    if (workspace_bytes < ps_verify_workspace_bytes(bytes)) {
        set_error("workspace smaller than ps_verify_workspace_bytes()");
        return PS_ERANGE;
    }
    ps_status_t st = need_device();
    if (st != PS_OK)
        return st;
    int e = launch_checksum(buf, bytes / 8, first_word_index, out, accumulate, workspace, stream);
    if (e != 0)
        return hip_fail((hipError_t)e, "checksum kernel launch");
    return PS_OK;
}

ps_status_t ps_step_update_offloaded(const ps_spec_t *spec, const ps_adamw_t *hp,
                                     const ps_offload_plan_t *plan, const ps_grads_t *grads)
{
    clear_error();
    ps_status_t st;
    if ((st = check_spec(spec)) != PS_OK || (st = check_hp(hp)) != PS_OK)
        return st;
    if (spec->theta != PS_O || spec->omega != PS_O || spec->grad != PS_S) {
        set_error("offloaded step needs pi_Theta = O, pi_Omega = O, pi_G = S");
        return PS_EUNSUPPORTED;
    }
    if (!plan || !grads) {
        set_error("plan or grads is NULL");
        return PS_EINVAL;
    }
    if ((st = no_accum(grads, "the offloaded step")) != PS_OK)
        return st;
    if ((plan->host_layout != PS_HOST_FLAT && plan->host_layout != PS_HOST_PACKED) ||
        plan->reserved != 0) {
        set_error("host_layout must be PS_HOST_FLAT or PS_HOST_PACKED, reserved 0");
        return PS_EINVAL;
    }
    const bool packed = plan->host_layout == PS_HOST_PACKED;
    if (packed ? !plan->host_packed
               : (!plan->host_master || !plan->host_m || !plan->host_v || !plan->host_param_out)) {
        set_error("plan has a NULL host buffer");
        return PS_EINVAL;
    }
    if (plan->n_slots != 2 && plan->n_slots != 3) {
        set_error("n_slots must be 2 or 3");
        return PS_EINVAL;
    }
    for (uint32_t k = 0; k < plan->n_slots; ++k) {
        if (!plan->slot[k]) {
            set_error("slot %u is NULL", k);
            return PS_EINVAL;
        }
        if (!aligned16(plan->slot[k])) {
            set_error("slot %u is not 16-byte aligned", k);
            return PS_EALIGN;
        }
        for (uint32_t j = 0; j < k; ++j)
            if (plan->slot[j] == plan->slot[k]) {
                set_error("slots must be distinct");
                return PS_EINVAL;
            }
    }
    if (plan->bucket_elems == 0 || plan->bucket_elems % 8 != 0) {
        set_error("bucket_elems must be a positive multiple of 8");
        return PS_EALIGN;
    }
    if (packed ? !aligned16(plan->host_packed)
               : (!aligned16(plan->host_master) || !aligned16(plan->host_m) ||
                  !aligned16(plan->host_v) || !aligned16(plan->host_param_out))) {
        set_error("host buffer not 16-byte aligned");
        return PS_EALIGN;
    }
    if (plan->h2d_stream == plan->compute_stream || plan->h2d_stream == plan->d2h_stream ||
        plan->compute_stream == plan->d2h_stream) {
        set_error("the three streams must differ");
        return PS_EINVAL;
    }
    uint64_t padded, off, len, valid;
    if ((st = shard_geometry(spec, &padded, &off, &len, &valid)) != PS_OK)
        return st;
    if (plan->len != len || plan->valid_len > plan->len) {
        set_error("plan.len %llu differs from psi_padded/N = %llu, or valid_len exceeds it",
                  (unsigned long long)plan->len, (unsigned long long)len);
        return PS_ERANGE;
    }
    if ((st = check_contribs(grads->contrib, grads->n_contrib, grads->dtype, spec->n_devices,
                             "contribution")) != PS_OK ||
        (st = check_param_dtype(plan->param_dtype, 0, grads->dtype)) != PS_OK)
        return st;
    const uint64_t B = plan->bucket_elems;
    const uint64_t n_buckets = (plan->valid_len + B - 1) / B;
    if (n_buckets == 0)
        return PS_OK;
    if ((st = need_device()) != PS_OK)
        return st;

    hipStream_t up = reinterpret_cast<hipStream_t>(plan->h2d_stream);
    hipStream_t comp = reinterpret_cast<hipStream_t>(plan->compute_stream);
    hipStream_t down = reinterpret_cast<hipStream_t>(plan->d2h_stream);
    const StepScalars s = derive_scalars(*hp, spec->n_devices, plan->param_dtype);
    const uint64_t eb = elem_bytes(grads->dtype);
    const uint32_t S = plan->n_slots;
    hipEvent_t loaded[3] = {}, computed[3] = {}, drained[3] = {};
    hipError_t e = hipSuccess;
    const char *what = "";
#define PS_TRY(call)                                                                              \
    do {                                                                                          \
        if (e == hipSuccess) {                                                                    \
            e = (call);                                                                           \
            what = #call;                                                                         \
        }                                                                                         \
    } while (0)
    for (uint32_t k = 0; k < S; ++k) {
        PS_TRY(hipEventCreateWithFlags(&loaded[k], hipEventDisableTiming));
        PS_TRY(hipEventCreateWithFlags(&computed[k], hipEventDisableTiming));
        PS_TRY(hipEventCreateWithFlags(&drained[k], hipEventDisableTiming));
    }
    for (uint64_t b = 0; b < n_buckets && e == hipSuccess; ++b) {
        const uint32_t k = (uint32_t)(b % S);
        const uint64_t lo = b * B;
        const uint64_t cnt = clamp_count(lo, B, plan->valid_len);
        char *slot = reinterpret_cast<char *>(plan->slot[k]);
        float *d_master = reinterpret_cast<float *>(slot);
        float *d_m = reinterpret_cast<float *>(slot + 4 * B);
        float *d_v = reinterpret_cast<float *>(slot + 8 * B);
        uint16_t *d_out = reinterpret_cast<uint16_t *>(slot + 12 * B);
        // upload: the slot is free once bucket b - S has been written back
        if (b >= S)
            PS_TRY(hipStreamWaitEvent(up, drained[k], 0));
        // where this bucket's four arrays lie on the host
        char *h_pack = packed ? reinterpret_cast<char *>(plan->host_packed) + b * 14 * B : nullptr;
        float *h_master = packed ? reinterpret_cast<float *>(h_pack) : plan->host_master + lo;
        float *h_m = packed ? reinterpret_cast<float *>(h_pack + 4 * B) : plan->host_m + lo;
        float *h_v = packed ? reinterpret_cast<float *>(h_pack + 8 * B) : plan->host_v + lo;
        uint16_t *h_out = packed ? reinterpret_cast<uint16_t *>(h_pack + 12 * B)
                                 : reinterpret_cast<uint16_t *>(plan->host_param_out) + lo;
        const bool one_copy = packed && cnt == B; // host and slot layouts coincide
        if (one_copy) {
            PS_TRY(hipMemcpyAsync(slot, h_pack, 12 * B, hipMemcpyHostToDevice, up));
        } else {
            PS_TRY(hipMemcpyAsync(d_master, h_master, cnt * 4, hipMemcpyHostToDevice, up));
            PS_TRY(hipMemcpyAsync(d_m, h_m, cnt * 4, hipMemcpyHostToDevice, up));
            PS_TRY(hipMemcpyAsync(d_v, h_v, cnt * 4, hipMemcpyHostToDevice, up));
        }
        PS_TRY(hipEventRecord(loaded[k], up));
        // update in the slot
        PS_TRY(hipStreamWaitEvent(comp, loaded[k], 0));
        if (e == hipSuccess) {
            ContribPtrs g;
            std::memset(&g, 0, sizeof g);
            for (uint32_t r = 0; r < grads->n_contrib; ++r)
                g.p[r] = reinterpret_cast<const char *>(grads->contrib[r]) + lo * eb;
            int le = launch_update(grads->dtype, grads->n_contrib, g, nullptr, d_master, d_m, d_v,
                                   d_out, cnt, s, comp);
            if (le != 0) {
                e = (hipError_t)le;
                what = "update kernel launch";
            }
        }
        PS_TRY(hipEventRecord(computed[k], comp));
        // download
        PS_TRY(hipStreamWaitEvent(down, computed[k], 0));
        if (one_copy) {
            PS_TRY(hipMemcpyAsync(h_pack, slot, 14 * B, hipMemcpyDeviceToHost, down));
        } else {
            PS_TRY(hipMemcpyAsync(h_master, d_master, cnt * 4, hipMemcpyDeviceToHost, down));
            PS_TRY(hipMemcpyAsync(h_m, d_m, cnt * 4, hipMemcpyDeviceToHost, down));
            PS_TRY(hipMemcpyAsync(h_v, d_v, cnt * 4, hipMemcpyDeviceToHost, down));
            PS_TRY(hipMemcpyAsync(h_out, d_out, cnt * 2, hipMemcpyDeviceToHost, down));
        }
        PS_TRY(hipEventRecord(drained[k], down));
    }
    // The next call on these streams uploads into the same slots and reads the same host
    // ranges: its first upload must not start before this call's last downloads are done.
    for (uint32_t k = 0; k < S && k < n_buckets; ++k)
        PS_TRY(hipStreamWaitEvent(up, drained[k], 0));
#undef PS_TRY
    for (uint32_t k = 0; k < S; ++k) {
        if (loaded[k])
            (void)hipEventDestroy(loaded[k]);
        if (computed[k])
            (void)hipEventDestroy(computed[k]);
        if (drained[k])
            (void)hipEventDestroy(drained[k]);
    }
    if (e != hipSuccess)
        return hip_fail(e, what);
    return PS_OK;
}

ps_status_t ps_probe_set_update_residency(uint32_t waves_per_cu)
{
    clear_error();
    if (waves_per_cu != 0 && waves_per_cu < 3) {
        set_error("waves_per_cu must be 0 (library's choice), 3..32, or above 32 (no cap)");
        return PS_ERANGE;
    }
    set_update_residency(waves_per_cu);
    return PS_OK;
}

ps_status_t ps_probe_copy(void *dst, const void *src, uint64_t bytes, void *stream)
{
    clear_error();
    if (!dst || !src) {
        set_error("dst or src is NULL");
        return PS_EINVAL;
    }
    if (!aligned16(dst) || !aligned16(src) || bytes % 16 != 0) {
        set_error("copy needs 16-byte aligned pointers and size");
        return PS_EALIGN;
    }
    if (bytes == 0)
        return PS_OK;
    ps_status_t st = need_device();
    if (st != PS_OK)
        return st;
    int e = launch_copy(dst, src, bytes, stream);
    if (e != 0)
        return hip_fail((hipError_t)e, "copy kernel launch");
    return PS_OK;
}

} // extern "C"
