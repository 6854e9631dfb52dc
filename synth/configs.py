"""The five workloads: sizes, placement, hyper-parameters and value recipes.

The paper names its workloads only by parameter count (7B, 13B, 70B models of
Sections 1 and 4) and byte accounting (Remark 1); the flat-buffer shapes below
stand in for a training job's master/moment/gradient shards at those sizes.
"""
from dataclasses import dataclass, field


@dataclass(frozen=True)
class Workload:
    name: str
    psi: int                 # flat parameter count (the paper's P)
    n_devices: int           # N
    shard_index: int         # i
    strategy: str            # row of the paper's Table 2
    grad_dtype: str          # "bf16", "f16" or "f32"
    lr: float = 1e-4
    beta1: float = 0.9
    beta2: float = 0.999
    eps: float = 1e-8
    weight_decay: float = 0.01
    first_step: int = 1      # t of the first step run
    n_steps: int = 1
    align_elems: int = 1
    theta_std: float = 0.02
    grad_std: float = 1e-3
    warm_moments: bool = False      # m ~ |N(0,1e-3)|, v ~ N(0,1e-3)^2 instead of zeros
    outlier_frac: float = 0.0       # fraction of gradient entries multiplied by outlier_mult
    outlier_mult: float = 1.0
    student_t_dof: int = 0          # >0: gradients are grad_std * Student-t(dof)
    bucket_elems: int = 0           # >0: gradients arrive in buckets of this many elements
    max_grad_norm: float = 0.0      # >0: global-norm clipping
    micro_batches: int = 1          # >1: gradient accumulation over this many micro-batches
    loss_scale: float = 1.0         # gradients are generated times this, grad_scale divides it out
    param_dtype: str = "bf16"       # the 16-bit format of the parameter image: "bf16" or "f16"
    seed: int = 20260102
    extra: dict = field(default_factory=dict)

    @property
    def psi_padded(self) -> int:
        unit = self.n_devices * max(1, self.align_elems)
        return -(-self.psi // unit) * unit

    @property
    def shard_len(self) -> int:
        return self.psi_padded // self.n_devices

    @property
    def shard_offset(self) -> int:
        return self.shard_index * self.shard_len

    @property
    def valid_len(self) -> int:
        return min(max(self.psi - self.shard_offset, 0), self.shard_len)


WORKLOADS = {
    # Tiny: all four shards are also checked against the unsharded update.
    "tiny": Workload("tiny", psi=1_048_576, n_devices=4, shard_index=0, strategy="zero3",
                     grad_dtype="bf16", n_steps=10),
    # GPT-2-small-sized state, one step late in training.
    "gpt2s": Workload("gpt2s", psi=124_439_808, n_devices=8, shard_index=3, strategy="zero3",
                      grad_dtype="bf16", first_step=1000, warm_moments=True),
    # 7B under ZeRO-2 (Theta replicated, Omega and G sharded).
    "7b_zero2": Workload("7b_zero2", psi=6_738_415_616, n_devices=8, shard_index=0,
                         strategy="zero2", grad_dtype="bf16", first_step=1000,
                         warm_moments=True, grad_std=1e-4, outlier_frac=1e-3,
                         outlier_mult=100.0),
    # 70B under ZeRO-3, gradients streamed in buckets of 2^28 elements.
    "70b_zero3": Workload("70b_zero3", psi=70_000_000_000, n_devices=8, shard_index=7,
                          strategy="zero3", grad_dtype="bf16", first_step=1000,
                          warm_moments=True, grad_std=1e-4, bucket_elems=1 << 28),
    # The other data-parallel rows of the paper's Table 2 on the 7B shard: ZeRO-1 (the
    # gradient arrives all-reduced, one replicated full-length buffer) and gradient
    # accumulation over four micro-batches before one ZeRO-2 update.
    # The same shard in the paper's own FP16 (Table 1): binary16 gradients carrying a loss
    # scale of 1024, binary16 parameter image.
    "7b_zero2_f16": Workload("7b_zero2_f16", psi=6_738_415_616, n_devices=8, shard_index=0,
                             strategy="zero2", grad_dtype="f16", param_dtype="f16", first_step=1000,
                             warm_moments=True, grad_std=1e-4, outlier_frac=0.001,
                             outlier_mult=100.0, loss_scale=1024.0),
    "7b_zero1": Workload("7b_zero1", psi=6_738_415_616, n_devices=8, shard_index=0,
                         strategy="zero1", grad_dtype="bf16", first_step=1000,
                         warm_moments=True, grad_std=8e-4),
    "7b_accum4": Workload("7b_accum4", psi=6_738_415_616, n_devices=8, shard_index=0,
                          strategy="zero2", grad_dtype="bf16", first_step=1000,
                          warm_moments=True, grad_std=1e-4, micro_batches=4),
    # ZeRO-Offload row: the 7B shard with master/m/v and the bf16 parameters in pinned
    # host memory (11.8 GB), streamed through the device (bound by the host link).
    "7b_offload": Workload("7b_offload", psi=6_738_415_616, n_devices=8, shard_index=0,
                           strategy="zero_offload", grad_dtype="bf16", first_step=1000,
                           warm_moments=True, grad_std=1e-4, bucket_elems=1 << 25),
    # Ragged 13B FSDP-style shard, fp32 heavy-tailed gradients, global-norm clip.
    # psi is already a multiple of 6*256; "psi_ragged" drops 1001 elements so that
    # the last shard owns a pad of 1001 elements that must stay untouched.
    "13b_clip": Workload("13b_clip", psi=13_015_864_320, n_devices=6, shard_index=5,
                         strategy="zero3", grad_dtype="f32", lr=3e-4, weight_decay=0.1,
                         first_step=1000, warm_moments=True, align_elems=256, grad_std=1e-4,
                         student_t_dof=3, max_grad_norm=1.0,
                         extra={"psi_ragged": 13_015_864_320 - 1001}),
}
