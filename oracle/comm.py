"""Oracle: communication volume of one rank's ZeRO step and the time it takes
on a given link.

TEST INFRASTRUCTURE ONLY - never imported by the product path.

Appendix "Analysis of Experiments" counts, for a feed-forward block of 8 h^2
parameters at ZeRO-3 on d devices, one all-gather in the forward pass and an
all-gather plus a reduce-scatter in the backward pass, each moving the block's
parameters to every device: 3 * 8 h^2 * d = 24 d h^2 elements in all.
Appendix "Details about ZeRO" names the collectives of the other stages.

Readings:
  * the paper's count is kept as printed: a collective over P elements moves
    P elements per device (the (d-1)/d share a device already holds is not
    deducted), so the volume summed over devices is P * d;
  * a world of one device exchanges nothing;
  * stage 0: all-reduce of the gradients at the end of the backward pass =
    reduce-scatter + all-gather, once per optimizer step;
    stage 1: the same up to the optimizer, then an all-gather of the updated
    parameters, once per optimizer step;
    stage 2: reduce-scatter of the gradients in every micro-step (a rank keeps
    only its gradient shard), all-gather of the parameters once per step;
    stage 3: two parameter all-gathers and one gradient reduce-scatter in
    every micro-step, nothing more per step;
  * time = bytes per device / bandwidth per device: the only model the
    paper's proportionality argument supports.
"""


def comm_elements(P, world, stage):
    """(per_micro_params, per_micro_grads, per_step_params, per_step_grads): elements one device moves."""
    if world <= 1:
        return 0, 0, 0, 0
    if stage == 0:
        return 0, 0, 0, 2 * P
    if stage == 1:
        return 0, 0, P, 2 * P
    if stage == 2:
        return 0, P, P, 0
    if stage == 3:
        return 2 * P, P, 0, 0
    raise ValueError("stage must be 0..3")


def comm_model(P, world, stage, param_bytes, grad_bytes, bytes_per_second):
    """dict(micro_bytes, step_bytes, total_micro_elements, t_micro, t_step) for one device;
    total_micro_elements is the per-micro-step count summed over the devices (the paper's Comm_Volume)."""
    mp, mg, sp, sg = comm_elements(P, world, stage)
    micro_bytes = mp * float(param_bytes) + mg * float(grad_bytes)
    step_bytes = sp * float(param_bytes) + sg * float(grad_bytes)
    return dict(micro_bytes=micro_bytes, step_bytes=step_bytes, total_micro_elements=(mp + mg) * world,
                t_micro=micro_bytes / float(bytes_per_second), t_step=step_bytes / float(bytes_per_second))
