"""Call counts of a pruning schedule and the FLOP total they imply (test infrastructure only).

Sec. 5.2 / Sec. 6.2: trajectories that a checkpoint drops take no further denoising steps, and
only the survivors are trained on.  The paper prints per-call costs and per-epoch totals for
three schedules; the per-epoch procedure itself is in an appendix that is not available, so the
model below is a reading, pinned by the printed totals (tests/golden/efficiency_table.txt):

  total = prompts * ( c_net * network_calls
                      + (c_vae + c_reward) * (preview_calls + final_reward_calls)
                      + train_mult * c_net * T * survivors )

with `network_calls` counted under the reading "a checkpoint at step s acts after the network
evaluation of step s" (the trajectories it drops were still evaluated at step s),
`preview_calls` = trajectories active at each checkpoint, and train_mult = 4 network-call
equivalents per trained trajectory-step.  With 96 prompts per epoch this reproduces all three
printed totals to 2e-4; counting the evaluation at the checkpoint step only for the survivors
admits no single train_mult that fits both pruned schedules.
"""


def schedule_counts(n0, T, schedule, prune_after_eval=True):
    """schedule: list of (step, keep).  Returns dict(network_calls, preview_calls, survivors,
    active=[trajectories evaluated at each step])."""
    sched = dict(schedule)
    n = n0
    calls = previews = 0
    active = []
    for s in range(T):
        if s in sched and not prune_after_eval:
            previews += n
            n = sched[s]
        calls += n
        active.append(n)
        if s in sched and prune_after_eval:
            previews += n
            n = sched[s]
    return dict(network_calls=calls, preview_calls=previews, survivors=n, active=active)


def epoch_tflops(counts, T, c_net, c_vae, c_reward, train_mult=4.0, prompts=96):
    per_prompt = (c_net * counts["network_calls"]
                  + (c_vae + c_reward) * (counts["preview_calls"] + counts["survivors"])
                  + train_mult * c_net * T * counts["survivors"])
    return prompts * per_prompt
