"""CPU oracle for one bulk-synchronous Parameter-Server training iteration.

TEST INFRASTRUCTURE ONLY.  This package is the slow, plain float64 statement of
what the iteration computes (numpy on the host).  Only the test-suite, the
smoke check and the benchmark's CPU-baseline leg may import it; the GPU
library never does, and this package never imports the GPU library.  The two
share no code: only the seeded input generators in `workload` feed both.

Structure of the iteration (Problem Formulation, Section II of the AntDT
paper): each of n workers computes a local gradient on its local batch B_i and
pushes it; the servers aggregate the workers' gradients and update the
parameters; the global batch sum_i B_i = B is fixed (constraint of Eq. 1).
The paper does not spell out the model, the aggregation weights or the
optimizer; the readings taken are stated in each function's docstring.

Pins (tests marked "not gpu"): torch-CPU embedding_bag/autograd/Adagrad/Adam as
library special cases, central finite differences, partition invariance
(sum_k (B_k/B) g_k equals the whole-batch gradient for any split), row
sparsity, closed forms of the first Adagrad/Adam step, brute-force coalescing
and brute-force enumeration of Eq. 3 / Eq. 4; for the shard queue its stated
transitions, at-least-once coverage under random losses and the re-queue order;
for the job-completion-time model the closed forms of undisturbed, persistently
disturbed and backup-worker runs, the Eq. 3 split it converges to, the rate of
its pseudo-random disturbance pattern, and schedules worked out by hand from the
stated rules (iteration end times, window means, decision iteration, sizes after
ADJUST_BS, kill time: tests/jct_schedules.py).  The bf16-operand reading of the
worker step is pinned by a worked example in which every rounding point (stored
input, operand weights forward and backward, stored activation, gradient after
the ReLU mask, unrounded biases and last layer) moves a hand-computed result.
The paper prints no worked numeric example of an iteration or of a schedule, so
no pin is a printed value.  Parity unpinned: which (window, worker) pairs the
pseudo-random disturbance pattern picks (only its rate and determinism are
checked).
"""
from .ps_iteration import (  # noqa: F401
    Model,
    ShardResult,
    Aggregated,
    round_bf16,
    embedding_pool,
    embedding_pool_loops,
    mlp_forward,
    bce_with_logits,
    worker_step,
    shard_weights,
    aggregate,
    coalesce_loops,
    apply_update,
    adagrad_elementwise,
    adagrad_rowwise,
)
from .dense_adam import weighted_average, adam_step, dense_aggregate_adam  # noqa: F401
from .shard_assign import (  # noqa: F401
    explicit_split,
    equal_split,
    minmax_split_bruteforce,
    minmax_objective,
    num_data_shards,
    data_shards,
    accumulation_plan_bruteforce,
)
from .dds_sim import (  # noqa: F401
    ShardQueue,
    SimConfig,
    SimResult,
    simulate_bsp,
    split_by_speed,
    equal_sizes,
    disturbed,
)
