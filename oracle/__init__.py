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
disturbed and backup-worker runs, the Eq. 3 split it converges to, and the rate
of its pseudo-random disturbance pattern.
Parity unpinned: the paper prints no worked numeric example of an iteration or
of a schedule, so no pin is a printed value; the decision rules of the
job-completion-time model beyond those closed forms (window bookkeeping, the
order of kill and batch-size decisions) are a reading stated in dds_sim.py and
are pinned only by construction: **parity unpinned** for them.
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
