"""CPU oracle for the MLPMoE branched forward and its slicing rules.

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the
benchmark's CPU-baseline leg.  The GPU library and its Python binding never
import anything from here, and nothing here imports them.
"""
from .forward import (build_oracle, dense_swiglu, mlpmoe_forward, mlpmoe_forward_routed, mlpmoe_hidden, num_threads,  # noqa: F401
                      rel_max_err, round_to_bf16)
from .fade import fade_block, fade_neurons, fractal_fade, linear_quantile, neuron_scores  # noqa: F401
from .slicing import (compact_layer, compensated_alpha, fade_sparsity, slice_plan,  # noqa: F401
                      split_sizes)
