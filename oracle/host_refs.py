"""Plain Python statements of the two host-side helpers (TEST INFRASTRUCTURE ONLY).

map_layers follows the paper's Alg. 1 step by step, in its order and notation: for each
batch size, for each layer, scan the implementations for the smallest CPU+GPU time
(strict '<'), sum the minima, keep the batch size with the smallest sum (strict '<'), then
read the per-layer mapping of that batch size.

step_from_batchnorm is the definition the folding helper must agree with: batch-norm
followed by the sign, evaluated directly in float64 on an integer pre-activation
(paper Sec. II-A, step layer).  Tie convention (BN(x) == 0 gives -1) is this build's
reading: parity unpinned by the paper.
"""
import math


def map_layers(cpu_time, gpu_time):
    """cpu_time, gpu_time: [batch][layer][implem] nested lists."""
    MAX = math.inf
    proper_batch_size = 0
    result_time = MAX
    MAP = {}
    for batch_size in range(len(cpu_time)):
        sum_min_time = 0.0
        MAP[batch_size] = {}
        for layer in range(len(cpu_time[batch_size])):
            min_time = MAX
            for implem in range(len(cpu_time[batch_size][layer])):
                inference_time = cpu_time[batch_size][layer][implem] + gpu_time[batch_size][layer][implem]
                if inference_time < min_time:
                    min_time = inference_time
                    MAP[batch_size][layer] = implem
            sum_min_time = sum_min_time + min_time
        if sum_min_time < result_time:
            result_time = sum_min_time
            proper_batch_size = batch_size
    configuration = [MAP[proper_batch_size][layer] for layer in range(len(cpu_time[proper_batch_size]))]
    return proper_batch_size, configuration, result_time


def step_from_batchnorm(x, gamma, beta, mean, var, eps):
    """+1 / -1 for one integer pre-activation x and one channel's batch-norm parameters."""
    y = gamma * (x - mean) / math.sqrt(var + eps) + beta
    return 1 if y > 0 else -1
