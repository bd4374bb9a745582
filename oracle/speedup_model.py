"""Single-node speed-up model of arXiv 1511.04561 (Appendix, "A theoretical single node model for
4 GPUs") -- test infrastructure, not the product.

The model: convolutional layers run data-parallel at single-GPU speed, the fully connected
layers run model-parallel over K sub-batches; communication that cannot be hidden under
computation is added as a penalty.  Speed-up = work of all GPUs over the time of one parallel pass:

    speedup = n_gpus * total / ((total - fc) + conv_penalty + sub_batches * parallel_fc + fc_penalty)

The fully connected penalty is the sum over the transfers of the part of each transfer that is
not covered by the computation it overlaps with, plus the transfers that overlap with nothing.
Plain double-precision arithmetic in the order written; nothing here is shared with the library.
"""


def penalty(pairs, unhidden=()):
    """pairs: (transfer_ms, overlapping_compute_ms); unhidden: transfers with nothing to hide under."""
    total = 0.0
    for transfer, compute in pairs:
        total = total + max(transfer - compute, 0.0)
    for transfer in unhidden:
        total = total + transfer
    return total


def speedup(n_gpus, total_ms, fc_ms, conv_penalty_ms, sub_batches, parallel_fc_ms, fc_penalty_ms):
    denominator = (total_ms - fc_ms) + conv_penalty_ms + sub_batches * parallel_fc_ms + fc_penalty_ms
    return n_gpus * total_ms / denominator
