"""Plain CPU oracle for blockwise parallel decoding (test infrastructure only).

Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may import
this package.  It shares no code with the HIP library and never calls it.
"""
from .transformer import CombinedModel, layer_norm, softmax_rows, multi_head_attention, feed_forward
from .decoding import (Decoded, Step, greedy_decode, blockwise_decode, blockwise_decode_two_calls,
                       accept_exact, accept_top_n, accept_distance)


def scorers(model: CombinedModel, src_ids, k=None):
    """(score, block_score) closures for one source sentence x.

    score(prefix)          -> z[k, V]     one full recomputation
    block_score(prefix, P) -> z[k, k, V]  all k block rows from ONE decoder pass over
                                          prefix + P (parallel scoring, Section 3)
    """
    memory = model.encode(src_ids)

    def score(prefix):
        return model.next_logits(memory, list(prefix), k)

    def block_score(prefix, P):
        kk = len(P)
        return model.all_position_logits(memory, list(prefix) + list(P), first=len(prefix) + 1, k=k)[:kk]

    return score, block_score
