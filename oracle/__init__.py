"""Plain CPU oracle of the Bi-GCN forward path (test infrastructure only; see reference.py)."""

from .reference import (aggregate, aggregate_transposed, binarize_rows, binned_entropy, binarize_weight, column_standardisation,
                        forward, gat_layer, gcn_norm, layer, layer_backward, mean_norm, num_threads, pack_bits, predict, rescale,
                        sage_forward, sage_layer, set_num_threads, sign_matmul, unpack_bits, weight_gradient)

__all__ = ["aggregate", "aggregate_transposed", "binarize_rows", "binned_entropy", "binarize_weight", "column_standardisation", "forward",
           "gat_layer", "gcn_norm", "layer", "layer_backward", "mean_norm", "num_threads", "pack_bits", "predict", "rescale",
           "sage_forward", "sage_layer", "set_num_threads", "sign_matmul", "unpack_bits", "weight_gradient"]
