"""CPU checker for the MaxScore routing hot path.  TEST INFRASTRUCTURE ONLY.

Imported by tests/, by the smoke check and by the benchmark's cpu_baseline leg; the product
package never imports it and it never imports the product.
"""
from .reference import (build, router_logits, softmax_rows, descending_rank, soft_topk, soft_topk_reading, quantise,
                        assign_literal_graph, assign_contracted, max_score_assignment,
                        max_score_assignment_caps, max_score_assignment_kvec, top1_then_residual, sinkhorn_plan, top1_then_sinkhorn,
                        max_flow_value, assignment_matrix, check_feasible, verify_optimal, gates,
                        dispatch, dispatch_tokens, combine, iter_reroute, sigmoid_scores, softkmax, itertopk, gradtopk, aux_loss, gates_backward, route, route_from_logits)
