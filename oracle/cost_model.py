"""Roofline cost of the expert stage (OP_3), written out from the paper's cost model.
Test infrastructure only: the library's estimator (moe_estimate_expert_stage) is checked
against this file, and this file against hand-derived values.

Quantities follow Table 1, row 3 (per expert: operand bytes D_X = 2*rows*d_h, D_Y = 6*d_h*d_e,
FLOPs C = 6*rows*d_h*d_e, bf16) and the roofline latency of Eq. 5,
    T_comp = M * max((D_X + D_Y) / BW_DEV, C / TF_DEV),
specialised to the expert stage as in Eq. 9 with every expert resident on the one device.
The table's "2BLd_h/E" is the uniform-routing average; here each expert has its own row count.
All arithmetic is plain Python floats (fp64), one expert and one micro-batch at a time.
"""
from __future__ import annotations


def expert_stage_estimate(rows, d_model, d_ff, tflops, gbytes_per_s):
    """rows: list (micro-batches) of lists (experts) of routed row counts.

    Returns a dict with
      flops              sum of C over experts and micro-batches
      operand_bytes      sum of D_X + D_Y over the experts that received rows
      intermediate_bytes H written and read (2*rows*d_e each) and the outputs written (2*rows*d_h)
      t_stage_s          Eq. 9 form: per micro-batch max(sum bytes / BW, sum C / TF), summed
      t_per_expert_s     Eq. 5 expert by expert: sum of max((D_X + D_Y) / BW, C / TF)
      t_kernels_s        gate/up and down as two grouped contractions per micro-batch, each
                         max(bytes / BW, FLOPs / TF) with the intermediate H counted
      expert_instances, memory_bound_instances, micro_batches, ridge_rows
    """
    BW = gbytes_per_s * 1e9
    TF = tflops * 1e12
    d, f = float(d_model), float(d_ff)
    out = dict(flops=0.0, operand_bytes=0.0, intermediate_bytes=0.0, t_stage_s=0.0,
               t_per_expert_s=0.0, t_kernels_s=0.0, expert_instances=0,
               memory_bound_instances=0, micro_batches=len(rows))
    for mb in rows:
        mb_bytes = mb_flops = 0.0
        gu_bytes = gu_flops = dn_bytes = dn_flops = 0.0
        for r in mb:
            if r <= 0:
                continue
            r = float(r)
            d_x = 2.0 * r * d                    # expert input rows, bf16
            d_y = 6.0 * d * f                    # the three d_h x d_e matrices, bf16
            c = 6.0 * r * d * f
            t_mem, t_cmp = (d_x + d_y) / BW, c / TF
            out["expert_instances"] += 1
            out["memory_bound_instances"] += 1 if t_mem > t_cmp else 0
            out["t_per_expert_s"] += max(t_mem, t_cmp)
            mb_bytes += d_x + d_y
            mb_flops += c
            out["intermediate_bytes"] += 4.0 * r * f + 2.0 * r * d
            gu_bytes += d_x + 4.0 * d * f + 2.0 * r * f
            gu_flops += 4.0 * r * d * f
            dn_bytes += 2.0 * r * f + 2.0 * d * f + 2.0 * r * d
            dn_flops += 2.0 * r * d * f
        out["flops"] += mb_flops
        out["operand_bytes"] += mb_bytes
        out["t_stage_s"] += max(mb_bytes / BW, mb_flops / TF)
        out["t_kernels_s"] += max(gu_bytes / BW, gu_flops / TF) + max(dn_bytes / BW, dn_flops / TF)
    # rows at which (2*r*d + 6*d*f)/BW == 6*r*d*f/TF
    denom = 6.0 * d * f / TF - 2.0 * d / BW
    out["ridge_rows"] = (6.0 * d * f / BW) / denom if denom > 0 else float("inf")
    return out


def streamed_expert_stage_estimate(rows, d_model, d_ff, n_moved, tflops, gbytes_per_s,
                                   pcie_gbytes_per_s, inputs_on_device=True):
    """Expert stage with n_moved experts' weights brought over PCIe (the paper's EXP_M group).

    rows: list (experts) of routed row counts of the one coalesced batch (m_exp = B).
      t_load_s     Eq. 7:  (D_X3 + EXP_M * D_Y3) / BW_PCIe, with D_Y3 = 6*d_h*d_e per expert and
                   D_X3 = 2*rows*d_h over all experts' inputs, left out when they already sit on
                   the device
      t_comp_s     Eq. 9 for the GPU with every expert computed there: max(bytes / BW, C / TF)
      t_sum_s      Eq. 3: T_load + T_comp (no T_store in the expert stage, Eq. 6)
      t_overlap_s  max(T_load, T_comp): transfer fully hidden behind computation or the reverse
    """
    d, f = float(d_model), float(d_ff)
    pcie = pcie_gbytes_per_s * 1e9
    if not 0 <= n_moved <= len(rows):
        raise ValueError("n_moved out of range")
    moved = n_moved * 6.0 * d * f
    if not inputs_on_device:
        moved += sum(2.0 * float(r) * d for r in rows if r > 0)
    t_load = moved / pcie
    t_comp = expert_stage_estimate([list(rows)], d_model, d_ff, tflops, gbytes_per_s)["t_stage_s"]
    return dict(moved_bytes=moved, t_load_s=t_load, t_comp_s=t_comp, t_sum_s=t_load + t_comp,
                t_overlap_s=max(t_load, t_comp))
