// Roofline estimate of the expert stage (host arithmetic only; no device code).
//
// Paper Table 1, row 3 gives, per expert, the operand bytes D_X = 2*rows*d_h (inputs) and
// D_Y = 6*d_h*d_e (three bf16 matrices) and the work C = 6*rows*d_h*d_e FLOP; Eq. 5 prices an
// operation at M * max((D_X + D_Y) / BW_DEV, C / TF_DEV) over its M micro-batches, and Eq. 9
// applies the same form to the whole expert stage of one device. Coalesced execution is M = 1.
#include <cmath>

#include "common.h"

extern "C" int moe_estimate_expert_stage(const moe_shape* shape, const int32_t* rows,
                                         int32_t micro_batches, const moe_machine* machine,
                                         moe_expert_estimate* out) {
    if (!shape || !machine || !out || micro_batches < 0 || (micro_batches > 0 && !rows))
        return MOE_ERR_INVALID_ARG;
    if (shape->d_model <= 0 || shape->d_ff <= 0 || shape->E <= 0) return MOE_ERR_INVALID_ARG;
    if (!(machine->tflops > 0.0) || !(machine->gbytes_per_s > 0.0)) return MOE_ERR_INVALID_ARG;
    const double rate_flop = machine->tflops * 1e12, rate_byte = machine->gbytes_per_s * 1e9;
    const double dh = shape->d_model, de = shape->d_ff;
    const double weights = 6.0 * dh * de;                       // D_Y of one expert
    moe_expert_estimate e{};
    e.micro_batches = micro_batches;
    for (int32_t m = 0; m < micro_batches; ++m) {
        double bytes = 0.0, flops = 0.0;                        // the whole micro-batch (Eq. 9)
        double gateup_b = 0.0, gateup_f = 0.0, down_b = 0.0, down_f = 0.0;
        for (int32_t x = 0; x < shape->E; ++x) {
            const int32_t n = rows[static_cast<size_t>(m) * shape->E + x];
            if (n < 0) return MOE_ERR_INVALID_ARG;
            if (n == 0) continue;                               // an idle expert moves nothing
            const double inputs = 2.0 * n * dh;                 // D_X
            const double work = weights * n;                    // C = 6 * rows * d_h * d_e
            const double t_bytes = (inputs + weights) / rate_byte, t_work = work / rate_flop;
            e.expert_instances += 1;
            if (t_bytes > t_work) e.memory_bound_instances += 1;
            e.t_per_expert_s += t_bytes > t_work ? t_bytes : t_work;
            bytes += inputs + weights;
            flops += work;
            const double h_bytes = 2.0 * n * de;                // H, once written, once read
            e.intermediate_bytes += 2.0 * h_bytes + inputs;     // ... and y_perm, as large as the inputs
            gateup_b += inputs + weights * (2.0 / 3.0) + h_bytes;
            gateup_f += work * (2.0 / 3.0);
            down_b += h_bytes + weights / 3.0 + inputs;
            down_f += work / 3.0;
        }
        e.flops += flops;
        e.operand_bytes += bytes;
        const double t_b = bytes / rate_byte, t_f = flops / rate_flop;
        e.t_stage_s += t_b > t_f ? t_b : t_f;
        const double gu_b = gateup_b / rate_byte, gu_f = gateup_f / rate_flop;
        const double dn_b = down_b / rate_byte, dn_f = down_f / rate_flop;
        e.t_kernels_s += (gu_b > gu_f ? gu_b : gu_f) + (dn_b > dn_f ? dn_b : dn_f);
    }
    // rows per expert at which the two sides of the roofline meet
    const double slope = weights / rate_flop - 2.0 * dh / rate_byte;
    e.ridge_rows = slope > 0.0 ? (weights / rate_byte) / slope : HUGE_VAL;
    *out = e;
    return MOE_OK;
}

// Section 4.1.1 with a group of experts moved over PCIe: the load term of Eq. 7 next to the
// computation term of Eq. 9 (GPU side, every expert computed there); Eq. 3 sums them.
extern "C" int moe_estimate_streamed_stage(const moe_shape* shape, const int32_t* rows,
                                           int32_t n_moved, const moe_machine* machine,
                                           double pcie_gbytes_per_s, int32_t inputs_on_device,
                                           moe_streamed_estimate* out) {
    if (!shape || !rows || !machine || !out) return MOE_ERR_INVALID_ARG;
    if (shape->d_model <= 0 || shape->d_ff <= 0 || shape->E <= 0) return MOE_ERR_INVALID_ARG;
    if (n_moved < 0 || n_moved > shape->E || !(pcie_gbytes_per_s > 0.0)) return MOE_ERR_INVALID_ARG;
    moe_expert_estimate stage;
    const int rc = moe_estimate_expert_stage(shape, rows, 1, machine, &stage);
    if (rc != MOE_OK) return rc;
    const double dh = shape->d_model, de = shape->d_ff;
    double over_link = 6.0 * dh * de * n_moved;                 // EXP_M * D_Y3
    if (!inputs_on_device)
        for (int32_t x = 0; x < shape->E; ++x) over_link += 2.0 * dh * rows[x];   // D_X3
    moe_streamed_estimate e;
    e.moved_bytes = over_link;
    e.t_load_s = over_link / (pcie_gbytes_per_s * 1e9);
    e.t_comp_s = stage.t_stage_s;
    e.t_sum_s = e.t_load_s + e.t_comp_s;
    e.t_overlap_s = e.t_load_s > e.t_comp_s ? e.t_load_s : e.t_comp_s;
    *out = e;
    return MOE_OK;
}
