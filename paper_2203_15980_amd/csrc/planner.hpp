// Internal interface of the planner (see planner.cpp).
#pragma once
#include <cstdint>
#include <string>
#include <vector>

#include "../../include/delta.h"

namespace delta {

struct PlanTensor {
    uint64_t bytes = 0, cost_ns = 0;
    uint32_t flags = 0;
    std::vector<uint32_t> parents;
};

struct PlanStep {
    int32_t produces = -1;
    uint64_t cost_ns = 0;
    std::vector<uint32_t> reads;
};

delta_status load_graph(const delta_tensor_desc *tensors, uint32_t n_tensors,
                        const delta_step_desc *steps, uint32_t n_steps,
                        const delta_plan_params *params, std::vector<PlanTensor> &T,
                        std::vector<PlanStep> &S, std::string &err);

delta_status run_plan(const std::vector<PlanTensor> &tensors, const std::vector<PlanStep> &steps,
                      const delta_plan_params &params, std::vector<delta_event> &events,
                      uint64_t &peak, std::string &err);

}  // namespace delta
