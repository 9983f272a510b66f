// In-memory forest shared by the loader / evaluator (model.cpp) and the trainer (fit.cpp).
#pragma once
#include <cstdint>
#include <vector>

#include "mo.h"

struct mo_model {
    int32_t n_trees = 0;
    std::vector<int32_t> tree_off;   // n_trees + 1; node i of tree t lives at tree_off[t] + i
    std::vector<int32_t> feature, left, right, klass;
    std::vector<double> threshold;
};
