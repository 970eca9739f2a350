// The step list of one forward pass: what the host builds from the skip mask and launches step by step.
#pragma once
#include "asd_attn.h"
#include "asd_gemm.h"

enum { OP_EMBED = 0, OP_QKV = 1, OP_ATTN = 2, OP_OPROJ = 3, OP_GU = 4, OP_DOWN = 5, OP_LM = 6, OP_FINISH = 7 };

struct PassOp {
    int32_t type;
    int32_t grid;        // workgroups of the step's launch
    int32_t cls;         // ASD_K_* class (profiling / byte accounting)
    int32_t pad;
    double bytes;        // algorithmic bytes of the step
    GemmArgs g;
    AttnArgs t;
};
