// Plain types shared by the device code (abs_kernels.hpp) and the host code that
// plans its launches: nothing here executes.
#pragma once

#include <stdint.h>

namespace absk {

constexpr int BLOCK = 256;             // threads per workgroup (4 wavefronts)
constexpr int ROW = BLOCK * 4;         // elements per workgroup row; tiles are whole rows

// Update rules of the fused combine + update pass.  Each keeps, besides x, up
// to two more per-parameter state vectors (s1, s2):
//   SGD   : s1 = momentum v                                   (s2 unused)
//   SGD_DC: s1 = momentum v,        s2 = previous iterate x_{t-1}
//   ADAM  : s1 = first moment m,    s2 = second moment v
//   SGD_DCM: s1 = momentum v; the compensation of SGD_DC with x_t - x_{t-1}
//            taken as -lr_{t-1} * v, which is what the previous update
//            subtracted from x (s2 unused, 8 bytes per parameter less traffic)
enum Rule { SGD = 0, SGD_DC = 1, ADAM = 2, SGD_DCM = 3 };

template <int RULE> constexpr bool uses_s2() { return RULE == SGD_DC || RULE == ADAM; }

struct Hyper {
    float M, lr, wd;
    float mu, lambda;                        // SGD, SGD_DC, SGD_DCM
    float nlr_prev;                          // SGD_DCM: minus the step size of the previous applied update
    float beta1, beta2, omb1, omb2, eps;     // ADAM: omb = 1 - beta (rounded to fp32 on the host)
    float bc1, bc2;                          // ADAM: 1 - beta^t, computed in double on the host
};

// Ragged layout: workgroup b looks its (tensor, tile index) up in a table.
struct Chunk { int32_t tensor; int32_t index; };

// One worker's share of a job-list accumulate launch.
constexpr int MAX_JOBS = 16;

struct Job {
    void *acc;              // flat: float*, the accumulator;  ragged: float *const *, its pointer table
    const void *g[8];       // flat: the gradients;            ragged: their pointer tables
    float n[8];             // sample counts, already converted
    int J;                  // gradients in this job, 1..8
    int first;              // the accumulator holds nothing yet
};

struct JobList { Job job[MAX_JOBS]; };

}  // namespace absk
