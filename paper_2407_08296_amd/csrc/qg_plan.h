// Launch plan of the grouped step: a flat blob (header + one record per matrix)
// built on the host, copied to the device by the caller, read by the grouped kernels.
#pragma once

#include <stdint.h>

#include "qgalore.h"

namespace qg {

constexpr uint32_t kPlanMagic = 0x51474C50u;  // "QGLP"

// Tile shapes of the grouped GEMM launches (must match the kernel instantiations).
constexpr int kManyProjBM = 128;  // rows of R (r) per tile
constexpr int kManyProjBN = 256;  // columns of R (n) per tile
constexpr int kManyBpBM = 128;    // rows of W (m) per tile
constexpr int kManyBpBN = 256;    // columns of W (n) per tile = one quantization block per row

struct PlanMatrix {
    int64_t m, n, r;
    int64_t ld;             // row pitch in elements of W, G, R, M, V, N (>= n)
    const uint8_t* Pq;
    const float* Ps;
    const uint16_t* G;
    int8_t* Wq;
    float* Ws;
    float* Wz;              // zero points of W (zero-point format) or null
    float* M;
    float* V;
    float* R;
    uint16_t* N;
    uint32_t adam_chunk0;   // first Adam chunk (workgroup) of this matrix
    uint32_t proj_tile0;    // first projection tile
    uint32_t bp_tile0;      // first back-projection tile
    uint32_t proj_tiles_r;  // tiles along r of the projection
    uint32_t bp_tiles_m;    // tiles along m of the back-projection
    uint32_t index;         // position in the caller's descriptor array (selects the SR seed of the matrix)
};

// The records are stored class by class, each class served by its own launch: shapes that need no edge checks,
// shapes with edges but 16-byte aligned rows, and the rest (see the kernels' edge modes).  A matrix takes the more
// demanding of the classes its projection and its back-projection need.  Tile indices (proj_tile0, bp_tile0) count
// within a class; Adam chunks run over all matrices.
constexpr int kPlanClasses = 3;
struct PlanHeader {
    uint32_t magic;
    int32_t count;
    uint32_t adam_chunks;
    uint32_t no_R;                        // 1 if some matrix has no R buffer
    int32_t class_count[kPlanClasses];    // matrices per class, in storage order
    uint32_t proj_tiles[kPlanClasses];
    uint32_t bp_tiles[kPlanClasses];
    uint32_t zero_points;                 // 1 if the weights carry zero points (all of them or none)
    uint32_t pad_[2];
};
static_assert(sizeof(PlanHeader) % 16 == 0, "records must stay 16-byte aligned");

__host__ __device__ inline const PlanMatrix* plan_matrices(const PlanHeader* h) {
    return reinterpret_cast<const PlanMatrix*>(h + 1);
}

}  // namespace qg
