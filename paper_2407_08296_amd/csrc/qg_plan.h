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
    const uint8_t* Pq;
    const float* Ps;
    const uint16_t* G;
    int8_t* Wq;
    float* Ws;
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

// The records are stored in two classes, each served by its own launch: first the `n_fast` matrices whose
// shapes fit the unguarded kernels, then the rest (bounds-checked kernels).  Tile indices (proj_tile0, bp_tile0)
// count within a class; Adam chunks run over all matrices.
struct PlanHeader {
    uint32_t magic;
    int32_t count;
    uint32_t adam_chunks;
    int32_t n_fast;            // matrices [0, n_fast) are the unguarded class
    uint32_t proj_tiles[2];    // per class: fast, guarded
    uint32_t bp_tiles[2];
    uint32_t no_R;             // 1 if some matrix has no R buffer
    uint32_t pad_[3];
};
static_assert(sizeof(PlanHeader) % 16 == 0, "records must stay 16-byte aligned");

__host__ __device__ inline const PlanMatrix* plan_matrices(const PlanHeader* h) {
    return reinterpret_cast<const PlanMatrix*>(h + 1);
}

}  // namespace qg
