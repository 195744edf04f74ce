// Batched form of the subspace cosine check, shared with the subspace refresh.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace qg {

constexpr int kCosBatchMax = 16;
struct CosBatch {   // pair z: old projection (PqA, PsA)[z] against new projection (PqB, PsB)[z]
    const uint8_t* PqA[kCosBatchMax];
    const float* PsA[kCosBatchMax];
    const uint8_t* PqB[kCosBatchMax];
    const float* PsB[kCosBatchMax];
};

// cos_out[z] for z < count <= kCosBatchMax; ws holds cossim_batch_workspace_bytes(m, r, count) bytes.  weights
// (nullable): pair z weights its column cosines with weights[z * w_stride + k], k < r.
int launch_cossim_batch(const CosBatch& batch, int count, int64_t m, int64_t r, float* cos_out, float* ws,
                        hipStream_t stream, const float* weights, int64_t w_stride);
size_t cossim_batch_workspace_bytes(int64_t m, int64_t r, int count);

}  // namespace qg
