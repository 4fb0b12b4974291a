// Parameter blocks of the adaptive-layer kernels (see layer_kernels.hpp).
#pragma once

namespace spinner {

struct LayerForwardParams {
    const float* x;
    const float* d[3];
    float* y;
    float* saved1;
    float* saved2;
    long long batch;
    float factor;            // scale * n^{-3/2}
};

struct LayerBackwardParams {
    const float* dy;
    const float* x;
    const float* saved1;
    const float* saved2;
    const float* d[3];
    float* dx;
    float* partial;          // [slots][3][n]: per-slot sums over the vectors of that slot (unscaled)
    long long batch;
    long long slots;         // number of (workgroup, tile slot) pairs = stride between the vectors of one slot
    float factor;            // scale * n^{-3/2}
};

}  // namespace spinner
