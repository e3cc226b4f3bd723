// Worker executor (internal): turns "gradient of the mini-batch loss" (Alg. 1, worker step 4)
// into a fixed sequence of kernel launches over a flat parameter vector, a flat gradient vector
// and a per-worker slice of the caller's workspace.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <string>

namespace dssp_model {

struct Plan;

Plan* create(int model_id, int batch, int n_classes, int K, void* workspace_dev, std::string& err);
void destroy(Plan* p);
int step(Plan* p, int worker, hipStream_t stream, const float* x, const int32_t* y, const float* w,
         float* g, float* loss, std::string& err);

}  // namespace dssp_model
