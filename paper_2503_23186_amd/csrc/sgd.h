#pragma once
#include "common.h"

constexpr int kSgdMaxTensors = 48;

struct SgdTable {
  int count;
  int block_begin[kSgdMaxTensors + 1];
  float* w[kSgdMaxTensors];
  float* v[kSgdMaxTensors];
  const float* g[kSgdMaxTensors];
  void* wlp[kSgdMaxTensors];
  size_t n[kSgdMaxTensors];
};

// Fills block_begin and launches one kernel over all tensors of the table.
int sgd_multi(SgdTable& t, float lr, float mu, float wd, hipStream_t st);
