// TEST INFRASTRUCTURE: what the host stand-ins record (see hip_stub.cpp).
#pragma once
#include <cstddef>
#include <vector>

#include "reduce_copy.h"

namespace shim {

struct Launch {
  bool fused;
  hcl::StepArgs step;        // !fused
  hcl::FusedArgs fusedargs;  // fused
  int dtype, nsrc, ndst;
  hcl::Tuning tune;
  void* stream;
};

struct StreamOp {
  enum Kind { RECORD, WAIT } kind;
  void* stream;
  void* event;
  size_t before_launch;  // number of launches recorded when the operation was issued
};

std::vector<Launch>& launches();
std::vector<StreamOp>& stream_ops();
void reset();

}  // namespace shim
