// Subspace refresh (Algorithm 2, refresh branch): host interface used by the C ABI.
#pragma once
#include "common.hpp"
#include <vector>

namespace galore {

struct RefreshItem {
  const void* G;      // gradient, rows x cols, dtype dt, leading dimension ldg
  int64_t ldg;
  int64_t rows, cols;
  DType dt;
  void* proj;         // output projector (short side x r), dtype dt, leading dimension ldp
  int64_t ldp;
  void* proj_t;       // output, the projector transposed (r x short side), leading dimension ldpt
  int64_t ldpt;
  unsigned char* ws;  // refresh_workspace_bytes(short side, r) bytes, 256-byte aligned
  uint64_t seed;      // seed of the Gaussian start block
};

// Scratch one tensor's refresh needs (Gram matrix, two iteration blocks, Rayleigh-Ritz
// matrices, reflector data).
size_t refresh_workspace_bytes(int64_t kdim, int64_t r);

// Recompute the projectors of up to kMaxGroup tensors with grouped launches on `stream`: `iters`
// rounds of orthogonal iteration from the seeded Gaussian block, or, with `warm_start`, from what
// proj_t holds on entry (a previous projector of the same tensor; must have full rank).
// `crowded`: other refreshes run beside this one (overlapped calls), so kernels whose launches then
// outnumber the CUs use their smaller-workgroup variants.  Results do not depend on it.
hipError_t refresh_group(const std::vector<RefreshItem>& items, int r, int iters, bool warm_start, bool crowded, hipStream_t stream);

}  // namespace galore
