// Internal declarations shared by the host-side planner and the HIP launchers.
#pragma once
#include <cstdarg>
#include <cstdint>
#include <cstring>

#include "mtf.h"

namespace mtf {

// Records `code` with a printf-style message in the calling thread's error slot; returns code.
int fail(int code, const char* fmt, ...);

// A validated tensor shape: names resolved to small integer ids that are unique per call.
struct Dims {
  int rank = 0;
  const char* name[MTF_MAX_RANK];
  int64_t size[MTF_MAX_RANK];
};

// Copies and checks a caller-supplied shape (NULL, rank range, positive sizes, duplicate names).
int load_shape(const mtf_shape* s, const char* what, Dims* out);

inline bool same(const char* a, const char* b) { return std::strcmp(a, b) == 0; }
inline int find(const Dims& d, const char* n) {
  for (int i = 0; i < d.rank; ++i)
    if (same(d.name[i], n)) return i;
  return -1;
}

// Per-dim (offset, local size) of the slice a processor holds ("Tensor Representations").
int slice_of(const Dims& t, const mtf_place* p, int64_t* offset, int64_t* size);

// A reshape that keeps rank and sizes and changes names (subsection "Reshape"): per tensor
// position, the mesh axis that splits it before / after (-1: not split) and the local sizes.
struct ReshapeInfo {
  int rank, mesh_rank;
  int64_t mesh_size[MTF_MAX_RANK];
  int in_axis[MTF_MAX_RANK], out_axis[MTF_MAX_RANK];
  int64_t in_local[MTF_MAX_RANK], out_local[MTF_MAX_RANK], out_offset[MTF_MAX_RANK];
  int64_t coord[MTF_MAX_RANK];
};
// need_coord: also validate p->coord and fill out_offset / coord (else they are 0).
int reshape_info(const Dims& in, const Dims& out, const mtf_place* p, bool need_coord, ReshapeInfo* r);

// A reshape that may change rank and sizes (the elements keep their row-major order): what the
// processor at p->coord holds of the output, and how any processor's input slice is cut.
struct GeneralReshapeInfo {
  int in_rank, out_rank, mesh_rank;
  int64_t mesh_size[MTF_MAX_RANK], coord[MTF_MAX_RANK];
  int in_axis[MTF_MAX_RANK];
  int64_t in_size[MTF_MAX_RANK], in_local[MTF_MAX_RANK];
  int64_t out_size[MTF_MAX_RANK], out_local[MTF_MAX_RANK], out_offset[MTF_MAX_RANK];
};
int reshape_general_info(const Dims& in, const Dims& out, const mtf_place* p, GeneralReshapeInfo* r);

// ---------------------------------------------------------------------------------------------
// Canonical form of a two-operand named einsum for the device kernels.
//
// Every dim of the union is one "loop"; a loop has an extent and an element stride in A, in B
// and in OUT (0 where the tensor lacks the dim).  Loops are grouped by role:
//   batch : in OUT and in both inputs        m : in OUT and A only       n : in OUT and B only
//   k     : in both inputs, not in OUT       ra / rb : in one input only, not in OUT
// Loops of one role that are contiguous in every tensor that has them are merged.
struct Loop {
  int64_t extent, sa, sb, so;
};
enum Role { R_BATCH = 0, R_M = 1, R_N = 2, R_K = 3, R_RA = 4, R_RB = 5, R_COUNT = 6 };
struct Canon {
  int n[R_COUNT];
  Loop loop[R_COUNT][MTF_MAX_RANK * 2];
  int64_t out_elems, space;  // elements of OUT; size of the whole iteration space
};
int canonicalize(const Dims& a, const Dims* b, const Dims& out, Canon* c);

}  // namespace mtf
