// Host-side integer logic: error slots, shape validation, mesh numbering, slices and the
// lowering plan of an einsum.  No GPU call is made from this file.
#include <cstdio>
#include <initializer_list>

#include "mtf_internal.h"

namespace mtf {

static thread_local char g_err[512] = "";

int fail(int code, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  int n = std::snprintf(g_err, sizeof g_err, "%s: ", mtf_status_string(code));
  if (n > 0 && n < (int)sizeof g_err) std::vsnprintf(g_err + n, sizeof g_err - n, fmt, ap);
  va_end(ap);
  return code;
}

int load_shape(const mtf_shape* s, const char* what, Dims* out) {
  if (!s) return fail(MTF_ERR_NULL, "%s shape", what);
  if (s->rank < 0 || s->rank > MTF_MAX_RANK) return fail(MTF_ERR_RANK, "%s rank %d", what, s->rank);
  if (s->rank > 0 && !s->dims) return fail(MTF_ERR_NULL, "%s dims", what);
  out->rank = s->rank;
  for (int i = 0; i < s->rank; ++i) {
    if (!s->dims[i].name) return fail(MTF_ERR_NULL, "%s dim %d name", what, i);
    if (s->dims[i].size <= 0)
      return fail(MTF_ERR_SIZE_MISMATCH, "%s dim '%s' has size %lld", what, s->dims[i].name,
                  (long long)s->dims[i].size);
    out->name[i] = s->dims[i].name;
    out->size[i] = s->dims[i].size;
    for (int j = 0; j < i; ++j)
      if (same(out->name[j], out->name[i]))
        return fail(MTF_ERR_DUP_DIM, "%s names '%s' twice", what, out->name[i]);
  }
  return MTF_OK;
}

// Mesh + rules + coordinate, checked once per call.
struct Place {
  Dims mesh;
  int n_rules = 0;
  const mtf_rule* rules = nullptr;
  int rule_axis[64];  // mesh axis of every rule
  const int64_t* coord = nullptr;
};

static int check_coord(const mtf_place* p, Place* out) {
  if (!p->coord) return fail(MTF_ERR_NULL, "coordinate");
  for (int i = 0; i < out->mesh.rank; ++i)
    if (p->coord[i] < 0 || p->coord[i] >= out->mesh.size[i])
      return fail(MTF_ERR_COORD_RANGE, "coordinate %lld on mesh dim '%s' of size %lld",
                  (long long)p->coord[i], out->mesh.name[i], (long long)out->mesh.size[i]);
  out->coord = p->coord;
  return MTF_OK;
}

static int load_place(const mtf_place* p, bool need_coord, Place* out) {
  if (!p) return fail(MTF_ERR_NULL, "place");
  if (int rc = load_shape(&p->mesh, "mesh", &out->mesh)) return rc;
  if (p->n_rules < 0 || p->n_rules > 64) return fail(MTF_ERR_RANK, "%d layout rules", p->n_rules);
  if (p->n_rules > 0 && !p->rules) return fail(MTF_ERR_NULL, "layout rules");
  out->n_rules = p->n_rules;
  out->rules = p->rules;
  for (int i = 0; i < p->n_rules; ++i) {
    const mtf_rule& r = p->rules[i];
    if (!r.tensor_dim || !r.mesh_dim) return fail(MTF_ERR_NULL, "layout rule %d", i);
    for (int j = 0; j < i; ++j)
      if (same(p->rules[j].tensor_dim, r.tensor_dim))
        return fail(MTF_ERR_DUP_RULE, "tensor dim '%s' is mapped twice", r.tensor_dim);
    out->rule_axis[i] = find(out->mesh, r.mesh_dim);
    if (out->rule_axis[i] < 0)
      return fail(MTF_ERR_UNKNOWN_MESH_DIM, "'%s' -> '%s'", r.tensor_dim, r.mesh_dim);
  }
  if (need_coord) return check_coord(p, out);
  return MTF_OK;
}

// Restriction of the layout to `t`: axis[i] = mesh axis dim i is split over, or -1.
static int restrict_layout(const Dims& t, const Place& pl, int* axis) {
  int owner[MTF_MAX_RANK];
  for (int m = 0; m < pl.mesh.rank; ++m) owner[m] = -1;
  for (int i = 0; i < t.rank; ++i) axis[i] = -1;
  for (int r = 0; r < pl.n_rules; ++r) {
    int i = find(t, pl.rules[r].tensor_dim);
    if (i < 0) continue;  // rule about a dim this tensor lacks: dropped by the restriction
    int m = pl.rule_axis[r];
    if (owner[m] >= 0)
      return fail(MTF_ERR_LAYOUT_CONFLICT, "dims '%s' and '%s' both split over mesh dim '%s'",
                  t.name[owner[m]], t.name[i], pl.mesh.name[m]);
    owner[m] = i;
    axis[i] = m;
  }
  return MTF_OK;
}

static int stripes(const Dims& t, const Place& pl, const int* axis, int64_t* offset, int64_t* size) {
  for (int i = 0; i < t.rank; ++i) {
    if (axis[i] < 0) {
      offset[i] = 0;
      size[i] = t.size[i];
      continue;
    }
    int64_t parts = pl.mesh.size[axis[i]];
    if (t.size[i] % parts)
      return fail(MTF_ERR_INDIVISIBLE, "dim '%s' of size %lld over mesh dim '%s' of size %lld",
                  t.name[i], (long long)t.size[i], pl.mesh.name[axis[i]], (long long)parts);
    size[i] = t.size[i] / parts;
    offset[i] = (pl.coord ? pl.coord[axis[i]] : 0) * size[i];
  }
  return MTF_OK;
}

// Order of checks (first failure wins): mesh and rules, injectivity of the tensor's layout,
// coordinate range, divisibility.
int slice_of(const Dims& t, const mtf_place* p, int64_t* offset, int64_t* size) {
  Place pl;
  if (int rc = load_place(p, false, &pl)) return rc;
  int axis[MTF_MAX_RANK];
  if (int rc = restrict_layout(t, pl, axis)) return rc;
  if (int rc = check_coord(p, &pl)) return rc;
  return stripes(t, pl, axis, offset, size);
}

int reshape_info(const Dims& in, const Dims& out, const mtf_place* p, bool need_coord, ReshapeInfo* r) {
  if (in.rank != out.rank) return fail(MTF_ERR_SIZE_MISMATCH, "reshape changes the rank (%d -> %d)", in.rank, out.rank);
  for (int i = 0; i < in.rank; ++i)
    if (in.size[i] != out.size[i])
      return fail(MTF_ERR_SIZE_MISMATCH, "reshape changes the size of position %d (%lld -> %lld)", i,
                  (long long)in.size[i], (long long)out.size[i]);
  Place pl;
  if (int rc = load_place(p, false, &pl)) return rc;
  if (int rc = restrict_layout(in, pl, r->in_axis)) return rc;
  if (int rc = restrict_layout(out, pl, r->out_axis)) return rc;
  if (need_coord)
    if (int rc = check_coord(p, &pl)) return rc;
  int64_t in_off[MTF_MAX_RANK];
  if (int rc = stripes(in, pl, r->in_axis, in_off, r->in_local)) return rc;
  if (int rc = stripes(out, pl, r->out_axis, r->out_offset, r->out_local)) return rc;
  r->rank = in.rank;
  r->mesh_rank = pl.mesh.rank;
  for (int m = 0; m < pl.mesh.rank; ++m) {
    r->mesh_size[m] = pl.mesh.size[m];
    r->coord[m] = need_coord ? p->coord[m] : 0;
  }
  return MTF_OK;
}

int reshape_general_info(const Dims& in, const Dims& out, const mtf_place* p, GeneralReshapeInfo* r) {
  int64_t n_in = 1, n_out = 1;
  for (int i = 0; i < in.rank; ++i) n_in *= in.size[i];
  for (int i = 0; i < out.rank; ++i) n_out *= out.size[i];
  if (n_in != n_out)
    return fail(MTF_ERR_SIZE_MISMATCH, "reshape changes the number of elements (%lld -> %lld)", (long long)n_in,
                (long long)n_out);
  Place pl;
  if (int rc = load_place(p, false, &pl)) return rc;
  int out_axis[MTF_MAX_RANK];
  if (int rc = restrict_layout(in, pl, r->in_axis)) return rc;
  if (int rc = restrict_layout(out, pl, out_axis)) return rc;
  if (int rc = check_coord(p, &pl)) return rc;
  int64_t in_off[MTF_MAX_RANK];
  if (int rc = stripes(in, pl, r->in_axis, in_off, r->in_local)) return rc;
  if (int rc = stripes(out, pl, out_axis, r->out_offset, r->out_local)) return rc;
  r->in_rank = in.rank;
  r->out_rank = out.rank;
  for (int i = 0; i < in.rank; ++i) r->in_size[i] = in.size[i];
  for (int i = 0; i < out.rank; ++i) r->out_size[i] = out.size[i];
  r->mesh_rank = pl.mesh.rank;
  for (int m = 0; m < pl.mesh.rank; ++m) {
    r->mesh_size[m] = pl.mesh.size[m];
    r->coord[m] = p->coord[m];
  }
  return MTF_OK;
}

// ------------------------------------------------------------------------- canonical einsum
static bool mergeable(const Loop& outer, const Loop& inner) {
  // outer/inner adjacent in every tensor that has them: outer stride = inner stride * extent
  auto ok = [&](int64_t so, int64_t si) { return so == si * inner.extent; };
  return ok(outer.sa, inner.sa) && ok(outer.sb, inner.sb) && ok(outer.so, inner.so);
}

int canonicalize(const Dims& a, const Dims* b, const Dims& out, Canon* c) {
  // union of dims in order of first appearance, with row-major strides per tensor
  Dims empty;
  const Dims& bb = b ? *b : empty;
  auto strides = [](const Dims& d, int64_t* s) {
    int64_t acc = 1;
    for (int i = d.rank - 1; i >= 0; --i) {
      s[i] = acc;
      acc *= d.size[i];
    }
    return acc;
  };
  int64_t sa[MTF_MAX_RANK], sb[MTF_MAX_RANK], so[MTF_MAX_RANK];
  strides(a, sa);
  strides(bb, sb);
  c->out_elems = strides(out, so);
  for (int i = 0; i < bb.rank; ++i) {
    int j = find(a, bb.name[i]);
    if (j >= 0 && a.size[j] != bb.size[i])
      return fail(MTF_ERR_SIZE_MISMATCH, "dim '%s' is %lld in a and %lld in b", bb.name[i],
                  (long long)a.size[j], (long long)bb.size[i]);
  }
  for (int i = 0; i < out.rank; ++i) {
    int ja = find(a, out.name[i]), jb = find(bb, out.name[i]);
    if (ja < 0 && jb < 0) return fail(MTF_ERR_OUT_NOT_SUBSET, "output dim '%s'", out.name[i]);
    int64_t sz = ja >= 0 ? a.size[ja] : bb.size[jb];
    if (sz != out.size[i])
      return fail(MTF_ERR_SIZE_MISMATCH, "dim '%s' is %lld in the output and %lld in an input",
                  out.name[i], (long long)out.size[i], (long long)sz);
  }
  for (int r = 0; r < R_COUNT; ++r) c->n[r] = 0;
  c->space = 1;
  // Visit the union in an order that keeps mergeable neighbours adjacent: OUT's dims in OUT's
  // order first (batch / m / n), then reduced dims in A's order, then B-only reduced dims.
  auto add = [&](const char* nm, int64_t extent) {
    int ia = find(a, nm), ib = find(bb, nm), io = find(out, nm);
    Loop l{extent, ia >= 0 ? sa[ia] : 0, ib >= 0 ? sb[ib] : 0, io >= 0 ? so[io] : 0};
    Role role = io >= 0 ? (ia >= 0 && ib >= 0 ? R_BATCH : (ia >= 0 ? R_M : R_N))
                        : (ia >= 0 && ib >= 0 ? R_K : (ia >= 0 ? R_RA : R_RB));
    c->space *= extent;
    if (extent == 1) return;  // contributes nothing to addressing
    int& n = c->n[role];
    if (n > 0 && mergeable(c->loop[role][n - 1], l)) {
      Loop& prev = c->loop[role][n - 1];
      prev.extent *= l.extent;
      prev.sa = l.sa;
      prev.sb = l.sb;
      prev.so = l.so;
    } else {
      c->loop[role][n++] = l;
    }
  };
  for (int i = 0; i < out.rank; ++i) add(out.name[i], out.size[i]);
  for (int i = 0; i < a.rank; ++i)
    if (find(out, a.name[i]) < 0) add(a.name[i], a.size[i]);
  for (int i = 0; i < bb.rank; ++i)
    if (find(out, bb.name[i]) < 0 && find(a, bb.name[i]) < 0) add(bb.name[i], bb.size[i]);
  return MTF_OK;
}

}  // namespace mtf

using namespace mtf;

extern "C" {

const char* mtf_status_string(int code) {
  switch (code) {
    case MTF_OK: return "MTF_OK";
    case MTF_ERR_NULL: return "MTF_ERR_NULL";
    case MTF_ERR_DUP_DIM: return "MTF_ERR_DUP_DIM";
    case MTF_ERR_SIZE_MISMATCH: return "MTF_ERR_SIZE_MISMATCH";
    case MTF_ERR_INDIVISIBLE: return "MTF_ERR_INDIVISIBLE";
    case MTF_ERR_LAYOUT_CONFLICT: return "MTF_ERR_LAYOUT_CONFLICT";
    case MTF_ERR_DUP_RULE: return "MTF_ERR_DUP_RULE";
    case MTF_ERR_UNKNOWN_MESH_DIM: return "MTF_ERR_UNKNOWN_MESH_DIM";
    case MTF_ERR_COORD_RANGE: return "MTF_ERR_COORD_RANGE";
    case MTF_ERR_OUT_NOT_SUBSET: return "MTF_ERR_OUT_NOT_SUBSET";
    case MTF_ERR_UNSUPPORTED: return "MTF_ERR_UNSUPPORTED";
    case MTF_ERR_WORKSPACE: return "MTF_ERR_WORKSPACE";
    case MTF_ERR_HIP: return "MTF_ERR_HIP";
    case MTF_ERR_RANK: return "MTF_ERR_RANK";
    case MTF_ERR_ALIGN: return "MTF_ERR_ALIGN";
    default: return "MTF_ERR_?";
  }
}

const char* mtf_last_error(void) { return g_err; }

int mtf_rank_to_coord(const mtf_shape* mesh, int64_t rank, int64_t* coord) {
  Dims m;
  if (int rc = load_shape(mesh, "mesh", &m)) return rc;
  if (!coord) return fail(MTF_ERR_NULL, "coord");
  int64_t total = 1;
  for (int i = 0; i < m.rank; ++i) total *= m.size[i];
  if (rank < 0 || rank >= total)
    return fail(MTF_ERR_COORD_RANGE, "rank %lld of %lld", (long long)rank, (long long)total);
  int64_t tmp[MTF_MAX_RANK];
  for (int i = m.rank - 1; i >= 0; --i) {  // last mesh dim fastest
    tmp[i] = rank % m.size[i];
    rank /= m.size[i];
  }
  for (int i = 0; i < m.rank; ++i) coord[i] = tmp[i];
  return MTF_OK;
}

int mtf_coord_to_rank(const mtf_shape* mesh, const int64_t* coord, int64_t* rank) {
  Dims m;
  if (int rc = load_shape(mesh, "mesh", &m)) return rc;
  if (!coord || !rank) return fail(MTF_ERR_NULL, "coord / rank");
  int64_t r = 0;
  for (int i = 0; i < m.rank; ++i) {
    if (coord[i] < 0 || coord[i] >= m.size[i])
      return fail(MTF_ERR_COORD_RANGE, "coordinate %lld on mesh dim '%s'", (long long)coord[i],
                  m.name[i]);
    r = r * m.size[i] + coord[i];
  }
  *rank = r;
  return MTF_OK;
}

int mtf_slice(const mtf_shape* t, const mtf_place* p, int64_t* offset, int64_t* size) {
  Dims d;
  if (int rc = load_shape(t, "tensor", &d)) return rc;
  if (!offset || !size) return fail(MTF_ERR_NULL, "offset / size");
  int64_t o[MTF_MAX_RANK], s[MTF_MAX_RANK];
  if (int rc = slice_of(d, p, o, s)) return rc;
  for (int i = 0; i < d.rank; ++i) {
    offset[i] = o[i];
    size[i] = s[i];
  }
  return MTF_OK;
}

int mtf_einsum_plan(const mtf_shape* a, const mtf_shape* b, const mtf_shape* out,
                    const mtf_place* p, int64_t* a_local, int64_t* b_local, int64_t* out_local,
                    uint32_t* reduce_mesh_dims_mask, int64_t* flops_local) {
  Dims da, db, dout;
  if (int rc = load_shape(a, "a", &da)) return rc;
  if (b)
    if (int rc = load_shape(b, "b", &db)) return rc;
  if (int rc = load_shape(out, "output", &dout)) return rc;
  // union of the operands' dims (may exceed MTF_MAX_RANK, so keep a wider table)
  const char* uname[2 * MTF_MAX_RANK];
  int64_t usize[2 * MTF_MAX_RANK];
  int un = 0;
  auto uni_find = [&](const char* nm) {
    for (int i = 0; i < un; ++i)
      if (same(uname[i], nm)) return i;
    return -1;
  };
  for (const Dims* d : {&da, &db})
    for (int i = 0; i < d->rank; ++i) {
      int j = uni_find(d->name[i]);
      if (j < 0) {
        uname[un] = d->name[i];
        usize[un++] = d->size[i];
      } else if (usize[j] != d->size[i]) {
        return fail(MTF_ERR_SIZE_MISMATCH, "dim '%s' is %lld and %lld", d->name[i],
                    (long long)usize[j], (long long)d->size[i]);
      }
    }
  for (int i = 0; i < dout.rank; ++i) {
    int j = uni_find(dout.name[i]);
    if (j < 0) return fail(MTF_ERR_OUT_NOT_SUBSET, "output dim '%s'", dout.name[i]);
    if (usize[j] != dout.size[i])
      return fail(MTF_ERR_SIZE_MISMATCH, "output dim '%s' is %lld, inputs have %lld", dout.name[i],
                  (long long)dout.size[i], (long long)usize[j]);
  }
  Place pl;
  if (int rc = load_place(p, false, &pl)) return rc;
  // layout restricted to the union: injective over the whole einsum
  int uaxis[2 * MTF_MAX_RANK], owner[MTF_MAX_RANK];
  for (int i = 0; i < un; ++i) uaxis[i] = -1;
  for (int m = 0; m < pl.mesh.rank; ++m) owner[m] = -1;
  for (int r = 0; r < pl.n_rules; ++r) {
    int i = uni_find(pl.rules[r].tensor_dim);
    if (i < 0) continue;
    int m = pl.rule_axis[r];
    if (owner[m] >= 0)
      return fail(MTF_ERR_LAYOUT_CONFLICT, "dims '%s' and '%s' both split over mesh dim '%s'",
                  uname[owner[m]], uname[i], pl.mesh.name[m]);
    owner[m] = i;
    uaxis[i] = m;
  }
  int64_t uloc[2 * MTF_MAX_RANK];
  int64_t space = 1;
  uint32_t mask = 0;
  for (int i = 0; i < un; ++i) {
    uloc[i] = usize[i];
    if (uaxis[i] >= 0) {
      int64_t parts = pl.mesh.size[uaxis[i]];
      if (usize[i] % parts)
        return fail(MTF_ERR_INDIVISIBLE, "dim '%s' of size %lld over mesh dim '%s' of size %lld",
                    uname[i], (long long)usize[i], pl.mesh.name[uaxis[i]], (long long)parts);
      uloc[i] = usize[i] / parts;
      if (find(dout, uname[i]) < 0) mask |= 1u << uaxis[i];  // reduced out and split
    }
    space *= uloc[i];
  }
  if (a_local)
    for (int i = 0; i < da.rank; ++i) a_local[i] = uloc[uni_find(da.name[i])];
  if (b_local)
    for (int i = 0; i < db.rank; ++i) b_local[i] = uloc[uni_find(db.name[i])];
  if (out_local)
    for (int i = 0; i < dout.rank; ++i) out_local[i] = uloc[uni_find(dout.name[i])];
  if (reduce_mesh_dims_mask) *reduce_mesh_dims_mask = mask;
  if (flops_local) *flops_local = 2 * space;
  return MTF_OK;
}

}  // extern "C"

extern "C" int mtf_reshape_plan(const mtf_shape* in, const mtf_shape* out, const mtf_place* p, int32_t* comm) {
  Dims din, dout;
  if (int rc = load_shape(in, "input", &din)) return rc;
  if (int rc = load_shape(out, "output", &dout)) return rc;
  if (!comm) return fail(MTF_ERR_NULL, "comm");
  ReshapeInfo r;
  if (int rc = reshape_info(din, dout, p, false, &r)) return rc;
  for (int m = 0; m < r.mesh_rank; ++m) {
    int pin = -1, pout = -1;
    for (int i = 0; i < r.rank; ++i) {
      if (r.in_axis[i] == m) pin = i;
      if (r.out_axis[i] == m) pout = i;
    }
    comm[m] = pin < 0 ? (pout < 0 ? MTF_COMM_NONE : MTF_COMM_SLICE)
                      : (pout < 0 ? MTF_COMM_ALLGATHER : (pin == pout ? MTF_COMM_NONE : MTF_COMM_ALLTOALL));
  }
  return MTF_OK;
}
