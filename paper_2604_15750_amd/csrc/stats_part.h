// Online-softmax state of a slice of one row of logits, and how two slices combine (Sec. 4.2: Eq. 3 and the entropy signal;
// Sec. 4.3: confidence and prediction).  Shared by the streamed vocabulary reduction and by the LM-head epilogue that produces
// the same states per column group.
#pragma once
#include "common.h"

constexpr float NEG_BIG = -3.0e38f;   // "minus infinity" that keeps every product finite
constexpr float MASKED = -1.0e30f;    // logit given to the mask token: e^(MASKED - m) == 0

struct Part {  // online-softmax state of a slice of one row
  float m, s, t, w;
  float bv;    // best logit
  int bi;      // its token id
  float pm, ps;  // max and sum e^(z'-pm) of the previous-step row (only when its lse is not stored)
};

static_assert(sizeof(Part) == STATS_STATE_BYTES, "the workspace is sized in states of 32 bytes");

__device__ inline Part part_init() { return Part{NEG_BIG, 0.f, 0.f, 0.f, NEG_BIG, 0x7fffffff, NEG_BIG, 0.f}; }

__device__ inline Part part_merge(const Part& a, const Part& b) {
  Part r;
  r.m = fmaxf(a.m, b.m);
  float da = a.m - r.m, db = b.m - r.m;
  float fa = __expf(da), fb = __expf(db);
  r.s = fa * a.s + fb * b.s;
  r.t = fa * (a.t + da * a.s) + fb * (b.t + db * b.s);
  r.w = fa * a.w + fb * b.w;
  bool tb = (b.bv > a.bv) || (b.bv == a.bv && b.bi < a.bi);
  r.bv = tb ? b.bv : a.bv;
  r.bi = tb ? b.bi : a.bi;
  r.pm = fmaxf(a.pm, b.pm);
  r.ps = __expf(a.pm - r.pm) * a.ps + __expf(b.pm - r.pm) * b.ps;
  return r;
}

__device__ inline Part part_shfl_xor(const Part& p, int o) {
  Part r;
  r.m = __shfl_xor(p.m, o, 64); r.s = __shfl_xor(p.s, o, 64); r.t = __shfl_xor(p.t, o, 64); r.w = __shfl_xor(p.w, o, 64);
  r.bv = __shfl_xor(p.bv, o, 64); r.bi = __shfl_xor(p.bi, o, 64); r.pm = __shfl_xor(p.pm, o, 64); r.ps = __shfl_xor(p.ps, o, 64);
  return r;
}

