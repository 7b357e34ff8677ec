// Optional per-kernel timing with HIP events on the launch stream (a measurement hook, off by default).
#pragma once
#include <hip/hip_runtime.h>

enum ProfId {
  PROF_PREP = 0, PROF_CMP_FWD, PROF_SLC_FWD, PROF_WIN_FWD, PROF_COMBINE,
  PROF_BWD_PREP, PROF_BWD_PRE, PROF_BWD_DQ_CMP, PROF_BWD_DQ, PROF_BWD_INVERT, PROF_BWD_DKV_WIN, PROF_BWD_DKV_SLC, PROF_BWD_DKV_CMP,
  PROF_BWD_FINISH, PROF_GENERIC, PROF_CMP_MODULE, PROF_CMP_MODULE_BWD, PROF_GATE_FWD, PROF_GATE_BWD,
  PROF_LINEAR_FWD, PROF_LINEAR_BWD, PROF_FWD_INVERT, PROF_BWD_DQ_MERGE, PROF_COUNT
};

bool prof_enabled();
void prof_begin(int id, hipStream_t s);
void prof_end(int id, hipStream_t s);

struct ProfScope {
  int id;
  hipStream_t s;
  bool on;
  ProfScope(int id_, hipStream_t s_) : id(id_), s(s_), on(prof_enabled()) {
    if (on) prof_begin(id, s);
  }
  ~ProfScope() {
    if (on) prof_end(id, s);
  }
};
