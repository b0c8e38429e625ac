// Optional per-kernel timing shared by the entry-point files: a scope object records a HIP event on the launch
// stream when it is created and another when it goes out of scope (only while hstu_profile_enable(1) is in force).
#pragma once
#include <hip/hip_runtime.h>

namespace hstu {

struct ProfSlot;
struct ProfScope {
  ProfSlot* s;
  hipStream_t stream;
  ProfScope(const char* name, hipStream_t st);
  ~ProfScope();
  ProfScope(const ProfScope&) = delete;
  ProfScope& operator=(const ProfScope&) = delete;
};

}  // namespace hstu
