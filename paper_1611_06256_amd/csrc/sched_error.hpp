// Error text shared by the scheduler (sched.hip) and the adjustment rule (tuner.cpp): thread-local, read through
// ga3c_sched_last_error().  Defined in tuner.cpp, which is plain C++ and also builds without HIP.
#pragma once

namespace ga3c {
int sfail(int code, const char *fmt, ...);      // stores the text, returns code
const char *sched_error_text();
}  // namespace ga3c
