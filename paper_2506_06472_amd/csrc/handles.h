// Definitions of the opaque handle types of the C ABI.
#pragma once
#include <string>

#include "analysis.h"

struct tio_trace { tio::Trace t; };
struct tio_lifetimes { tio::Lifetimes l; };
struct tio_plan { tio::Plan p; };

namespace tio {
int fail(int code, const std::string &msg);   // records the thread-local message, returns code
}
