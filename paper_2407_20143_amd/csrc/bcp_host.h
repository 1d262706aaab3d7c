// What the host-only part of the library (bcp_host.cpp: no GPU, no HIP headers, also built on its own
// with a plain C++ compiler and sanitizers) shares with the rest.
#pragma once
#include <string>

#include "bcp.h"

namespace bcp {

void set_error(const std::string& msg);  // thread-local text behind bcp_last_error()

// No exception leaves the library: every entry point that can allocate on the host is a function
// try block that ends here (call from inside a catch handler).
bcp_status on_exception(const char* who) noexcept;

// status and error text for an error code of the record checks (bcp_validate.h); `index`: the record's
// position on its side
bcp_status record_error(unsigned code, bool is_saved, int64_t index);

}  // namespace bcp
