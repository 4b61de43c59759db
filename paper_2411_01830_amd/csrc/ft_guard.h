// No C++ exception may cross the C ABI: the entry points that allocate on the host are
// function-try-blocks that end in this handler.
#pragma once
#include <new>

#include "../../include/faastube.h"

#define FT_CATCH_ALL                                     \
  catch (const std::bad_alloc &) { return FT_ENOMEM; }   \
  catch (...) { return FT_EINVAL; }
