// Closing halves of the function try blocks around the extern "C" entry points that allocate host memory: no C++
// exception crosses the C boundary.  A failed host allocation reports GNNSTAGE_ENOMEM (-4), anything else
// GNNSTAGE_EINVAL (-1); size queries report 0.  No message is recorded on these paths (recording one allocates).
#pragma once
#include <new>

#define GNNSTAGE_GUARD_INT \
  catch (const std::bad_alloc &) { return -4; } \
  catch (...) { return -1; }
#define GNNSTAGE_GUARD_INT64 \
  catch (const std::bad_alloc &) { return -4; } \
  catch (...) { return -1; }
#define GNNSTAGE_GUARD_SIZE \
  catch (...) { return 0; }
