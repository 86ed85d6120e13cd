// Device side of libef, all of it: the tile scheme and its helpers (ef_tile.h),
// the worker kernels (ef_worker.h), the server kernels (ef_server.h), the
// kernels that finish a call and the parameter update (ef_finish.h), the
// compressor-quality diagnostics (ef_quality.h).
#pragma once
#include "ef_tile.h"
#include "ef_quality.h"
#include "ef_worker.h"
#include "ef_server.h"
#include "ef_finish.h"
