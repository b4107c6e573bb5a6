// Batched trace replay (placeholder entry points until the replay kernel lands).
#include "tg_internal.h"

extern "C" int tg_build_trace(const tg_trace_desc*, void*, tg_trace** out) { if (out) *out = nullptr; return TG_E_INVALID_ARG; }
extern "C" void tg_free_trace(tg_trace*) {}
extern "C" int tg_replay_workspace_bytes(const tg_trace*, size_t*) { return TG_E_INVALID_ARG; }
extern "C" int tg_replay_trace(const tg_trace*, const tg_replay_out*, void*, size_t, void*) { return TG_E_INVALID_ARG; }
