// Recording stand-ins for the kernel launchers declared in seco_internal.h: they never touch the pointers they are
// given (those are fake in the sanitizer run), only note what the host side decided to launch.
#include "stub_launch.h"

StubLog g_stub;

namespace seco {
int launch_fwd_f32(const AttnParams& p, hipStream_t) { g_stub.fwd++; g_stub.last = p; return SECO_OK; }
int launch_fwd_bf16(const AttnParams& p, hipStream_t) { g_stub.fwd++; g_stub.last = p; return SECO_OK; }
int launch_dq_f32(const AttnParams& p, const SegTable* r, hipStream_t) {
  g_stub.dq++; g_stub.last = p; if (r) g_stub.dq_tables.push_back(*r); return SECO_OK;
}
int launch_dq_bf16(const AttnParams& p, const SegTable* r, hipStream_t) {
  g_stub.dq++; g_stub.last = p; if (r) g_stub.dq_tables.push_back(*r); return SECO_OK;
}
int launch_dkdv_f32(const AttnParams& p, const SegTable& seg, hipStream_t) {
  g_stub.dkdv++; g_stub.last = p; g_stub.dkdv_tables.push_back(seg); return SECO_OK;
}
int launch_dkdv_bf16(const AttnParams& p, const SegTable& seg, hipStream_t) {
  g_stub.dkdv++; g_stub.last = p; g_stub.dkdv_tables.push_back(seg); return SECO_OK;
}
int launch_dkdv_rows_bf16(const AttnParams& p, const SegTable& seg, const RowRuns& rr, hipStream_t) {
  g_stub.dkdv++; g_stub.last = p; g_stub.dkdv_tables.push_back(seg); g_stub.row_runs.push_back(rr); return SECO_OK;
}
int launch_delta(const AttnParams&, int, hipStream_t) { g_stub.delta++; return SECO_OK; }
int launch_kvgrad_zero(float*, float*, int, int, int, const int64_t*, int64_t, int64_t, hipStream_t) {
  g_stub.zero++; return SECO_OK;
}
int launch_kvgrad_axpy(float*, float*, const float*, const float*, float, int, int, int, const int64_t*, int64_t, int64_t,
                       hipStream_t) { g_stub.axpy++; return SECO_OK; }
int launch_rows_copy(void*, void*, const void*, const void*, int, int, int, int, int, const int64_t*, const int64_t*,
                     int64_t, hipStream_t) { g_stub.copy++; return SECO_OK; }
int launch_readout(void*, void*, const float*, const float*, float, bool, int, int, int, int, const int64_t*,
                   const int64_t*, int64_t, hipStream_t) { g_stub.readout++; return SECO_OK; }
int launch_rope_rows(void*, const void*, void*, const void*, int, int, int, int, int, int, const int64_t*, const int64_t*,
                     int64_t, int64_t, int64_t, float, bool, float, hipStream_t) { g_stub.rope++; return SECO_OK; }
}  // namespace seco
