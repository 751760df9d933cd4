// What the recording launch stubs saw (tests/test_host_sanitizer.py only).
#pragma once
#include <vector>
#include "seco_internal.h"

struct StubLog {
  int fwd = 0, dq = 0, dkdv = 0, delta = 0, zero = 0, axpy = 0, copy = 0, readout = 0, rope = 0;
  std::vector<seco::SegTable> dkdv_tables;   // one per dK/dV launch
  std::vector<seco::SegTable> dq_tables;     // one per dQ launch that carried runs
  std::vector<seco::RowRuns> row_runs;
  seco::AttnParams last;
  void clear() { *this = StubLog(); }
};
extern StubLog g_stub;
