// Test-side controls of the host-only HIP model (see hip/hip_runtime.h here).
#pragma once

#include <cstddef>

#include <hip/hip_runtime.h>

namespace stub {

void set_compute_units(int n);             // what hipDeviceGetAttribute reports
// false: the launch models skip the rows of q, k, v, out and the FP8 arrays (layers too large to allocate here)
void set_tensor_checks(bool on);
bool tensor_checks();
void* device_alloc(size_t bytes);          // "device" memory: an exact-size host allocation, registered
void device_free(void* p);
// true when [p, p + bytes) lies inside one live device allocation
bool in_device(const void* p, size_t bytes);

hipStream_t create_stream();               // a caller-owned stream
void destroy_stream(hipStream_t s);
void begin_capture(hipStream_t s);         // s becomes the origin of a capture
hipError_t end_capture(hipStream_t s);     // hipErrorStreamCaptureUnjoined when forked work was not joined back

// One forward pass writes every row of `out` exactly once: the harness opens a pass, the launch models
// report the rows they store (a second store of a row is a violation: two launches or items own it),
// the harness reads the count.
void new_forward();
void note_out_row(const void* row);
size_t out_rows_written();

// called by the launch models: the stream handle is checked, captured launches are counted
void note_launch(hipStream_t s, const char* what);
void violation(const char* fmt, ...);      // prints and counts a broken rule
int violations();
long launches();
long captured_nodes();

}  // namespace stub
