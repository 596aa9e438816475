// A small host model of the HIP runtime calls the library makes: streams and
// events are heap objects (a use after destroy is a heap-use-after-free for
// AddressSanitizer), stream capture follows the fork/join rules of the real
// runtime (a stream joins a capture by waiting on an event recorded in it; all
// forked work must be joined back before the capture ends; synchronising or
// destroying a capturing stream is an error), and device memory is host memory
// of the exact size asked for.
#include "hip_stub.h"

#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <map>
#include <set>
#include <unordered_set>

struct ihipStream_t {
  unsigned magic = 0x57AEA3u;
  ihipStream_t* origin = nullptr;         // capture this stream belongs to (itself for the origin)
  std::set<ihipStream_t*> forked;         // origin only: streams that joined its capture
  std::set<ihipStream_t*> unjoined;       // origin only: forked streams with work not yet joined back
  long last_work = 0;                     // sequence number of the last work enqueued
};
struct ihipEvent_t {
  unsigned magic = 0xE7E27u;
  ihipStream_t* origin = nullptr;         // capture the last record belongs to
  ihipStream_t* from = nullptr;           // stream of the last record
  long seq = 0;
  bool recorded = false;
};

namespace {
int g_cu = 256;
bool g_tensor_checks = true;
int g_violations = 0;
long g_launches = 0, g_nodes = 0, g_seq = 0;
int g_captures = 0;                        // captures in progress
std::map<const char*, size_t> g_allocs;
ihipStream_t g_null_stream;               // the default stream

ihipStream_t* resolve(hipStream_t s) { return s ? s : &g_null_stream; }
bool alive(ihipStream_t* s) { return s->magic == 0x57AEA3u; }   // reads the object: ASan reports a freed one
bool alive(ihipEvent_t* e) { return e->magic == 0xE7E27u; }

void work_on(ihipStream_t* s) {
  s->last_work = ++g_seq;
  if (s->origin && s->origin != s) s->origin->unjoined.insert(s);
}
}  // namespace

namespace stub {

void violation(const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  std::fprintf(stderr, "hip model violation: ");
  std::vfprintf(stderr, fmt, ap);
  std::fprintf(stderr, "\n");
  va_end(ap);
  ++g_violations;
}
int violations() { return g_violations; }
long launches() { return g_launches; }
long captured_nodes() { return g_nodes; }
void set_compute_units(int n) { g_cu = n; }

namespace {
std::unordered_set<const void*> g_out_rows;
}
void new_forward() { g_out_rows.clear(); }
void note_out_row(const void* row) {
  if (!g_out_rows.insert(row).second) violation("an output row is stored twice in one forward pass (launch %ld)", launches());
}
size_t out_rows_written() { return g_out_rows.size(); }
void set_tensor_checks(bool on) { g_tensor_checks = on; }
bool tensor_checks() { return g_tensor_checks; }

void* device_alloc(size_t bytes) {
  char* p = static_cast<char*>(std::malloc(bytes ? bytes : 1));
  std::memset(p, 0xCD, bytes);
  g_allocs[p] = bytes;
  return p;
}
void device_free(void* p) {
  g_allocs.erase(static_cast<const char*>(p));
  std::free(p);
}
bool in_device(const void* p, size_t bytes) {
  const char* c = static_cast<const char*>(p);
  auto it = g_allocs.upper_bound(c);
  if (it == g_allocs.begin()) return false;
  --it;
  return c >= it->first && c + bytes <= it->first + it->second;
}

hipStream_t create_stream() { return new ihipStream_t(); }
void destroy_stream(hipStream_t s) { (void)hipStreamDestroy(s); }

void begin_capture(hipStream_t s) {
  ihipStream_t* st = resolve(s);
  if (st->origin) violation("begin_capture on a stream that is already capturing");
  st->origin = st;
  st->forked.clear();
  st->unjoined.clear();
  ++g_captures;
}

hipError_t end_capture(hipStream_t s) {
  ihipStream_t* st = resolve(s);
  if (st->origin != st) {
    violation("end_capture on a stream that is not the origin of a capture");
    return hipErrorInvalidValue;
  }
  const bool unjoined = !st->unjoined.empty();
  for (ihipStream_t* f : st->forked)
    if (alive(f)) f->origin = nullptr;
  st->forked.clear();
  st->unjoined.clear();
  st->origin = nullptr;
  --g_captures;
  if (unjoined) violation("capture ended with forked work that was not joined back");
  return unjoined ? hipErrorStreamCaptureUnjoined : hipSuccess;
}

void note_launch(hipStream_t s, const char* what) {
  ihipStream_t* st = resolve(s);
  if (!alive(st)) violation("launch of %s on a dead stream", what);
  ++g_launches;
  if (st->origin) ++g_nodes;
  work_on(st);
}

}  // namespace stub

hipError_t hipGetDevice(int* device) {
  if (g_cu <= 0) return hipErrorUnknown;   // a box without a GPU
  *device = 0;
  return hipSuccess;
}
hipError_t hipDeviceGetAttribute(int* value, hipDeviceAttribute_t attr, int) {
  if (attr != hipDeviceAttributeMultiprocessorCount) return hipErrorInvalidValue;
  *value = g_cu;
  return hipSuccess;
}
hipError_t hipGetLastError() { return hipSuccess; }

hipError_t hipStreamCreateWithFlags(hipStream_t* stream, unsigned) {
  *stream = new ihipStream_t();
  return hipSuccess;
}
hipError_t hipStreamDestroy(hipStream_t stream) {
  if (!stream) return hipErrorInvalidResourceHandle;
  if (!alive(stream)) stub::violation("hipStreamDestroy of a dead stream");
  if (stream->origin) stub::violation("hipStreamDestroy of a stream that is capturing");
  stream->magic = 0;
  delete stream;
  return hipSuccess;
}
hipError_t hipStreamSynchronize(hipStream_t stream) {
  ihipStream_t* st = resolve(stream);
  if (!alive(st)) stub::violation("hipStreamSynchronize on a dead stream");
  if (st->origin) {
    stub::violation("hipStreamSynchronize on a capturing stream");
    return hipErrorStreamCaptureUnsupported;
  }
  return hipSuccess;
}
hipError_t hipDeviceSynchronize() {
  if (g_captures > 0) {
    stub::violation("hipDeviceSynchronize while a capture is active");
    return hipErrorStreamCaptureUnsupported;
  }
  return hipSuccess;
}
hipError_t hipStreamIsCapturing(hipStream_t stream, hipStreamCaptureStatus* status) {
  ihipStream_t* st = resolve(stream);
  if (!alive(st)) stub::violation("hipStreamIsCapturing on a dead stream");
  *status = st->origin ? hipStreamCaptureStatusActive : hipStreamCaptureStatusNone;
  return hipSuccess;
}
hipError_t hipEventCreateWithFlags(hipEvent_t* event, unsigned) {
  *event = new ihipEvent_t();
  return hipSuccess;
}
hipError_t hipEventDestroy(hipEvent_t event) {
  if (!event) return hipErrorInvalidResourceHandle;
  if (!alive(event)) stub::violation("hipEventDestroy of a dead event");
  event->magic = 0;
  delete event;
  return hipSuccess;
}
hipError_t hipEventRecord(hipEvent_t event, hipStream_t stream) {
  ihipStream_t* st = resolve(stream);
  if (!event || !alive(event) || !alive(st)) {
    stub::violation("hipEventRecord with a dead handle");
    return hipErrorInvalidResourceHandle;
  }
  event->origin = st->origin;
  event->from = st;
  event->seq = ++g_seq;
  event->recorded = true;
  return hipSuccess;
}
hipError_t hipStreamWaitEvent(hipStream_t stream, hipEvent_t event, unsigned) {
  ihipStream_t* st = resolve(stream);
  if (!event || !alive(event) || !alive(st)) {
    stub::violation("hipStreamWaitEvent with a dead handle");
    return hipErrorInvalidResourceHandle;
  }
  if (!event->recorded) return hipSuccess;
  if (event->origin) {
    ihipStream_t* o = event->origin;
    if (!alive(o) || o->origin != o) {
      stub::violation("wait on an event recorded in a capture that has ended");
      return hipErrorStreamCaptureIsolation;
    }
    if (st->origin && st->origin != o) {
      stub::violation("a stream of one capture waits on an event of another");
      return hipErrorStreamCaptureIsolation;
    }
    if (!st->origin) {   // joins the capture
      st->origin = o;
      o->forked.insert(st);
    }
    // the origin (or any stream of the capture) waiting on a forked stream's event joins that
    // stream's work up to the record
    ihipStream_t* f = event->from;
    if (f != o && f != st && alive(f) && f->last_work <= event->seq) o->unjoined.erase(f);
  } else if (st->origin) {
    stub::violation("a capturing stream waits on an event recorded outside the capture");
    return hipErrorStreamCaptureIsolation;
  }
  return hipSuccess;
}
hipError_t hipMemcpyAsync(void* dst, const void* src, size_t bytes, hipMemcpyKind kind, hipStream_t stream) {
  ihipStream_t* st = resolve(stream);
  if (!alive(st)) stub::violation("hipMemcpyAsync on a dead stream");
  if (st->origin) stub::violation("hipMemcpyAsync recorded into a capture (the forward pass promises launches only)");
  if (kind == hipMemcpyHostToDevice && !stub::in_device(dst, bytes)) stub::violation("H2D copy outside a device allocation");
  if (kind == hipMemcpyDeviceToHost && !stub::in_device(src, bytes)) stub::violation("D2H copy outside a device allocation");
  std::memcpy(dst, src, bytes);
  return hipSuccess;
}
