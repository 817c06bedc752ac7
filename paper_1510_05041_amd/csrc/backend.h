// Device interface used by the scheduler.  The product implementation is HipBackend
// (hip_backend.hip); tests substitute a host-only double to exercise the scheduling and
// caching logic without a GPU.  Everything asynchronous is expressed with the three
// primitives the paper's runtime relies on (Section IV.D): in-order streams, tile copies in
// both directions, and kernel launches -- plus events for cross-stream ordering.
#pragma once
#include <stddef.h>
#include <stdint.h>

#include <string>

#include "tile_step.h"

namespace blasx {

enum StreamRole { STREAM_COMPUTE = 0, STREAM_H2D = 1, STREAM_D2H = 2, STREAM_H2D_B = 3 };

class Backend {
public:
    virtual ~Backend() {}
    virtual char*  arena() = 0;            // device base address of the tile arena
    virtual size_t arena_bytes() = 0;
    virtual int    num_streams() = 0;      // 2..4
    // Use the first n (2..4) of the streams this backend was given or has made for the roles
    // below; streams are neither created anew nor destroyed.  Non-zero: n is out of range or
    // more than the caller handed over.  Only between calls (nothing in flight).
    virtual int    set_num_streams(int n) = 0;
    // Strided tile copies: `height` runs of `width` bytes.  Host pointers may be pageable.
    virtual int copy_h2d(void* dev_dst, size_t dpitch, const void* host_src, size_t spitch,
                         size_t width, size_t height, int stream) = 0;
    virtual int copy_d2h(void* host_dst, size_t dpitch, const void* dev_src, size_t spitch,
                         size_t width, size_t height, int stream) = 0;
    // Zeroes `height` runs of `width` bytes, `pitch` bytes apart, in device memory (width and the address
    // are multiples of 4): the padding of a ragged tile in its slot.
    virtual int fill_zero(void* dev, size_t pitch, size_t width, size_t height, int stream) = 0;
    virtual int launch(int dtype, bool ta, bool tb, int mode, const LaunchPack& pack, int stream) = 0;   // mode: step_mode()
    // Invert the nb x nb diagonal blocks of an n x n triangular tile (device pointers, column-
    // major); flags: TS_TRI_LOWER / TS_TRI_UNIT of the source.  Used by the TRSM diagonal step.
    virtual int launch_trtri_blocks(int dtype, const void* tri, int ld_tri, void* inv, int ld_inv, int n, int nb,
                                    uint32_t flags, int stream) = 0;
    // dst <- the n x n symmetric tile whose `lower` (or upper) triangle src stores (device pointers,
    // column-major); the other triangle of src is never read.  Used by the SYMM diagonal step.
    virtual int launch_symmetrize(int dtype, const void* src, int ld_src, void* dst, int ld_dst, int n, bool lower,
                                  int stream) = 0;
    // dst (cols x rows) <- transpose of src (rows x cols); device pointers, column-major.
    virtual int launch_transpose(int dtype, const void* src, int ld_src, int rows, int cols, void* dst, int ld_dst, int stream) = 0;
    // Events are small integers; event_destroy() hands one back for reuse.  After reserve_events(n)
    // the backend owns at least n events and event_create() never makes another one: it returns -1
    // when they are all in use (the allocation-free entry point must not create anything).
    virtual int  reserve_events(int n) = 0;
    virtual int  event_create() = 0;
    virtual void event_destroy(int ev) = 0;
    virtual int  event_record(int ev, int stream) = 0;
    virtual int  stream_wait_event(int stream, int ev) = 0;
    virtual bool event_done(int ev) = 0;   // non-blocking
    virtual int  event_sync(int ev) = 0;   // blocks the host
    virtual double event_elapsed_s(int ev_start, int ev_stop) = 0;  // both completed
    virtual int  sync_all() = 0;
    virtual const char* last_error() = 0;
};

// Provided once per library build: the HIP implementation in the product library, a host-only
// double in the test library.
Backend* make_backend(void* arena, size_t bytes, void* const* streams, int nstreams, std::string* err);
void* backend_host_alloc(size_t bytes);
int   backend_host_free(void* p);
// Frees device memory that the backend allocated itself and kept for a later init (blasx_shutdown).
void  backend_release_device_memory();
// The statically allocated tile arena of the current device (for callers that cannot allocate):
// device address and size.  Looked up once per device; non-zero on failure.
int   backend_static_arena(void** ptr, size_t* bytes);
// Whether [p, p + bytes) is host memory that the device can reach without staging (page-locked).
bool  backend_host_is_pinned(const void* p);
// Runs every instantiation of the tile kernel for `dtype` once with no work, so that the runtime
// has loaded them before a caller that cannot allocate launches them.  Non-zero on failure.
int   backend_warm_kernels(Backend& be, int dtype);

}  // namespace blasx
