// Tags of the persistent kernels' exchanged words, as plain functions of a workgroup's launch count so that
// host code (and a host-only unit test) can evaluate exactly what the kernels evaluate.
//
// A tagged word carries the epoch of the launch that wrote it; 0 is the tag the buffers are cleared to and
// must never be produced.  Launch counts therefore run through 1 .. 2^31 - 1 and wrap back to 1.  The
// forward kernel tags with the count itself.  The backward kernel runs with two grids (with and without
// gradient worker workgroups), each with counts of its own: the grid with workers tags with 2 * count
// (even, 2 .. 2^32 - 2), the grid without with 2 * count + 1 (odd, 3 .. 2^32 - 1), so the words of one
// grid can never pass for the other's and neither ever produces 0.
#pragma once

#if defined(__HIPCC__)
#define LF_HOST_DEVICE __host__ __device__
#else
#define LF_HOST_DEVICE
#endif

namespace lf {

LF_HOST_DEVICE inline unsigned next_launch_count(unsigned c) {
    const unsigned n = (c + 1u) & 0x7fffffffu;
    return n != 0u ? n : 1u;
}
LF_HOST_DEVICE inline unsigned forward_epoch(unsigned count) { return count; }
LF_HOST_DEVICE inline unsigned backward_epoch(unsigned count, bool grid_has_workers) {
    return 2u * count + (grid_has_workers ? 0u : 1u);
}

}  // namespace lf
