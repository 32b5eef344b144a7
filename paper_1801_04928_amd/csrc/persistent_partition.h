// Which worker partition a gradient worker workgroup of the persistent backward kernel belongs to and which rows
// of a layer it stores, as plain functions so that host code (and a host-only unit test) can evaluate exactly
// what the kernel evaluates.
//
// Layer l belongs to worker (L - l) mod k (section 3); worker j is the partition of workgroups with slot % k == j,
// and member slot / k of a partition with m members stores rows [member * ceil(N / m), ...) of its layers.
// The slot is the workgroup's index among the workers, or a permutation of it:
// workgroups are dealt to the 8 XCDs round-robin, so slot = index confines a partition to 8 / gcd(k, 8) of the
// XCDs -- to one, for k = 8 -- and a layer's stores to those XCDs' ports.  When k is a multiple of 4 (and divides
// the workers per XCD) the partition is therefore taken from index / 8 instead, and a partition's members are
// numbered XCD by XCD within each run of 8k workgroups: every partition then has members on every XCD, and
// neighbouring blocks of rows still leave through different XCDs.
// (L = 64, N = 4096: 1.64 -> 1.53 ms at k = 8, 1.56 -> 1.51 ms at k = 4.  k = 2, whose partitions have four XCDs
// each anyway, is faster as it is.)
#pragma once

#if defined(__HIPCC__)
#define LF_PARTITION_HD __host__ __device__
#else
#define LF_PARTITION_HD
#endif

namespace lf {

LF_PARTITION_HD inline int worker_slot(int wid, int nworkers, int k, bool spread) {
    if (spread && k % 4 == 0 && nworkers % 8 == 0 && (nworkers / 8) % k == 0)
        return (((wid / 8) / k) * 8 + wid % 8) * k + (wid / 8) % k;
    return wid;
}
// Members of partition `part`: the slots part, part + k, ... below nworkers.
LF_PARTITION_HD inline int partition_members(int part, int nworkers, int k) { return (nworkers - part + k - 1) / k; }
// First row and end of the rows that member `member` of a partition with `members` members stores, of N rows.
LF_PARTITION_HD inline void member_rows(int member, int members, int N, int* begin, int* end) {
    const int per = (N + members - 1) / members;
    const int b = member * per < N ? member * per : N;
    *begin = b;
    *end = b + per < N ? b + per : N;
}

}  // namespace lf
