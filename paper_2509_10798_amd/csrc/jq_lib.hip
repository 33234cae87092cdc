// libjq.so is built from this ONE translation unit.
//
// Why: the four kernels of an eviction step (both passes over K, pooling, selection + gather) run back to back,
// thousands of times, and the instruction cache of a compute-unit pair (64 KB) keeps its contents across kernel
// launches.  Their code is 62 KB together.  Compiled as separate translation units every file becomes a code
// object of its own and the loader decides where each one goes; in one code object the kernels lie where the
// order of definitions and instantiations puts them, and that order is chosen so that those four are neighbours:
// the non-template kernels come first in the order of the includes below (the selection's last), then the
// kernel templates in the order of their first instantiation -- which is why jq_score.hip and jq_pool.hip
// instantiate the instances of the headline shape explicitly, ahead of their launch switches.  A contiguous
// stretch of code no larger than the cache maps onto it without two lines competing for a place.  Measured with
// the builds loaded side by side in one process, on the same buffers: 1.1-1.8 us per step less than the same
// sources built file by file (selection 18.8 -> 18.0 us, first pass up to 0.7 us).
#include "jq_score.hip"
#include "jq_pool.hip"
#include "jq_compact.hip"
#include "jq_select.hip"
#include "jq_api.hip"
