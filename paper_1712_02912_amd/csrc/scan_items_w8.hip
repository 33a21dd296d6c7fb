// Second build of the tuned scan kernels for the work items of inverted lists: blocks of 8 waves,
// two per CU (each with its own 64 KB of tables), so that one block stages the tables of its next
// item while the other scans.  See scan_common.h.
#define PQ_TUNED_WAVES 8
#define PQ_TUNED_NS w8
#define PQ_TUNED_ITEMS_ONLY 1
#include "scan_tuned.hip"
