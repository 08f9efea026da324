// The row kernels (row.hip) built a second time for many short rows: 512 threads per row, rows of
// at most 8192 ids, two workgroups per compute unit.  See the note at the head of row.hip.
#define SCD_ROW_BATCHED 1
#include "row.hip"
