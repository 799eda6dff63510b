// The kernel in which every lane holds whole rows, for rows of more than DC_ROWS_SHORT_MAX elements.
#include "dc_rows.inl"

namespace dc {

// Blocks of the kernel that one compute unit holds at a time with `lds` bytes of LDS per block (0 if the query fails).
int rows_blocks_per_cu_long(const Plan& p, size_t lds) {
    int n = 0;
    hipError_t e = hipErrorInvalidValue;
    switch (p.M) {
#define DC_ROWS_CASE(m) case m: e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, dc_scan_rows_kernel<m, false>, DC_SCAN_THREADS, lds); break;
        DC_ROWS_CASE(13) DC_ROWS_CASE(14) DC_ROWS_CASE(15) DC_ROWS_CASE(16) DC_ROWS_CASE(17) DC_ROWS_CASE(18) DC_ROWS_CASE(22) DC_ROWS_CASE(26) DC_ROWS_CASE(30)
#undef DC_ROWS_CASE
        default: break;
    }
    return e == hipSuccess ? n : 0;
}

void launch_rows_scan_long(const Plan& p, const int32_t* lat, const uint32_t* tau_chunk, uint32_t kc, uint32_t* unit_max,
                      uint32_t* hist_part, uint32_t* status, hipStream_t stream) {
    switch (p.M) {
#define DC_ROWS_CASE(m) case m: launch_rows<m>(p, lat, tau_chunk, kc, unit_max, hist_part, status, stream); break;
        DC_ROWS_CASE(13) DC_ROWS_CASE(14) DC_ROWS_CASE(15) DC_ROWS_CASE(16) DC_ROWS_CASE(17) DC_ROWS_CASE(18) DC_ROWS_CASE(22) DC_ROWS_CASE(26) DC_ROWS_CASE(30)
#undef DC_ROWS_CASE
        default: break;                             // make_plan sets lane_rows for these row lengths only
    }
}

}  // namespace dc
