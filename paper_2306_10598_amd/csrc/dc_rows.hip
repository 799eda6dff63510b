// The kernel in which every lane holds whole rows, for rows of up to DC_ROWS_SHORT_MAX elements, and the dispatch over
// both halves of the row lengths (dc::lane_rows_length names the whole set for the host's plan).
#include "dc_rows.inl"

namespace dc {

// Blocks of the kernel that one compute unit holds at a time with `lds` bytes of LDS per block (0 if the query fails).
int rows_blocks_per_cu_short(const Plan& p, size_t lds) {
    int n = 0;
    hipError_t e = hipErrorInvalidValue;
    switch (p.M) {
#define DC_ROWS_CASE(m) case m: e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, dc_scan_rows_kernel<m, false>, DC_SCAN_THREADS, lds); break;
        DC_ROWS_CASE(1) DC_ROWS_CASE(2) DC_ROWS_CASE(3) DC_ROWS_CASE(4) DC_ROWS_CASE(5) DC_ROWS_CASE(6) DC_ROWS_CASE(7) DC_ROWS_CASE(8) DC_ROWS_CASE(9) DC_ROWS_CASE(10) DC_ROWS_CASE(11) DC_ROWS_CASE(12)
#undef DC_ROWS_CASE
        default: break;
    }
    return e == hipSuccess ? n : 0;
}

void launch_rows_scan_short(const Plan& p, const int32_t* lat, const uint32_t* tau_chunk, uint32_t kc, uint32_t* unit_max,
                      uint32_t* hist_part, uint32_t* status, hipStream_t stream) {
    switch (p.M) {
#define DC_ROWS_CASE(m) case m: launch_rows<m>(p, lat, tau_chunk, kc, unit_max, hist_part, status, stream); break;
        DC_ROWS_CASE(1) DC_ROWS_CASE(2) DC_ROWS_CASE(3) DC_ROWS_CASE(4) DC_ROWS_CASE(5) DC_ROWS_CASE(6) DC_ROWS_CASE(7) DC_ROWS_CASE(8) DC_ROWS_CASE(9) DC_ROWS_CASE(10) DC_ROWS_CASE(11) DC_ROWS_CASE(12)
#undef DC_ROWS_CASE
        default: break;                             // make_plan sets lane_rows for these row lengths only
    }
}

int rows_blocks_per_cu_long(const Plan& p, size_t lds);
void launch_rows_scan_long(const Plan& p, const int32_t* lat, const uint32_t* tau_chunk, uint32_t kc, uint32_t* unit_max,
                           uint32_t* hist_part, uint32_t* status, hipStream_t stream);

int rows_blocks_per_cu(const Plan& p, size_t lds) {
    return p.M <= DC_ROWS_SHORT_MAX ? rows_blocks_per_cu_short(p, lds) : rows_blocks_per_cu_long(p, lds);
}

void launch_rows_scan(const Plan& p, const int32_t* lat, const uint32_t* tau_chunk, uint32_t kc, uint32_t* unit_max,
                      uint32_t* hist_part, uint32_t* status, hipStream_t stream) {
    if (p.M <= DC_ROWS_SHORT_MAX) launch_rows_scan_short(p, lat, tau_chunk, kc, unit_max, hist_part, status, stream);
    else launch_rows_scan_long(p, lat, tau_chunk, kc, unit_max, hist_part, status, stream);
}

}  // namespace dc
