// Generic query kernel, tables copied from device memory (biq_query); also the dispatcher that
// both variants are reached through.
#define BIQ_GENERIC_FUSED false
#define BIQ_GENERIC_NAME launch_query_generic_tables
#include "launch_generic.inc"

namespace biq {

hipError_t launch_query_generic_fused(int mu, int bt, const QueryParams& qp, int grid, int threads, int lds,
                                      hipStream_t s);

hipError_t launch_query_generic(bool fused, int mu, int bt, const QueryParams& qp, int grid, int threads,
                                int lds, hipStream_t s) {
    return fused ? launch_query_generic_fused(mu, bt, qp, grid, threads, lds, s)
                 : launch_query_generic_tables(mu, bt, qp, grid, threads, lds, s);
}

}  // namespace biq
