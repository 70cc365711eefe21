#include "bdr_internal.hpp"
namespace bdr {
int quantize_col(const bdr_format &, const void *, int, int64_t, int64_t, int64_t, void *, void *, void *, hipStream_t) { return BDR_ERR_LAUNCH; }
int dequantize_col(const bdr_format &, const void *, const void *, const void *, int64_t, int64_t, void *, int, int64_t, hipStream_t) { return BDR_ERR_LAUNCH; }
int qdq_col(const bdr_format &, const void *, void *, int, int64_t, int64_t, int64_t, hipStream_t) { return BDR_ERR_LAUNCH; }
}
