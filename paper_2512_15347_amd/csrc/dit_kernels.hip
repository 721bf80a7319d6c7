// placeholder until the network kernels land
#include "ctx.hpp"
namespace pg {
pg_status net_plan(pg_ctx* c) { c->net = NetPlan{}; return PG_OK; }
pg_status net_prepare(pg_ctx*, hipStream_t) { return fail(PG_EINVAL, "network kernels not built"); }
pg_status net_forward(pg_ctx*, int, hipStream_t) { return fail(PG_EINVAL, "network kernels not built"); }
}
extern "C" pg_status pg_gemm_bf16(const uint16_t*, int64_t, const uint16_t*, int64_t, const uint16_t*, float*, int64_t, int64_t, int64_t, int64_t, void*) { return pg::fail(PG_EINVAL, "not built"); }
extern "C" pg_status pg_attention_bf16(const uint16_t*, const uint16_t*, const uint16_t*, uint16_t*, int32_t, int32_t, int32_t, int32_t, int32_t, void*) { return pg::fail(PG_EINVAL, "not built"); }
