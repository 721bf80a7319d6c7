// placeholder until the network kernels land
#include "ctx.hpp"
namespace pg {
pg_status net_plan(pg_ctx* c) { c->net = NetPlan{}; return PG_OK; }
pg_status net_prepare(pg_ctx*, hipStream_t) { return fail(PG_EINVAL, "network kernels not built"); }
pg_status net_forward(pg_ctx*, int, hipStream_t) { return fail(PG_EINVAL, "network kernels not built"); }
}
