// placeholder replaced below
#include "common.hpp"
namespace lithos {
int attn_plan(const lithos_op_t& op, OpPlan*) { return fail(LITHOS_EINVAL, "attention kind %d is not built", op.kind); }
int attn_launch(const lithos_op_t& op, const OpPlan&, const AtomArgs&, hipStream_t) { return fail(LITHOS_EINVAL, "attention kind %d is not built", op.kind); }
}
