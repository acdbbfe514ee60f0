// placeholder until the scheduler is in place
#include "sts.h"
extern "C" int sts_sched_replay(const sts_profile*, const sts_model_desc*, const sts_sched_config*, const int64_t*, int64_t,
                                sts_decision*, int64_t, sts_replay_stats*) { return STS_EINVAL; }
