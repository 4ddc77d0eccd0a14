#include "dev_common.cuh"
int zk_zkrelu(zkdl_ctx* ctx, const int64_t* z_dev, const int64_t* ga_dev, uint64_t D, int Q, int R) {
    return ZKDL_EINVAL;
}
