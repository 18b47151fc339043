// Layer-shared replica buffer (Section 5.1): the parameter arrays carry EP*r replica slots behind
// the E home experts, refilled for every micro-batch and layer.  The forward push copies each
// live replica's home parameters into its slot.  It is meant to run beside compute on a second
// stream, so the launch takes a small, caller-chosen number of workgroups (the counterpart of
// the paper's few-SM persistent copy kernel): each walks the copy list with a grid stride and
// exits when the list is done.
#include "common.h"

namespace relibra {

// One launch copies, for every slot s with replica_expert[s] = e >= 0, the three parameter
// blocks of expert e (per_expert_vec 16-byte vectors each) to slot E + s.
__global__ void __launch_bounds__(256)
replica_push_kernel(uint4 *__restrict__ Wg, uint4 *__restrict__ Wu, uint4 *__restrict__ Wd,
                    const int32_t *__restrict__ replica_expert, int n_slots, int E, size_t per_expert_vec,
                    int32_t *__restrict__ err_flag)
{
    const size_t stride = (size_t)gridDim.x * 256;
    for (int s = 0; s < n_slots; ++s) {
        const int e = replica_expert[s];
        if (e < 0) continue;                               // empty slot
        if (e >= E) {
            if (blockIdx.x == 0 && threadIdx.x == 0) atomicOr(err_flag, RELIBRA_ERR_ID_RANGE);
            continue;
        }
        const size_t src = (size_t)e * per_expert_vec, dst = (size_t)(E + s) * per_expert_vec;
        for (int which = 0; which < 3; ++which) {
            uint4 *__restrict__ W = which == 0 ? Wg : which == 1 ? Wu : Wd;
            size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
            // four independent 16-byte copies per trip
            for (; i + 3 * stride < per_expert_vec; i += 4 * stride) {
                const uint4 a = W[src + i], b = W[src + i + stride], c = W[src + i + 2 * stride], d = W[src + i + 3 * stride];
                W[dst + i] = a;
                W[dst + i + stride] = b;
                W[dst + i + 2 * stride] = c;
                W[dst + i + 3 * stride] = d;
            }
            for (; i < per_expert_vec; i += stride) W[dst + i] = W[src + i];
        }
    }
}

// Gradient return: for every live slot s (replica_expert[s] = e >= 0), in ascending slot order,
// dW[e] += dW[E + s], for the three gradient tensors (per_expert_vec float4 vectors each).  A
// thread owns element positions and walks the slots in order, so every element's sum has the same
// fixed order as the in-line sum of the backward call: results are identical bit for bit.
__global__ void __launch_bounds__(256)
replica_pull_kernel(float4 *__restrict__ dWg, float4 *__restrict__ dWu, float4 *__restrict__ dWd,
                    const int32_t *__restrict__ replica_expert, int n_slots, int E, size_t per_expert_vec,
                    int32_t *__restrict__ err_flag)
{
    const size_t stride = (size_t)gridDim.x * 256;
    bool bad = false;
    for (int which = 0; which < 3; ++which) {
        float4 *__restrict__ dW = which == 0 ? dWg : which == 1 ? dWu : dWd;
        for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < per_expert_vec; i += stride)
            for (int s = 0; s < n_slots; ++s) {
                const int e = replica_expert[s];
                if (e < 0) continue;
                if (e >= E) { bad = true; continue; }
                const float4 src = dW[(size_t)(E + s) * per_expert_vec + i];
                float4 *dst = &dW[(size_t)e * per_expert_vec + i];
                float4 d = *dst;
                d.x += src.x; d.y += src.y; d.z += src.z; d.w += src.w;
                *dst = d;
            }
    }
    if (bad && blockIdx.x == 0 && threadIdx.x == 0) atomicOr(err_flag, RELIBRA_ERR_ID_RANGE);
}

}  // namespace relibra

using namespace relibra;

extern "C" int relibra_replica_push(void *Wg_dev, void *Wu_dev, void *Wd_dev,
                                    const int32_t *replica_expert_dev, int E, int EP, int r, int h, int hff,
                                    int n_workgroups, int32_t *err_flag_dev, relibra_stream stream_)
{
    hipStream_t stream = (hipStream_t)stream_;
    if (E < 1 || EP < 1 || r < 0 || h < 8 || hff < 8 || n_workgroups < 1) return RELIBRA_EINVAL;
    if (((size_t)h * hff) % 8) return RELIBRA_EUNSUPPORTED;
    if (r == 0) return RELIBRA_OK;
    if (!Wg_dev || !Wu_dev || !Wd_dev || !replica_expert_dev || !err_flag_dev) return RELIBRA_EINVAL;
    if (!aligned16(Wg_dev) || !aligned16(Wu_dev) || !aligned16(Wd_dev)) return RELIBRA_EINVAL;
    const size_t per_expert_vec = (size_t)h * hff / 8;
    const int grid = n_workgroups > 4096 ? 4096 : n_workgroups;
    RELIBRA_LAUNCH(RELIBRA_K_REPLICA_PUSH, stream, replica_push_kernel<<<grid, 256, 0, stream>>>(
        (uint4 *)Wg_dev, (uint4 *)Wu_dev, (uint4 *)Wd_dev, replica_expert_dev, EP * r, E, per_expert_vec, err_flag_dev));
    RELIBRA_HIP_TRY(launch_check());
    return RELIBRA_OK;
}

extern "C" int relibra_replica_pull(float *dWg_dev, float *dWu_dev, float *dWd_dev,
                                    const int32_t *replica_expert_dev, int E, int EP, int r, int h, int hff,
                                    int n_workgroups, int32_t *err_flag_dev, relibra_stream stream_)
{
    hipStream_t stream = (hipStream_t)stream_;
    if (E < 1 || EP < 1 || r < 0 || h < 4 || hff < 4 || n_workgroups < 1) return RELIBRA_EINVAL;
    if (((size_t)h * hff) % 4) return RELIBRA_EUNSUPPORTED;
    if (r == 0) return RELIBRA_OK;
    if (!dWg_dev || !dWu_dev || !dWd_dev || !replica_expert_dev || !err_flag_dev) return RELIBRA_EINVAL;
    if (!aligned16(dWg_dev) || !aligned16(dWu_dev) || !aligned16(dWd_dev)) return RELIBRA_EINVAL;
    const size_t per_expert_vec = (size_t)h * hff / 4;
    const int grid = n_workgroups > 4096 ? 4096 : n_workgroups;
    RELIBRA_LAUNCH(RELIBRA_K_REPLICA_PULL, stream, replica_pull_kernel<<<grid, 256, 0, stream>>>(
        (float4 *)dWg_dev, (float4 *)dWu_dev, (float4 *)dWd_dev, replica_expert_dev, EP * r, E, per_expert_vec, err_flag_dev));
    RELIBRA_HIP_TRY(launch_check());
    return RELIBRA_OK;
}
