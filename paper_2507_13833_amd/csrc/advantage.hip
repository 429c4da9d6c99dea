// Group-relative advantage (the GRPO "advantage" stage, App. B Table 2; advantages
// are part of the payload the Data Coordinator moves, Sec. 1) fused with its
// broadcast over the rollout layout's tokens.
//
// One launch, one wavefront per sequence.  The wave finds the sequence's prompt group,
// recomputes the group's mean and std from its G rewards (float64, in index order;
// cheaper than a second launch or a grid-wide dependency), writes adv_seq[i] and then
// streams the sequence's own token range: 4 mask bytes in, 16 bytes of float32 out per
// lane and step (5 B/token, HBM-bound).  A sequence is one contiguous run in its
// rollout shard, so no lane ever has to search for the sequence a token belongs to.
#include "advantage_device.h"

namespace dc {

constexpr int ADV_BLOCK = 256;
constexpr int ADV_WAVES = ADV_BLOCK / WAVE;

__global__ __launch_bounds__(ADV_BLOCK) void advantage_kernel(AdvArgs a, SourceDesc sd) {
    advantage_wave(a, sd, (int64_t)blockIdx.x * ADV_WAVES + __builtin_amdgcn_readfirstlane((int)(threadIdx.x / WAVE)));   // one wave per sequence
}

AdvArgs make_adv_args(int32_t n_seq, const SourceDesc& src, const int64_t* d_src_tok_off, const int32_t* d_seq_len,
                      const float* d_reward, const int32_t* d_group_off, int32_t n_groups, double eps, int32_t ddof,
                      const uint8_t* const* mask_base, float* d_adv_seq, float* const* adv_tok_base, int32_t* d_status) {
    AdvArgs a;
    a.n_seq = n_seq; a.n_groups = n_groups; a.ddof = ddof; a.eps = eps;
    a.src_tok_off = d_src_tok_off; a.seq_len = d_seq_len; a.reward = d_reward; a.group_off = d_group_off;
    a.adv_seq = d_adv_seq; a.status = d_status;
    a.per_token = adv_tok_base != nullptr;
    for (int s = 0; s < DC_MAX_SRC_SHARDS; ++s) {
        a.mask[s] = (a.per_token && s < src.n_src) ? mask_base[s] : nullptr;
        a.adv_tok[s] = (a.per_token && s < src.n_src) ? adv_tok_base[s] : nullptr;
    }
    return a;
}

hipError_t launch_advantage(int32_t n_seq, const SourceDesc& src, const int64_t* d_src_tok_off,
                            const int32_t* d_seq_len, const float* d_reward, const int32_t* d_group_off,
                            int32_t n_groups, double eps, int32_t ddof,
                            const uint8_t* const* mask_base, float* d_adv_seq, float* const* adv_tok_base,
                            int32_t* d_status, hipStream_t st) {
    const AdvArgs a = make_adv_args(n_seq, src, d_src_tok_off, d_seq_len, d_reward, d_group_off, n_groups, eps, ddof,
                                    mask_base, d_adv_seq, adv_tok_base, d_status);
    const int64_t grid = (adv_waves(n_seq, n_groups) + ADV_WAVES - 1) / ADV_WAVES;
    hipLaunchKernelGGL(advantage_kernel, dim3((unsigned)grid), dim3(ADV_BLOCK), 0, st, a, src);
    return hipGetLastError();
}

}  // namespace dc
