// Additive load-balancing loss (Eq. 4): inter = n * sum_i f_i P_i, intra = m * sum_j f_j Q_j with
// f = count / T and P, Q = probability sum / T; total = alpha*inter + beta*intra.  n + m values:
// one wave, each lane sums its strided share serially, then a fixed butterfly across lanes.
#include "smile_internal.hpp"

namespace smile {

namespace {

__global__ __launch_bounds__(64) void aux_loss_kernel(
    const int32_t *__restrict__ group_count, const int32_t *__restrict__ local_count,
    const float *__restrict__ p_sum, const float *__restrict__ q_sum, int T, int n, int m,
    float alpha, float beta, float *__restrict__ out3)
{
    aux_loss_wave(group_count, local_count, p_sum, q_sum, T, n, m, alpha, beta, out3);
}

}  // namespace

hipError_t launch_aux_loss(const smile_layer_desc &d, const int32_t *group_count, const int32_t *local_count,
                           const float *p_sum, const float *q_sum, float *out3, hipStream_t s)
{
    SMILE_LAUNCH(aux_loss_kernel, dim3(1), dim3(64), 0, s, group_count, local_count, p_sum, q_sum, d.T,
                       d.n_groups, d.m_local, d.alpha, d.beta, out3);
    return hipGetLastError();
}

}  // namespace smile
