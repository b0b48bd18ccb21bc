// Device-side input check (debug aid): what the host-side validation of the C ABI cannot see --
// scenario / behaviour ids, candidate offsets and temperature entries that live in device memory.
// Eq. (3) of Climber (arXiv 2502.09888) divides a query row's logits by the temperature its
// (scenario, behaviour) pair selects, so an id must lie inside the table and the entry must be
// finite and positive.  One small kernel ORs problem bits into a caller-owned status word; it
// reads inside the given bounds only and always runs to completion.
#include "../../include/climber.h"

#include <cmath>

#include "internal.h"

namespace climber {
namespace {

struct CheckParams {
    const float *tau;
    const int32_t *scen, *beh, *cand_off;
    const int32_t *hist_len, *tok_off;  // history rows: valid-prefix geometry; nullptr for candidates
    int32_t *status;
    int64_t n_rows;
    int B, n_scen, n_beh, m_max;
};

__global__ __launch_bounds__(256) void check_inputs_kernel(const CheckParams p)
{
    int bad = 0;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    const int64_t i0 = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (p.hist_len) {
        // history rows: user b owns rows tok_off[b] .. tok_off[b+1]-1, the first hist_len[b] valid
        for (int b = 0; b < p.B; ++b) {
            const int64_t t0 = p.tok_off[b], n = p.hist_len[b];
            for (int64_t i = i0; i < n; i += stride) {
                const int sc = p.scen[t0 + i], bh = p.beh[t0 + i];
                if (sc < 0 || sc >= p.n_scen) bad |= CLIMBER_BAD_SCEN;
                if (bh < 0 || bh >= p.n_beh) bad |= CLIMBER_BAD_BEH;
                if (sc >= 0 && sc < p.n_scen && bh >= 0 && bh < p.n_beh) {
                    const float t = p.tau[sc * p.n_beh + bh];
                    if (!(t > 0.f) || !(t < INFINITY)) bad |= CLIMBER_BAD_TAU;
                }
            }
        }
    } else {
        for (int64_t i = i0; i < p.n_rows; i += stride) {
            const int sc = p.scen[i], bh = p.beh[i];
            if (sc < 0 || sc >= p.n_scen) bad |= CLIMBER_BAD_SCEN;
            if (bh < 0 || bh >= p.n_beh) bad |= CLIMBER_BAD_BEH;
            if (sc >= 0 && sc < p.n_scen && bh >= 0 && bh < p.n_beh) {
                const float t = p.tau[sc * p.n_beh + bh];
                if (!(t > 0.f) || !(t < INFINITY)) bad |= CLIMBER_BAD_TAU;
            }
        }
        if (p.cand_off) {
            for (int64_t b = i0; b < p.B; b += stride) {
                const int lo = p.cand_off[b], hi = p.cand_off[b + 1];
                if (hi < lo || (b == 0 && lo != 0) || (b == p.B - 1 && hi != p.n_rows)) bad |= CLIMBER_BAD_OFFSETS;
                if (hi - lo > p.m_max) bad |= CLIMBER_BAD_M_MAX;
            }
        }
    }
    if (bad) atomicOr(p.status, bad);
}

}  // namespace

hipError_t launch_check_inputs(const float *tau, const int32_t *scen, const int32_t *beh, int64_t n_rows,
                               const int32_t *hist_len, const int32_t *tok_off, const int32_t *cand_off,
                               int B, int n_scen, int n_beh, int m_max, int32_t *status, hipStream_t s)
{
    CheckParams p{tau, scen, beh, cand_off, hist_len, tok_off, status, n_rows, B, n_scen, n_beh, m_max};
    const int64_t blocks = std::min<int64_t>(std::max<int64_t>((n_rows + 255) / 256, 1), 1024);
    hipLaunchKernelGGL(check_inputs_kernel, dim3((unsigned)blocks), dim3(256), 0, s, p);
    return hipGetLastError();
}

}  // namespace climber
