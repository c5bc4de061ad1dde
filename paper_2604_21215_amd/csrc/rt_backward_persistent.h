// Interface of the single-launch reverse loop of the backward pass (rt_backward_persistent.hip), paper Sec. 6.4.
#pragma once
#include "rt_common.h"

namespace rt {

struct BwpState {
    bool available = false;
    int grid = 0, H = 0;
    size_t lds_bytes = 0;
    long long spin_limit = 0;
    unsigned nonce = 0;   // per-launch tag prefix of the exchange words
};

// Device tensors of one backward call as the reverse loop sees them (fp32 rows are position-first: row n B + b).
struct BwpTensors {
    const bf16_t *WkvT, *W2T, *W1T, *WoT;   // transposed weights [d][2d], [F][d], [d][F], [d][d]
    const bf16_t *g_kv, *g_mlp, *g_k;       // gains or null
    const bf16_t *gy;                       // [B][N][d]
    const float *unit_k, *rk;               // [M][2d] (first d columns: normalised raw keys), [M][H]
    const float *unit_z, *rinv_z, *unit_h, *rinv_h;
    const float *gp;                        // [M][F] gelu'(pre)
    const float *A_gy, *A_uz;               // [M][F] W2^T gy, W2^T unit_z
    const float *C_gy, *C_uz, *C_uh;        // [M][d] Wo^T gy, Wo^T unit_z, Wo^T unit_h
    const float *Qn, *Ktn, *Vt, *Kp, *Vp, *c, *lse;
    float *dK, *dV, *dkraw, *d_rz, *Gz, *dpre, *t1, *d_h, *dc, *Ds, *dq, *dkt, *dvt;
};

size_t bwp_exchange_bytes(int d, int F);
bool bwp_create(BwpState &P, int device, int d, int F, int H, int max_batch, bool bf16_mfma);
bool bwp_supported(const BwpState &P, const LayerDims &D);
// zero the exchange words (once after allocation)
hipError_t bwp_clear(void *exchange, size_t bytes, hipStream_t st);
// positions i_hi down to i_lo, all inside one block of 32 positions [i_lo, i_lo + 31]
hipError_t bwp_run_block(BwpState &P, const LayerDims &D, const BwpTensors &T, void *exchange, int i_hi, int i_lo, hipStream_t st);

}  // namespace rt
