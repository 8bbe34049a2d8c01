// Host side of bs_spmv: picks the launch shape from the matrix shape.
#include "bs_spmv_kernel.h"

namespace bs {

namespace {

constexpr int kCus = 256;   // compute units of the MI355X

struct LstmPart {
    const float* h_in;
    const float* bias;
    const float* c_in;
    float* c_out;
    float* h_out;
    int H, I;
};

// The launch shape for one product.  lstm: the fused step (M = 4H, K = I + H).
struct SpmvPlan {
    bool slab;              // x does not fit LDS: bs_spmv_slab.hip, nothing else below is set
    int ch, lpr, u, rpw, threads;
    int64_t grid;
    size_t lds;
    int table_off, bank_mode, pre_off;
    int64_t row_len, cpr;
};


// isize: bytes per stored offset (1, or 2 for the kernels of bs_spmv_wide.hip, which exist for
// the widest chunk or single entries, 8..64 lanes per row and 2, 4 or 8 chunk slots)
int plan_spmv(int dtype, int64_t M, int64_t K, int bank, int k, int lanes_per_row, int rows_per_wg,
              bool lstm, int isize, SpmvPlan& p) {
    p = SpmvPlan{};
    const bool wide = isize == 2;
    const int64_t row_len = (K / bank) * k;
    // LDS: x, then (if it fits) one word per row entry for the bank table
    const size_t x_floats = ((size_t)K + 3) / 4 * 4;
    size_t lds = x_floats * sizeof(float);
    if (M > INT32_MAX) return BS_ERR_UNSUPPORTED;
    if (lds > (size_t)kMaxLdsBytes) {
        // x does not fit one compute unit's LDS: the slab-by-slab kernel (no launch-shape
        // overrides, no fused LSTM step there)
        if (lstm || wide || lanes_per_row != 0 || rows_per_wg != 0) return BS_ERR_UNSUPPORTED;
        p.slab = true;
        return BS_OK;
    }
    int table_off = 0;
    if (lds + (size_t)row_len * 4 <= (size_t)kMaxLdsBytes) {
        table_off = (int)x_floats;
        lds += (size_t)row_len * 4;
    }
    const int vsize = dtype == BS_F16 ? 2 : 4;

    // widest chunk that divides the row, so chunks never straddle rows and stay aligned
    int ch = 16 / vsize;
    while (ch > 1 && row_len % ch != 0) ch >>= 1;
    if (wide && ch != 16 / vsize) ch = 1;
    const int64_t cpr = row_len / ch;

    constexpr int kMaxInFlight = 8;
    int lpr = lanes_per_row;
    if (lpr == 0) {
        // smallest group that leaves at most 4 chunks per lane (measured best on both
        // the 9 MB and the 84 MB matrices: a short dependent chain per lane, still
        // 80 bytes in flight per lane); rows longer than 256 chunks use all 64 lanes
        lpr = lstm || wide ? 8 : 1;   // the fused step is built for 8..64 lanes per row
        while (lpr < 64 && (cpr + lpr - 1) / lpr > 4) lpr <<= 1;
        // a small matrix: wider groups (down to one chunk per lane) until there are 512
        // lanes for every compute unit (measured: 4096 x 4096 with 2 of 64 kept 3.29 -> 2.82 us,
        // the 1024-unit LSTM matrix 3.41 -> 3.17 us)
        while (lpr < 64 && (cpr + lpr - 1) / lpr > 1 && M * lpr < (int64_t)kCus * 512) lpr <<= 1;
    }
    if (lpr < 1 || lpr > 64 || (lpr & (lpr - 1)) || (wide && lpr < 8)) return BS_ERR_UNSUPPORTED;
    // chunk slots per lane and round: as many as the row needs, 2..8 (a slot that is empty for
    // every lane still costs its two loads: 0.06 of 3.98 us on the 6000 x 3000 matrix, which
    // needs 3; 1-3 % on the shapes that need 5)
    int64_t need = (cpr + lpr - 1) / lpr;
    int u = need >= kMaxInFlight ? kMaxInFlight : (int)need;
    if (u < 2) u = 2;
    if (lstm) u = u <= 4 ? 4 : 8;
    if (wide) u = u <= 2 ? 2 : u <= 4 ? 4 : 8;

    int rpw = rows_per_wg;
    if (rpw == 0) {
        // Workgroup size by a byte count for the busiest compute unit: it runs
        // ceil(workgroups / 256) workgroups, each streaming its rows and copying x (from L2:
        // counted half).  Fewer, larger workgroups copy x less often; a count that does not
        // fill the last round of compute units evenly doubles the tail; the largest
        // workgroups carry a handicap (their wavefronts start and retire together: measured
        // 3-10 % slower than 512 lanes at equal byte counts).  Over the ten shapes of the
        // launch-shape sweep this picks the best shape or one within 2 % of it (256 lanes
        // always: 2-14 % slower).
        const double row_bytes = (double)row_len * (vsize + isize), x_cost = 0.5 * (double)lds;
        double best = 0;
        int best_thr = 0;
        for (int thr : {256, 384, 512, 768, 1024}) {
            if (thr % lpr) continue;
            const int r = thr / lpr;
            if (lstm && r % 4) continue;
            const int64_t g = (M + r - 1) / r;
            const double handicap = thr == 1024 ? 1.2 : thr == 768 ? 1.05 : 1.0;
            const double cost = handicap * (double)((g + kCus - 1) / kCus) * (r * row_bytes + x_cost);
            if (best_thr == 0 || cost < best) { best = cost; best_thr = thr; }
        }
        if (best_thr == 0) return BS_ERR_UNSUPPORTED;
        rpw = best_thr / lpr;
    }
    const int64_t threads = (int64_t)lpr * rpw;
    if (rpw < 1 || threads > 1024 || threads % kWave) return BS_ERR_UNSUPPORTED;
    if (lstm && rpw % 4) return BS_ERR_UNSUPPORTED;   // whole units per workgroup
    int pre_off = 0;
    if (lstm) {   // the workgroup's pre-activations, behind x and the table
        pre_off = (int)(lds / sizeof(float));
        lds += (size_t)rpw * sizeof(float);
        if (lds > (size_t)kMaxLdsBytes) return BS_ERR_UNSUPPORTED;
    }
    const int64_t grid = (M + rpw - 1) / rpw;
    if (grid > INT32_MAX) return BS_ERR_UNSUPPORTED;
    p.ch = ch; p.lpr = lpr; p.u = u; p.rpw = rpw; p.threads = (int)threads; p.grid = grid;
    p.lds = lds; p.table_off = table_off; p.pre_off = pre_off;
    p.bank_mode = (k % ch == 0) ? 0 : (k >= ch ? 1 : 2);
    p.row_len = row_len; p.cpr = cpr;
    return BS_OK;
}

// Shared by bs_spmv and the fused LSTM step (lstm != nullptr: M = 4H, K = I + H,
// x is the first I entries of the input vector, y is unused).
int launch_common(const void* vals, const void* idx, int isize, int dtype, int64_t M, int64_t K, int bank,
                  int k, const float* x, float* y, int lanes_per_row, int rows_per_wg,
                  const LstmPart* lstm, hipEvent_t ev_start, hipEvent_t ev_stop, hipStream_t st) {
    SpmvPlan p;
    const int rc = plan_spmv(dtype, M, K, bank, k, lanes_per_row, rows_per_wg, lstm != nullptr, isize, p);
    if (rc != BS_OK) return rc;
    if (p.slab)
        return launch_spmv_slabbed(vals, static_cast<const uint8_t*>(idx), dtype, M, K, bank, k, x, y,
                                   ev_start, ev_stop, st);

    SpmvArgs a;
    a.vals = vals; a.idx = idx; a.x = x; a.y = y;
    a.M = (int)M; a.K = (int)K; a.B = bank; a.k = k;
    a.magic_k = magic_u32((uint32_t)k);
    a.row_len = (int)p.row_len;
    a.chunks_per_row = (int)p.cpr;
    a.rows_per_wg = p.rpw;
    a.bank_mode = p.bank_mode;
    a.table_off = p.table_off;
    a.h_in = nullptr; a.bias = nullptr; a.c_in = nullptr; a.c_out = nullptr; a.h_out = nullptr;
    a.H = 0; a.I = 0; a.pre_off = p.pre_off;
    if (lstm) {
        a.h_in = lstm->h_in; a.bias = lstm->bias; a.c_in = lstm->c_in;
        a.c_out = lstm->c_out; a.h_out = lstm->h_out; a.H = lstm->H; a.I = lstm->I;
    }

    const SpmvLaunch l{lstm != nullptr, p.threads, (int)p.grid, p.lds, ev_start, ev_stop, st};
    if (isize == 2) return spmv_launch_wide(dtype, p.ch, p.lpr, p.u, a, l);
    if (dtype == BS_F16) return spmv_launch_f16(p.ch, p.lpr, p.u, a, l);
    return spmv_launch_f32(p.ch, p.lpr, p.u, a, l);
}

}  // namespace

int launch_spmv(const void* vals, const uint8_t* idx, int dtype, int64_t M, int64_t K, int bank,
                int k, const float* x, float* y, int lanes_per_row, int rows_per_wg,
                hipEvent_t ev_start, hipEvent_t ev_stop, hipStream_t st) {
    return launch_common(vals, idx, 1, dtype, M, K, bank, k, x, y, lanes_per_row, rows_per_wg,
                         nullptr, ev_start, ev_stop, st);
}

int launch_spmv_wide(const void* vals, const uint16_t* idx, int dtype, int64_t M, int64_t K, int bank,
                     int k, const float* x, float* y, hipStream_t st) {
    return launch_common(vals, idx, 2, dtype, M, K, bank, k, x, y, 0, 0, nullptr, nullptr, nullptr, st);
}

int spmv_plan_describe(int dtype, int64_t M, int64_t K, int bank, int k, int lanes_per_row,
                       int rows_per_wg, int64_t* out, int n_out) {
    SpmvPlan p;
    const int rc = plan_spmv(dtype, M, K, bank, k, lanes_per_row, rows_per_wg, false, 1, p);
    if (rc != BS_OK) return rc;
    const int64_t v[10] = {p.slab ? 1 : 0, p.ch, p.lpr, p.u, p.threads, p.rpw, p.grid, (int64_t)p.lds,
                           p.table_off > 0 ? 1 : 0, p.bank_mode};
    for (int i = 0; i < n_out && i < 10; ++i) out[i] = v[i];
    return BS_OK;
}

int launch_lstm_step(const void* vals, const uint8_t* idx, int dtype, int64_t H, int64_t I, int bank,
                     int k, const float* x, const float* h_in, const float* bias,
                     const float* c_in, float* c_out, float* h_out, hipStream_t st) {
    if (H % 4 || I % 4 || 4 * H > INT32_MAX) return BS_ERR_UNSUPPORTED;
    const LstmPart part{h_in, bias, c_in, c_out, h_out, (int)H, (int)I};
    return launch_common(vals, idx, 1, dtype, 4 * H, I + H, bank, k, x, nullptr, 0, 0, &part, nullptr,
                         nullptr, st);
}

}  // namespace bs
