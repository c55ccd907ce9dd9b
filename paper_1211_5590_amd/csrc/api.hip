// C ABI of the Elman-RNN training path: argument checks, workspace carving, kernel dispatch.
// Every call only enqueues kernels on the caller's stream (the paper's section on
// asynchronous GPU calls) into caller-owned buffers (its garbage-collection-free linker),
// and does O(1) host work whatever the sequence length (its trusted-input switch).
#include "../../include/rnn.h"

#include <atomic>

#include "internal.hpp"
#include "prof.hpp"

namespace {

using namespace rnn;

std::atomic<int> g_wait_limit{1 << 22};

constexpr size_t kAlign = 256;
inline size_t up(size_t v) { return (v + kAlign - 1) / kAlign * kAlign; }

struct Plan {
    // byte offsets into the workspace
    size_t Z, lse, rowloss, U, G, Delta, WhT, hring, part, splitk, scratch, flags, statbox, gbox, gpart, vy, seen,
        lstat, HsS, HsT, VS, VT, dZS, dZT, DT, XS, WxS, splitk3, total;
};

// Which kernel family serves these sizes.
struct Variant {
    bool resident;        // resident-weight persistent loops (else shape-agnostic loops)
    bool skinny;          // column-strip output layer + fused tail of the reverse loop
    bool stepwise;        // batched recurrence as one fused MFMA launch per step
    bool batch_mfma;      // batched persistent loop, weights in registers (H <= 256)
    RecResPlan fwd, bwd;  // plans of the two loops when resident
    bool grid;            // several workgroups per sequence, role-split form (recurrence_grid.hip)
    RecGridPlan gplan;
};

struct Sizes {
    int NVin, H, O, T, B;
    long long N;
    bool tokens, ce;
};

bool dims_valid(const rnn_dims* d) {
    if (!d) return false;
    if (d->in_dim <= 0 || d->hidden <= 0 || d->out_dim <= 0 || d->seq_len <= 0 || d->batch <= 0)
        return false;
    if (d->input_kind != RNN_INPUT_TOKENS && d->input_kind != RNN_INPUT_DENSE) return false;
    if (d->act != RNN_ACT_SIGMOID && d->act != RNN_ACT_TANH) return false;
    if (d->loss_kind != RNN_LOSS_SOFTMAX_CE && d->loss_kind != RNN_LOSS_LINEAR_MSE) return false;
    if (d->flags & ~(RNN_FLAG_ACCUMULATE | RNN_FLAG_SYNC | RNN_FLAG_BPTT_RECOMPUTE |
                     RNN_FLAG_REFERENCE_KERNELS | RNN_FLAG_BF16X3_OUTPUT))   // RNN_FLAG_COOPERATIVE: rnn_window only
        return false;
    const long long N = (long long)d->seq_len * d->batch;
    // keep every row index and every N*width product the kernels form inside int32 / size_t
    if (N > (1LL << 30)) return false;
    if (N * (long long)d->out_dim > (1LL << 40) || N * (long long)d->hidden > (1LL << 40))
        return false;
    return true;
}

Sizes sizes_of(const rnn_dims* d) {
    Sizes s;
    s.NVin = d->in_dim; s.H = d->hidden; s.O = d->out_dim; s.T = d->seq_len; s.B = d->batch;
    s.N = (long long)d->seq_len * d->batch;
    s.tokens = d->input_kind == RNN_INPUT_TOKENS;
    s.ce = d->loss_kind == RNN_LOSS_SOFTMAX_CE;
    return s;
}

size_t max_splitk_floats(const Sizes& s) {
    const int N = (int)s.N, H = s.H, O = s.O, D = s.NVin;
    size_t m = 0;
    auto take = [&](size_t v) { if (v > m) m = v; };
    take(gemm_splitk_floats(N, O, H));   // Z = Hs V
    take(gemm_splitk_floats(H, O, N));   // dV = Hs^T dZ
    take(gemm_splitk_floats(N, H, O));   // G = dZ V^T
    take(gemm_splitk_floats(H, H, N));   // dWh = Delta^T Hprev
    take(gemm_splitk_floats(s.B, H, H)); // dh0 = delta_0 Wh (stepwise recurrence)
    if (!s.tokens) {
        take(gemm_splitk_floats(N, H, D));  // U = X Wx^T
        take(gemm_splitk_floats(H, D, N));  // dWx = Delta^T X
    }
    return m;
}

Variant pick_variant(const rnn_dims* d) {
    const Sizes s = sizes_of(d);
    Variant v{};
    if (d->flags & RNN_FLAG_REFERENCE_KERNELS) return v;
    v.resident = rec_resident_plan(s.H, s.B, s.T, false, false, 0, &v.fwd) &&
                 rec_resident_plan(s.H, s.B, s.T, true, false, 0, &v.bwd);
    if (!v.resident) {
        v.batch_mfma = rec_batch_mfma_supported(s.H, s.B);
        v.stepwise = !v.batch_mfma && s.B > 4;
        return v;
    }
    v.grid = (v.fwd.P > 1 || v.bwd.P > 1) && rec_grid_plan(s.H, s.B, &v.gplan);
    RecResPlan fused;
    if (s.tokens && s.ce && s.B == 1 && skinny_supported((int)s.N, s.H, s.O) &&
        rec_resident_plan(s.H, s.B, s.T, true, true, skinny_strips(s.O), &fused)) {
        v.skinny = true;
        v.bwd = fused;
    }
    return v;
}

Plan make_plan(const rnn_dims* d) {
    const Sizes s = sizes_of(d);
    const size_t N = (size_t)s.N, H = (size_t)s.H, O = (size_t)s.O, B = (size_t)s.B;
    Plan p;
    size_t off = 0;
    auto take = [&](size_t bytes) { const size_t o = off; off += up(bytes); return o; };
    p.Z = take(N * O * 4);
    p.lse = take(N * 4);
    p.rowloss = take(N * 4);
    p.U = take((!s.tokens || s.B > 4) ? N * H * 4 : 0);  // hoisted input term (dense, or batched tokens)
    p.G = take(N * H * 4);
    p.Delta = take(N * H * 4);
    p.WhT = take(H * H * 4);
    p.hring = take(2 * B * H * 4);
    const size_t widest = O > H ? O : H;
    p.part = take((size_t)colsum_chunks((int)N) * widest * 4);
    p.splitk = take(max_splitk_floats(s) * 4);
    p.scratch = take(256);
    p.flags = take(4096 + 16 * B * H);   // state-exchange boxes of the multi-workgroup loops
    const size_t strips = (size_t)skinny_strips(s.O);
    const bool small = N <= 32;
    p.statbox = take(small ? skinny_stat_box_bytes((int)N, s.O) : 0);
    p.gbox = take(small ? N * H * 8 : 0);
    p.gpart = take(small ? strips * N * H * 4 : 0);
    p.vy = take(small ? N * H * 4 : 0);
    p.seen = take(s.tokens && N > 32 ? dwx_table_ints((int)N, s.NVin) * 4 : 0);
    // row statistics the logits product leaves per 64-column part (fused log-sum-exp)
    const bool bf3 = (d->flags & RNN_FLAG_BF16X3_OUTPUT) != 0;
    const bool fuses = bf3 ? bf3_fuses_stats((int)N, s.O, s.H) : gemm_fuses_stats((int)N, s.O, s.H);
    const size_t parts = bf3 ? (size_t)bf3_stat_parts((int)N, s.O, s.H) : (size_t)gemm_stat_parts(s.O);
    p.lstat = take(s.ce && fuses ? N * parts * 8 : 0);
    // bf16 hi/lo plane pairs of the output layer's operands (4 bytes per padded element)
    const size_t Np = (size_t)bf3_pad((int)N), Hp = (size_t)bf3_pad(s.H), Op = (size_t)bf3_pad(s.O);
    p.HsS = take(bf3 ? N * Hp * 4 : 0);
    p.HsT = take(bf3 ? H * Np * 4 : 0);
    p.VS = take(bf3 ? H * Op * 4 : 0);
    p.VT = take(bf3 ? O * Hp * 4 : 0);
    p.dZS = take(bf3 ? N * Op * 4 : 0);
    p.dZT = take(bf3 ? O * Np * 4 : 0);
    p.DT = take(bf3 ? H * Np * 4 : 0);
    // dense input: X transposed, for dWx (the input projection itself stays float32: the hidden
    // states it feeds are held to a tighter tolerance than the gradients)
    p.XS = take(bf3 && !s.tokens ? (size_t)s.NVin * Np * 4 : 0);
    p.WxS = take(0);
    size_t sk3 = 0;
    if (bf3) {
        sk3 = bf3_splitk_floats((int)N, s.O, s.H);
        if (bf3_splitk_floats(s.H, s.O, (int)N) > sk3) sk3 = bf3_splitk_floats(s.H, s.O, (int)N);
        if (bf3_splitk_floats((int)N, s.H, s.O) > sk3) sk3 = bf3_splitk_floats((int)N, s.H, s.O);
        if (bf3_splitk_floats(s.H, s.H, (int)N) > sk3) sk3 = bf3_splitk_floats(s.H, s.H, (int)N);
        if (!s.tokens && bf3_splitk_floats(s.H, s.NVin, (int)N) > sk3) sk3 = bf3_splitk_floats(s.H, s.NVin, (int)N);
    }
    p.splitk3 = take(sk3 * 4);
    p.total = off;
    return p;
}

int check_ws(const rnn_dims* d, void* ws, size_t ws_bytes, Plan* plan) {
    *plan = make_plan(d);
    if (!ws || (reinterpret_cast<uintptr_t>(ws) & 15u) || ws_bytes < plan->total)
        return RNN_EWORKSPACE;
    return RNN_OK;
}

template <typename T>
T* at(void* ws, size_t off) { return reinterpret_cast<T*>(static_cast<char*>(ws) + off); }

bool misaligned(const void* p) { return p && (reinterpret_cast<uintptr_t>(p) & 15u); }
// ids, targets and the loss scalar are only ever accessed as 4-byte words (windows of a stream
// start at arbitrary element offsets)
bool misaligned4(const void* p) { return p && (reinterpret_cast<uintptr_t>(p) & 3u); }

int finish(const rnn_dims* d, hipStream_t s, hipError_t e) {
    if (e != hipSuccess) return RNN_EHIP;
    if (d->flags & RNN_FLAG_SYNC)
        if (hipStreamSynchronize(s) != hipSuccess) return RNN_EHIP;
    return RNN_OK;
}

#define RNN_TRY(expr)                      \
    do {                                   \
        hipError_t e_ = (expr);            \
        if (e_ != hipSuccess) return e_;   \
    } while (0)

// ---- stages ------------------------------------------------------------------------------

hipError_t run_forward(const rnn_dims* d, const rnn_params* P, const void* x, const float* h0,
                       float* h_all, float* h_last, void* ws, const Plan& pl, hipStream_t s) {
    const Sizes z = sizes_of(d);
    RecFwdArgs a{};
    a.Wh = P->Wh; a.Wx = P->Wx; a.b = P->b;
    a.h0 = h0; a.h_last = h_last;
    a.H = z.H; a.T = z.T; a.B = z.B; a.act = d->act;
    a.ring = h_all ? 0 : 1;
    a.hist = h_all ? h_all : at<float>(ws, pl.hring);
    if (z.tokens) {
        a.x = static_cast<const int32_t*>(x);
        a.U = nullptr;
    } else {
        // input term for every step at once: U = X Wx^T + b
        GemmArgs g{};
        g.A = static_cast<const float*>(x); g.B = P->Wx; g.C = at<float>(ws, pl.U);
        g.M = (int)z.N; g.N = z.H; g.K = z.NVin;
        g.lda = z.NVin; g.ldb = z.NVin; g.ldc = z.H;
        g.a_t = false; g.b_t = true; g.bias_n = P->b; g.beta = 0; g.prof_id = K_GEMM_U;
        g.splitk_ws = at<float>(ws, pl.splitk);
        RNN_TRY(launch_gemm(g, s));
        a.x = nullptr;
        a.U = at<float>(ws, pl.U);
    }
    const Variant v = pick_variant(d);
    if (v.resident) {
        RecResArgs r{};
        r.Wh = P->Wh; r.H = z.H; r.T = z.T; r.B = z.B; r.act = d->act;
        r.flags = at<int32_t>(ws, pl.flags); r.status = at<int32_t>(ws, pl.scratch) + 1;
        r.Wx = P->Wx; r.b = P->b; r.x = a.x; r.U = a.U; r.h0 = h0;
        r.hist = a.hist; r.h_last = h_last; r.ring = a.ring;
        if (v.grid) return launch_rec_grid(r, v.gplan, false, s);
        return launch_rec_resident(r, v.fwd, false, s);
    }
    if (v.batch_mfma) {
        float* U = at<float>(ws, pl.U);
        if (z.tokens) RNN_TRY(launch_gather_input(a.x, P->Wx, P->b, U, (int)z.N, z.H, s));
        RecMfmaArgs m{};
        m.Wh = P->Wh; m.H = z.H; m.T = z.T; m.B = z.B; m.act = d->act;
        m.U = U; m.h0 = h0; m.hist = a.hist; m.h_last = h_last; m.ring = a.ring;
        return launch_rec_batch_mfma(m, false, s);
    }
    if (v.stepwise && h_all && rec_xcd_supported(z.H, z.B, z.T) && rec_xcd_ready(z.H, d->act, false)) {
        // one persistent launch for all steps (one batch group per XCD)
        float* U = at<float>(ws, pl.U);
        if (z.tokens) RNN_TRY(launch_gather_input(a.x, P->Wx, P->b, U, (int)z.N, z.H, s));
        RecXcdArgs m{};
        m.Wh = P->Wh; m.H = z.H; m.T = z.T; m.B = z.B; m.act = d->act;
        m.U = U; m.h0 = h0; m.hist = h_all; m.h_last = h_last;
        m.counters = at<int32_t>(ws, pl.flags); m.status = at<int32_t>(ws, pl.scratch) + 1;
        return launch_rec_xcd(m, false, s);
    }
    if (v.stepwise) return run_rec_fwd_stepwise(a, s);
    return launch_rec_fwd_reference(a, s);
}

SkinnyArgs skinny_args(const rnn_dims* d, const rnn_params* P, const float* h_all, const void* targets,
                       void* ws, const Plan& pl) {
    const Sizes z = sizes_of(d);
    SkinnyArgs k{};
    k.Hs = h_all + (size_t)z.B * z.H; k.V = P->V; k.c = P->c;
    k.y = static_cast<const int32_t*>(targets);
    k.Z = at<float>(ws, pl.Z); k.stat_box = at<unsigned long long>(ws, pl.statbox);
    k.status = at<int32_t>(ws, pl.scratch) + 1;
    k.epoch_word = at<uint32_t>(ws, pl.scratch) + 2;   // the launches' tags are device state
    k.spin_limit = wait_limit();
    k.lse = at<float>(ws, pl.lse); k.gpart = at<float>(ws, pl.gpart); k.vy = at<float>(ws, pl.vy);
    k.H = z.H; k.O = z.O; k.N = (int)z.N; k.NV = z.NVin;
    return k;
}

hipError_t run_loss(const rnn_dims* d, const rnn_params* P, const float* h_all, const void* targets,
                    float* loss, void* ws, const Plan& pl, hipStream_t s) {
    const Sizes z = sizes_of(d);
    const int N = (int)z.N;
    if (pick_variant(d).skinny) {
        SkinnyArgs k = skinny_args(d, P, h_all, targets, ws, pl);
        k.loss = loss;
        return launch_skinny_logits(k, s);
    }
    float* Z = at<float>(ws, pl.Z);
    if (d->flags & RNN_FLAG_BF16X3_OUTPUT) {
        // operands as bf16 hi/lo planes (h also transposed, for dV later; V both ways), then the
        // product on the bf16 matrix cores
        const float* Hs = h_all + (size_t)z.B * z.H;
        RNN_TRY(launch_split_bf16(Hs, N, z.H, z.H, at<uint16_t>(ws, pl.HsS), at<uint16_t>(ws, pl.HsT), s));
        RNN_TRY(launch_split_bf16(P->V, z.H, z.O, z.O, at<uint16_t>(ws, pl.VS), at<uint16_t>(ws, pl.VT), s));
        const bool fused = z.ce && bf3_fuses_stats(N, z.O, z.H);
        Bf3Args b{};
        b.A = at<uint16_t>(ws, pl.HsS); b.B = at<uint16_t>(ws, pl.VT); b.C = Z;
        b.M = N; b.N = z.O; b.K = z.H; b.lda = bf3_pad(z.H); b.ldb = bf3_pad(z.H); b.ldc = z.O;
        b.bias_n = P->c; b.beta = 0; b.splitk_ws = at<float>(ws, pl.splitk3); b.prof_id = K_GEMM_LOGITS;
        b.row_stats = fused ? at<float>(ws, pl.lstat) : nullptr;
        RNN_TRY(launch_gemm_bf16x3(b, s));
        float* rowloss = at<float>(ws, pl.rowloss);
        if (fused) {
            RNN_TRY(launch_ce_merge_stats(b.row_stats, bf3_stat_parts(N, z.O, z.H), Z, static_cast<const int32_t*>(targets),
                                          at<float>(ws, pl.lse), rowloss, N, z.O, s));
            return launch_loss_reduce(rowloss, N, 1.0f / (float)N, loss, s);
        }
        if (z.ce) {
            RNN_TRY(launch_ce_row_stats(Z, static_cast<const int32_t*>(targets), at<float>(ws, pl.lse),
                                        rowloss, N, z.O, s));
            return launch_loss_reduce(rowloss, N, 1.0f / (float)N, loss, s);
        }
        int n_partial = 0;
        RNN_TRY(launch_mse_partial(Z, static_cast<const float*>(targets), rowloss, N, z.O, &n_partial, s));
        return launch_loss_reduce(rowloss, n_partial, (float)(1.0 / ((double)N * (double)z.O)), loss, s);
    }
    GemmArgs g{};
    g.A = h_all + (size_t)z.B * z.H;  // rows of h_all[1:]
    g.B = P->V; g.C = Z;
    g.M = N; g.N = z.O; g.K = z.H;
    g.lda = z.H; g.ldb = z.O; g.ldc = z.O;
    g.a_t = false; g.b_t = false; g.bias_n = P->c; g.beta = 0; g.prof_id = K_GEMM_LOGITS;
    g.splitk_ws = at<float>(ws, pl.splitk);
    // softmax-CE: the product's epilogue leaves (max, sum exp) per row and 64-column part, so the
    // logits are not read again for the log-sum-exp
    const bool fused = z.ce && gemm_fuses_stats(N, z.O, z.H);
    g.row_stats = fused ? at<float>(ws, pl.lstat) : nullptr;
    RNN_TRY(launch_gemm(g, s));
    float* rowloss = at<float>(ws, pl.rowloss);
    if (fused) {
        RNN_TRY(launch_ce_merge_stats(g.row_stats, gemm_stat_parts(z.O), Z, static_cast<const int32_t*>(targets),
                                      at<float>(ws, pl.lse), rowloss, N, z.O, s));
        return launch_loss_reduce(rowloss, N, 1.0f / (float)N, loss, s);
    }
    if (z.ce) {
        RNN_TRY(launch_ce_row_stats(Z, static_cast<const int32_t*>(targets), at<float>(ws, pl.lse),
                                    rowloss, N, z.O, s));
        return launch_loss_reduce(rowloss, N, 1.0f / (float)N, loss, s);
    }
    int n_partial = 0;
    RNN_TRY(launch_mse_partial(Z, static_cast<const float*>(targets), rowloss, N, z.O, &n_partial, s));
    return launch_loss_reduce(rowloss, n_partial, (float)(1.0 / ((double)N * (double)z.O)), loss, s);
}

// Reverse-time loop delta_t = (G_t + Wh^T delta_{t+1}) * act'(h_t) with the kernel family that
// serves these sizes (never the fused short-sequence form).  Wh and its transposed copy are
// passed explicitly: the R-operator's forward sweep is the same recurrence run on time-reversed
// rows with the two exchanged.
hipError_t run_reverse_loop(const rnn_dims* d, const float* Wh, const float* WhT_or_null, float* WhT_ws,
                            const float* G, const float* h_all, const float* dh_last, float* Delta,
                            float* dh0, void* ws, const Plan& pl, hipStream_t s) {
    const Sizes z = sizes_of(d);
    const int H = z.H;
    Variant v = pick_variant(d);
    if (v.skinny) {   // the plain plan of the resident loop
        if (!rec_resident_plan(z.H, z.B, z.T, true, false, 0, &v.bwd)) v.resident = false;
    }
    if (v.resident) {
        RecResArgs r{};
        r.Wh = Wh; r.H = H; r.T = z.T; r.B = z.B; r.act = d->act;
        r.flags = at<int32_t>(ws, pl.flags); r.status = at<int32_t>(ws, pl.scratch) + 1;
        r.G = G; r.h_all = h_all; r.dh_last = dh_last; r.Delta = Delta; r.dh0 = dh0;
        if (v.grid) return launch_rec_grid(r, v.gplan, true, s);
        return launch_rec_resident(r, v.bwd, true, s);
    }
    if (v.batch_mfma) {
        RecMfmaArgs m{};
        m.Wh = Wh; m.H = H; m.T = z.T; m.B = z.B; m.act = d->act;
        m.G = G; m.h_all = h_all; m.dh_last = dh_last; m.Delta = Delta; m.dh0 = dh0;
        return launch_rec_batch_mfma(m, true, s);
    }
    if (v.stepwise && rec_xcd_supported(z.H, z.B, z.T) && rec_xcd_ready(z.H, d->act, true)) {
        RecXcdArgs m{};
        m.Wh = Wh; m.H = H; m.T = z.T; m.B = z.B; m.act = d->act;
        m.G = G; m.h_all = h_all; m.dh_last = dh_last; m.Delta = Delta; m.dh0 = dh0;
        m.counters = at<int32_t>(ws, pl.flags); m.status = at<int32_t>(ws, pl.scratch) + 1;
        return launch_rec_xcd(m, true, s);
    }
    // the remaining families read the matrix transposed: one copy per call
    const float* WhT = WhT_or_null;
    if (!WhT) {
        RNN_TRY(launch_transpose(Wh, WhT_ws, H, H, s));
        WhT = WhT_ws;
    }
    if (v.stepwise) {
        RecBwdArgs a{};
        a.Wh = Wh; a.WhT = WhT; a.G = G; a.h_all = h_all; a.dh_last = dh_last;
        a.Delta = Delta; a.dh0 = dh0; a.splitk_ws = at<float>(ws, pl.splitk);
        a.H = H; a.T = z.T; a.B = z.B; a.act = d->act;
        return run_rec_bwd_stepwise(a, s);
    }
    RecBwdArgs a{};
    a.Wh = Wh; a.WhT = WhT; a.G = G; a.h_all = h_all; a.dh_last = dh_last;
    a.Delta = Delta; a.dh0 = dh0;
    a.H = H; a.T = z.T; a.B = z.B; a.act = d->act;
    return launch_rec_bwd_reference(a, s);
}

// Everything of backpropagation that follows d loss / d z (held in the logits buffer of the
// workspace): dV, G, the reverse loop, dWh, db, dWx.  dc is the caller's.
// bf3: dZ is also there as bf16 plane pairs (row-major and transposed) next to the planes of h and
// V that run_loss left, and dV, G run on the bf16 matrix cores.
hipError_t run_backward_from_dz(const rnn_dims* d, const rnn_params* P, const void* x, const float* h_all,
                                const float* dh_last, const rnn_grads* Gr, float* dh0, void* ws,
                                const Plan& pl, bool bf3, hipStream_t s) {
    const Sizes z = sizes_of(d);
    const int N = (int)z.N, H = z.H, O = z.O;
    const int beta = (d->flags & RNN_FLAG_ACCUMULATE) ? 1 : 0;
    float* Z = at<float>(ws, pl.Z);
    float* part = at<float>(ws, pl.part);
    float* splitk = at<float>(ws, pl.splitk);
    float* G = at<float>(ws, pl.G);
    float* Delta = at<float>(ws, pl.Delta);
    const float* Hs = h_all + (size_t)z.B * H;  // h_t rows
    const int chunks = colsum_chunks(N);
    if (bf3) {
        const int Np = bf3_pad(N), Op = bf3_pad(O);
        Bf3Args b{};   // dV = Hs^T dZ, K = N
        b.A = at<uint16_t>(ws, pl.HsT); b.B = at<uint16_t>(ws, pl.dZT); b.C = Gr->dV;
        b.M = H; b.N = O; b.K = N; b.lda = Np; b.ldb = Np; b.ldc = O;
        b.beta = beta; b.splitk_ws = at<float>(ws, pl.splitk3); b.prof_id = K_GEMM_DV;
        RNN_TRY(launch_gemm_bf16x3(b, s));
        Bf3Args c{};   // G = dZ V^T, K = O
        c.A = at<uint16_t>(ws, pl.dZS); c.B = at<uint16_t>(ws, pl.VS); c.C = G;
        c.M = N; c.N = H; c.K = O; c.lda = Op; c.ldb = Op; c.ldc = H;
        c.beta = 0; c.splitk_ws = at<float>(ws, pl.splitk3); c.prof_id = K_GEMM_G;
        RNN_TRY(launch_gemm_bf16x3(c, s));
    } else {
    // dV = Hs^T dZ
    {
        GemmArgs g{};
        g.A = Hs; g.B = Z; g.C = Gr->dV;
        g.M = H; g.N = O; g.K = N;
        g.lda = H; g.ldb = O; g.ldc = O;
        g.a_t = true; g.b_t = false; g.beta = beta; g.splitk_ws = splitk; g.prof_id = K_GEMM_DV;
        RNN_TRY(launch_gemm(g, s));
    }
    // G = dZ V^T
    {
        GemmArgs g{};
        g.A = Z; g.B = P->V; g.C = G;
        g.M = N; g.N = H; g.K = O;
        g.lda = O; g.ldb = O; g.ldc = H;
        g.a_t = false; g.b_t = true; g.beta = 0; g.splitk_ws = splitk; g.prof_id = K_GEMM_G;
        RNN_TRY(launch_gemm(g, s));
    }
    }
    RNN_TRY(run_reverse_loop(d, P->Wh, nullptr, at<float>(ws, pl.WhT), G, h_all, dh_last, Delta, dh0, ws, pl, s));
    // dWh = Delta^T Hprev  (Hprev rows = h_all[0:T])
    if (bf3) {
        // both operands transposed into split form (the planes of h^T used by dV are free again)
        const int Np = bf3_pad(N);
        RNN_TRY(launch_split_bf16(Delta, N, H, H, nullptr, at<uint16_t>(ws, pl.DT), s));
        RNN_TRY(launch_split_bf16(h_all, N, H, H, nullptr, at<uint16_t>(ws, pl.HsT), s));
        Bf3Args b{};
        b.A = at<uint16_t>(ws, pl.DT); b.B = at<uint16_t>(ws, pl.HsT); b.C = Gr->dWh;
        b.M = H; b.N = H; b.K = N; b.lda = Np; b.ldb = Np; b.ldc = H;
        b.beta = beta; b.splitk_ws = at<float>(ws, pl.splitk3); b.prof_id = K_GEMM_DWH;
        RNN_TRY(launch_gemm_bf16x3(b, s));
    } else {
        GemmArgs g{};
        g.A = Delta; g.B = h_all; g.C = Gr->dWh;
        g.M = H; g.N = H; g.K = N;
        g.lda = H; g.ldb = H; g.ldc = H;
        g.a_t = true; g.b_t = false; g.beta = beta; g.splitk_ws = splitk; g.prof_id = K_GEMM_DWH;
        RNN_TRY(launch_gemm(g, s));
    }
    // db = column sums of Delta
    RNN_TRY(launch_colsum_partial(Delta, part, N, H, s));
    RNN_TRY(launch_colsum_finish(part, Gr->db, chunks, H, beta, s));
    // dWx
    if (z.tokens) {
        // the logits buffer is dead by now and serves as scratch for per-range partial rows
        RNN_TRY(launch_dwx_tokens(static_cast<const int32_t*>(x), Delta, Gr->dWx, N, z.NVin, H, beta,
                                  Z, (size_t)N * O, N > 32 ? at<int32_t>(ws, pl.seen) : nullptr, s));
    } else if (bf3) {
        // dWx = Delta^T X: Delta^T is in split form already (dWh), X is transposed into it now
        const int Np = bf3_pad(N);
        RNN_TRY(launch_split_bf16(static_cast<const float*>(x), N, z.NVin, z.NVin, nullptr,
                                  at<uint16_t>(ws, pl.XS), s));
        Bf3Args b{};
        b.A = at<uint16_t>(ws, pl.DT); b.B = at<uint16_t>(ws, pl.XS); b.C = Gr->dWx;
        b.M = H; b.N = z.NVin; b.K = N; b.lda = Np; b.ldb = Np; b.ldc = z.NVin;
        b.beta = beta; b.splitk_ws = at<float>(ws, pl.splitk3); b.prof_id = K_GEMM_DWX;
        RNN_TRY(launch_gemm_bf16x3(b, s));
    } else {
        GemmArgs g{};
        g.A = Delta; g.B = static_cast<const float*>(x); g.C = Gr->dWx;
        g.M = H; g.N = z.NVin; g.K = N;
        g.lda = H; g.ldb = z.NVin; g.ldc = z.NVin;
        g.a_t = true; g.b_t = false; g.beta = beta; g.splitk_ws = splitk; g.prof_id = K_GEMM_DWX;
        RNN_TRY(launch_gemm(g, s));
    }
    return hipSuccess;
}

hipError_t run_bptt(const rnn_dims* d, const rnn_params* P, const void* x, const void* targets,
                    const float* h_all, const float* dh_last, const rnn_grads* Gr, float* dh0,
                    void* ws, const Plan& pl, hipStream_t s) {
    const Sizes z = sizes_of(d);
    const int N = (int)z.N, H = z.H, O = z.O;
    const int beta = (d->flags & RNN_FLAG_ACCUMULATE) ? 1 : 0;
    float* Z = at<float>(ws, pl.Z);
    float* part = at<float>(ws, pl.part);
    float* G = at<float>(ws, pl.G);
    float* Delta = at<float>(ws, pl.Delta);
    const int chunks = colsum_chunks(N);
    const Variant v = pick_variant(d);

    RecResArgs r{};
    r.Wh = P->Wh; r.H = H; r.T = z.T; r.B = z.B; r.act = d->act;
    r.flags = at<int32_t>(ws, pl.flags); r.status = at<int32_t>(ws, pl.scratch) + 1;
    r.G = G; r.h_all = h_all; r.dh_last = dh_last; r.Delta = Delta; r.dh0 = dh0;

    if (v.skinny) {
        // column-strip output layer, then one kernel for the reverse loop and the small
        // weight gradients (dWh, db, touched rows of dWx)
        SkinnyArgs k = skinny_args(d, P, h_all, targets, ws, pl);
        k.dV = Gr->dV; k.dc = Gr->dc; k.beta = beta;
        k.dWx_zero = beta ? nullptr : Gr->dWx;
        k.xids = static_cast<const int32_t*>(x);
        r.gpart = k.gpart; r.gstrips = skinny_strips(O); r.Gw = G;
        k.g_box = at<unsigned long long>(ws, pl.gbox);
        r.g_box = k.g_box;
        r.fuse_post = 1; r.x = static_cast<const int32_t*>(x);
        r.dWh = Gr->dWh; r.db = Gr->db; r.dWx = Gr->dWx; r.beta = beta;
        return launch_rec_bwd_with_strips(r, v.bwd, k, s);
    }

    const bool bf3 = (d->flags & RNN_FLAG_BF16X3_OUTPUT) != 0;
    if (bf3) {
        // logits -> d loss / d logits straight into split form (no float32 copy: nothing reads one) and dc
        int used = 0;
        RNN_TRY(launch_dz_split(Z, at<float>(ws, pl.lse), z.ce ? static_cast<const int32_t*>(targets) : nullptr,
                                z.ce ? nullptr : static_cast<const float*>(targets), part, N, O, d->loss_kind,
                                at<uint16_t>(ws, pl.dZS), at<uint16_t>(ws, pl.dZT), &used, s));
        RNN_TRY(launch_colsum_finish(part, Gr->dc, used, O, beta, s));
        return run_backward_from_dz(d, P, x, h_all, dh_last, Gr, dh0, ws, pl, true, s);
    }
    // logits -> d loss / d logits (in place) and dc
    RNN_TRY(launch_dz(Z, at<float>(ws, pl.lse), z.ce ? static_cast<const int32_t*>(targets) : nullptr,
                      z.ce ? nullptr : static_cast<const float*>(targets), part, N, O,
                      d->loss_kind, s));
    RNN_TRY(launch_colsum_finish(part, Gr->dc, chunks, O, beta, s));
    return run_backward_from_dz(d, P, x, h_all, dh_last, Gr, dh0, ws, pl, false, s);
}

// Extra regions of the Gauss-Newton-vector product behind the ordinary plan.
struct GnPlan {
    Plan base;
    size_t logits, Rh, hrev, splitk_c, RhS, gVT, total;
};

GnPlan make_gn_plan(const rnn_dims* d) {
    const Sizes s = sizes_of(d);
    const size_t N = (size_t)s.N, H = (size_t)s.H, O = (size_t)s.O, B = (size_t)s.B;
    GnPlan p;
    p.base = make_plan(d);
    size_t off = p.base.total;
    auto take = [&](size_t bytes) { const size_t o = off; off += up(bytes); return o; };
    p.logits = take(N * O * 4);
    p.Rh = take(N * H * 4);
    p.hrev = take((N + B) * H * 4);
    p.splitk_c = take(gemm_splitk_floats((int)N, (int)H, (int)H) * 4);   // Hprev gWh^T
    const bool bf3 = (d->flags & RNN_FLAG_BF16X3_OUTPUT) != 0;                // split forms of R h and gamma.V^T
    p.RhS = take(bf3 ? N * (size_t)bf3_pad(s.H) * 4 : 0);
    p.gVT = take(bf3 ? O * (size_t)bf3_pad(s.H) * 4 : 0);
    p.total = off;
    return p;
}

// G gamma = J^T M J gamma (the paper's section on the R-operator).  Forward sweep of the
// R-operator:  R a_t = gin_t + gb + gWh h_{t-1} + Wh R h_{t-1},  R h_t = act'(h_t) R a_t.  Its
// non-recurrent part C_t = gin_t + gb + gWh h_{t-1} is one product over all steps (hoisted like
// the input term); what stays in the loop has the form of the reverse loop of backpropagation
// with time running the other way and Wh transposed, so it runs on that loop's kernels over
// time-reversed rows.  R z = R h V + h gV + gc, the loss metric row by row, then ordinary
// backpropagation of the result.
hipError_t run_gauss_newton(const rnn_dims* d, const rnn_params* P, const rnn_params* Ga, const void* x,
                            const float* h_all, int metric, const rnn_grads* Out, float* Rz_out,
                            void* ws, const GnPlan& gp, hipStream_t s) {
    const Plan& pl = gp.base;
    const Sizes z = sizes_of(d);
    const int N = (int)z.N, H = z.H, O = z.O;
    const size_t BH = (size_t)z.B * H;
    const int beta = (d->flags & RNN_FLAG_ACCUMULATE) ? 1 : 0;
    float* U = at<float>(ws, pl.Z);          // R z, then u = M R z (what backpropagation reads)
    float* Zl = at<float>(ws, gp.logits);
    float* C = at<float>(ws, pl.Delta);
    float* Crev = at<float>(ws, pl.G);
    float* Rhrev = at<float>(ws, pl.Delta);  // C is dead once Crev exists
    float* Rh = at<float>(ws, gp.Rh);
    float* hrev = at<float>(ws, gp.hrev);
    float* WhT = at<float>(ws, pl.WhT);
    float* splitk = at<float>(ws, pl.splitk);
    const float* Hs = h_all + BH;
    const bool ce_metric = metric == RNN_GN_METRIC_LOSS && z.ce;

    const bool bf3 = (d->flags & RNN_FLAG_BF16X3_OUTPUT) != 0;
    const int Hp = bf3_pad(H);
    auto big = [&](const uint16_t* A, const uint16_t* B, float* dst, const float* bias, int acc, int prof) {
        Bf3Args b{};   // [N,O] = A[N,H] B[O,H]^T (+ bias), the shape of all three forward-side products
        b.A = A; b.B = B; b.C = dst;
        b.M = N; b.N = O; b.K = H; b.lda = Hp; b.ldb = Hp; b.ldc = O;
        b.bias_n = bias; b.beta = acc; b.splitk_ws = at<float>(ws, pl.splitk3); b.prof_id = prof;
        return launch_gemm_bf16x3(b, s);
    };
    if (bf3) {   // operands of the large products in split form
        RNN_TRY(launch_split_bf16(Hs, N, H, H, at<uint16_t>(ws, pl.HsS), at<uint16_t>(ws, pl.HsT), s));
        RNN_TRY(launch_split_bf16(P->V, H, O, O, at<uint16_t>(ws, pl.VS), at<uint16_t>(ws, pl.VT), s));
        RNN_TRY(launch_split_bf16(Ga->V, H, O, O, nullptr, at<uint16_t>(ws, gp.gVT), s));
    }
    if (ce_metric && bf3) {
        RNN_TRY(big(at<uint16_t>(ws, pl.HsS), at<uint16_t>(ws, pl.VT), Zl, P->c, 0, K_GEMM_LOGITS));
    } else if (ce_metric) {   // logits of the current parameters, for the softmax in the metric
        GemmArgs g{};
        g.A = Hs; g.B = P->V; g.C = Zl;
        g.M = N; g.N = O; g.K = H; g.lda = H; g.ldb = O; g.ldc = O;
        g.a_t = false; g.b_t = false; g.bias_n = P->c; g.beta = 0; g.prof_id = K_GEMM_LOGITS;
        g.splitk_ws = splitk;
        RNN_TRY(launch_gemm(g, s));
    }
    {   // C = Hprev gWh^T + gb
        GemmArgs g{};
        g.A = h_all; g.B = Ga->Wh; g.C = C;
        g.M = N; g.N = H; g.K = H; g.lda = H; g.ldb = H; g.ldc = H;
        g.a_t = false; g.b_t = true; g.bias_n = Ga->b; g.beta = 0; g.prof_id = K_GEMM_U;
        g.splitk_ws = at<float>(ws, gp.splitk_c);
        RNN_TRY(launch_gemm(g, s));
    }
    if (z.tokens) {
        RNN_TRY(launch_gather_add(static_cast<const int32_t*>(x), Ga->Wx, C, N, H, s));
    } else {   // C += X gWx^T
        GemmArgs g{};
        g.A = static_cast<const float*>(x); g.B = Ga->Wx; g.C = C;
        g.M = N; g.N = H; g.K = z.NVin; g.lda = z.NVin; g.ldb = z.NVin; g.ldc = H;
        g.a_t = false; g.b_t = true; g.beta = 1; g.prof_id = K_GEMM_U; g.splitk_ws = splitk;
        RNN_TRY(launch_gemm(g, s));
    }
    // time-reversed rows: Crev[t] = C[T-1-t], hrev[t+1] = h_{T-1-t}
    RNN_TRY(launch_reverse_rows(C, Crev, z.T, (int)BH, s));
    RNN_TRY(launch_reverse_rows(Hs, hrev + BH, z.T, (int)BH, s));
    RNN_TRY(launch_transpose(P->Wh, WhT, H, H, s));
    RNN_TRY(run_reverse_loop(d, WhT, P->Wh, nullptr, Crev, hrev, nullptr, Rhrev, nullptr, ws, pl, s));
    RNN_TRY(launch_reverse_rows(Rhrev, Rh, z.T, (int)BH, s));
    if (bf3) {   // R z = Rh V + gc + Hs gV
        RNN_TRY(launch_split_bf16(Rh, N, H, H, at<uint16_t>(ws, gp.RhS), nullptr, s));
        RNN_TRY(big(at<uint16_t>(ws, gp.RhS), at<uint16_t>(ws, pl.VT), U, Ga->c, 0, K_GEMM_LOGITS));
        RNN_TRY(big(at<uint16_t>(ws, pl.HsS), at<uint16_t>(ws, gp.gVT), U, nullptr, 1, K_GEMM_LOGITS));
    } else {   // R z = Rh V + gc
        GemmArgs g{};
        g.A = Rh; g.B = P->V; g.C = U;
        g.M = N; g.N = O; g.K = H; g.lda = H; g.ldb = O; g.ldc = O;
        g.a_t = false; g.b_t = false; g.bias_n = Ga->c; g.beta = 0; g.prof_id = K_GEMM_LOGITS;
        g.splitk_ws = splitk;
        RNN_TRY(launch_gemm(g, s));
        // ... + Hs gV
        g.A = Hs; g.B = Ga->V; g.bias_n = nullptr; g.beta = 1;
        RNN_TRY(launch_gemm(g, s));
    }
    if (Rz_out)
        RNN_TRY(hipMemcpyAsync(Rz_out, U, (size_t)N * O * 4, hipMemcpyDeviceToDevice, s));
    if (ce_metric)
        RNN_TRY(launch_gn_softmax_metric(Zl, U, N, O, 1.0f / (float)N, s));
    else if (metric == RNN_GN_METRIC_LOSS)
        RNN_TRY(launch_scale(U, (size_t)N * O, (float)(2.0 / ((double)N * (double)O)), s));
    // Gc = column sums of u, then the rest of backpropagation
    RNN_TRY(launch_colsum_partial(U, at<float>(ws, pl.part), N, O, s));
    RNN_TRY(launch_colsum_finish(at<float>(ws, pl.part), Out->dc, colsum_chunks(N), O, beta, s));
    if (bf3) RNN_TRY(launch_split_bf16(U, N, O, O, at<uint16_t>(ws, pl.dZS), at<uint16_t>(ws, pl.dZT), s));
    return run_backward_from_dz(d, P, x, h_all, nullptr, Out, nullptr, ws, pl, bf3, s);
}

bool params_ok(const rnn_params* P) {
    return P && P->Wx && P->Wh && P->b && P->V && P->c && !misaligned(P->Wx) && !misaligned(P->Wh) &&
           !misaligned(P->b) && !misaligned(P->V) && !misaligned(P->c);
}

bool reference_supported(const rnn_dims* d) { return d->hidden <= 8192; }

}  // namespace

namespace rnn {
int wait_limit() { return g_wait_limit.load(std::memory_order_relaxed); }
}  // namespace rnn

namespace rnn {
// device address of the status word inside a three-call workspace (checked by the caller)
int32_t* three_call_status_word(const rnn_dims* dims, void* workspace) {
    Plan pl;
    size_t bytes = 0;
    if (rnn_workspace_bytes(dims, &bytes) != RNN_OK || check_ws(dims, workspace, bytes, &pl) != RNN_OK) return nullptr;
    return at<int32_t>(workspace, pl.scratch) + 1;
}
}  // namespace rnn

extern "C" {

int rnn_set_wait_limit(int polls) {
    g_wait_limit.store(polls > 0 ? polls : (1 << 22), std::memory_order_relaxed);
    return RNN_OK;
}

int rnn_workspace_bytes(const rnn_dims* dims, size_t* bytes) {
    if (!dims_valid(dims) || !bytes) return RNN_EINVAL;
    *bytes = make_plan(dims).total;
    return RNN_OK;
}

int rnn_forward(const rnn_dims* dims, const rnn_params* params, const void* x, const float* h0,
                float* h_all, float* h_last, void* workspace, size_t workspace_bytes,
                void* hip_stream) {
    if (!dims_valid(dims) || !params_ok(params) || !x || (!h_all && !h_last)) return RNN_EINVAL;
    if (misaligned4(x) || misaligned(h0) || misaligned(h_all) || misaligned(h_last)) return RNN_EINVAL;
    if (!reference_supported(dims)) return RNN_EUNSUPPORTED;
    Plan pl;
    const int rc = check_ws(dims, workspace, workspace_bytes, &pl);
    if (rc != RNN_OK) return rc;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    return finish(dims, s, run_forward(dims, params, x, h0, h_all, h_last, workspace, pl, s));
}

int rnn_loss(const rnn_dims* dims, const rnn_params* params, const float* h_all, const void* targets,
             float* loss, void* workspace, size_t workspace_bytes, void* hip_stream) {
    if (!dims_valid(dims) || !params_ok(params) || !h_all || !targets || !loss) return RNN_EINVAL;
    if (misaligned(h_all) || misaligned4(targets) || misaligned4(loss)) return RNN_EINVAL;
    Plan pl;
    const int rc = check_ws(dims, workspace, workspace_bytes, &pl);
    if (rc != RNN_OK) return rc;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    return finish(dims, s, run_loss(dims, params, h_all, targets, loss, workspace, pl, s));
}

int rnn_bptt(const rnn_dims* dims, const rnn_params* params, const void* x, const void* targets,
             const float* h_all, const float* dh_last, const rnn_grads* grads, float* dh0,
             void* workspace, size_t workspace_bytes, void* hip_stream) {
    if (!dims_valid(dims) || !params_ok(params) || !x || !targets || !h_all || !grads)
        return RNN_EINVAL;
    if (!grads->dWx || !grads->dWh || !grads->db || !grads->dV || !grads->dc) return RNN_EINVAL;
    if (misaligned4(x) || misaligned4(targets) || misaligned(h_all) || misaligned(dh_last) ||
        misaligned(dh0) || misaligned(grads->dWx) || misaligned(grads->dWh) ||
        misaligned(grads->db) || misaligned(grads->dV) || misaligned(grads->dc))
        return RNN_EINVAL;
    if (!reference_supported(dims)) return RNN_EUNSUPPORTED;
    Plan pl;
    const int rc = check_ws(dims, workspace, workspace_bytes, &pl);
    if (rc != RNN_OK) return rc;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    if (dims->flags & RNN_FLAG_BPTT_RECOMPUTE) {
        // recompute logits and row statistics; the scalar loss goes to workspace scratch
        hipError_t e = run_loss(dims, params, h_all, targets, at<float>(workspace, pl.scratch),
                                workspace, pl, s);
        if (e != hipSuccess) return RNN_EHIP;
    }
    return finish(dims, s, run_bptt(dims, params, x, targets, h_all, dh_last, grads, dh0, workspace, pl, s));
}

int rnn_gauss_newton_workspace_bytes(const rnn_dims* dims, size_t* bytes) {
    if (!dims_valid(dims) || !bytes) return RNN_EINVAL;
    *bytes = make_gn_plan(dims).total;
    return RNN_OK;
}

int rnn_gauss_newton_vec(const rnn_dims* dims, const rnn_params* params, const rnn_params* gamma,
                         const void* x, const float* h_all, int32_t metric, const rnn_grads* out,
                         float* Rz, void* workspace, size_t workspace_bytes, void* hip_stream) {
    if (!dims_valid(dims) || !params_ok(params) || !params_ok(gamma) || !x || !h_all || !out)
        return RNN_EINVAL;
    if (metric != RNN_GN_METRIC_LOSS && metric != RNN_GN_METRIC_IDENTITY) return RNN_EINVAL;
    if (dims->flags & RNN_FLAG_BPTT_RECOMPUTE) return RNN_EINVAL;
    if (!out->dWx || !out->dWh || !out->db || !out->dV || !out->dc) return RNN_EINVAL;
    if (misaligned4(x) || misaligned(h_all) || misaligned(Rz) || misaligned(out->dWx) ||
        misaligned(out->dWh) || misaligned(out->db) || misaligned(out->dV) || misaligned(out->dc))
        return RNN_EINVAL;
    if (!reference_supported(dims)) return RNN_EUNSUPPORTED;
    const GnPlan gp = make_gn_plan(dims);
    if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 15u) || workspace_bytes < gp.total)
        return RNN_EWORKSPACE;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    return finish(dims, s, run_gauss_newton(dims, params, gamma, x, h_all, metric, out, Rz, workspace, gp, s));
}

int rnn_check_tokens(const void* ids, int64_t n, int32_t limit, int32_t* bad_count, void* hip_stream) {
    if (!ids || !bad_count || n < 0 || limit <= 0) return RNN_EINVAL;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    return launch_check_tokens(static_cast<const int32_t*>(ids), n, limit, bad_count, s) == hipSuccess
               ? RNN_OK : RNN_EHIP;
}

const char* rnn_strerror(int code) {
    switch (code) {
        case RNN_OK: return "ok";
        case RNN_EINVAL: return "invalid argument (size, enum, flag, alignment or NULL required pointer)";
        case RNN_EWORKSPACE: return "workspace missing, misaligned or too small (see rnn_workspace_bytes)";
        case RNN_EUNSUPPORTED: return "no kernel for this shape in this build";
        case RNN_EHIP: return "HIP launch or synchronisation failed";
        case RNN_ETOOLARGE: return "problem needs more than the fixed scratch array of rnn_window_static (use rnn_window)";
        default: return "unknown error code";
    }
}

const char* rnn_recurrence_variant(const rnn_dims* dims) {
    if (!dims_valid(dims)) return "invalid";
    const Variant v = pick_variant(dims);
    if (v.batch_mfma) return "batch_mfma";
    if (v.stepwise) return rec_xcd_supported(dims->hidden, dims->batch, dims->seq_len) ? "xcd_mfma" : "step_mfma";
    if (!v.resident) return "reference";
    return (v.fwd.P == 1 && !v.grid) ? "wg_resident" : "grid_resident";
}

int rnn_recurrence_workgroups(const rnn_dims* dims) {
    if (!dims_valid(dims)) return RNN_EINVAL;
    const Variant v = pick_variant(dims);
    const Sizes s = sizes_of(dims);
    if (v.batch_mfma) return (s.B + 3) / 4;
    if (v.stepwise && rec_xcd_supported(s.H, s.B, s.T)) return ((s.B + 3) / 4) * ((s.H + 63) / 64);
    if (v.stepwise) return ((s.H + 15) / 16) * ((s.B + 15) / 16);   // tiles of one step launch
    if (!v.resident) return s.B;
    if (v.grid) return v.gplan.P * s.B;
    return v.fwd.P * s.B;
}

int rnn_workspace_status(const rnn_dims* dims, const void* workspace, size_t workspace_bytes,
                         void* hip_stream, int32_t* status_host) {
    if (!dims_valid(dims) || !status_host) return RNN_EINVAL;
    Plan pl;
    const int rc = check_ws(dims, const_cast<void*>(workspace), workspace_bytes, &pl);
    if (rc != RNN_OK) return rc;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    if (hipMemcpyAsync(status_host, at<int32_t>(const_cast<void*>(workspace), pl.scratch) + 1, 4,
                       hipMemcpyDeviceToHost, s) != hipSuccess)
        return RNN_EHIP;
    return hipStreamSynchronize(s) == hipSuccess ? RNN_OK : RNN_EHIP;
}

int rnn_workspace_init(const rnn_dims* dims, void* workspace, size_t workspace_bytes, void* hip_stream) {
    if (!dims_valid(dims)) return RNN_EINVAL;
    Plan pl;
    const int rc = check_ws(dims, workspace, workspace_bytes, &pl);
    if (rc != RNN_OK) return rc;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    if (launch_zero_words(at<int32_t>(workspace, pl.scratch), 64, s) != hipSuccess) return RNN_EHIP;
    // exchange words start cleared: tag 0 is never a valid tag
    const Sizes z = sizes_of(dims);
    if (z.N <= 32) {
        const size_t words = skinny_stat_box_bytes((int)z.N, z.O) / 4;
        if (launch_zero_words(at<int32_t>(workspace, pl.statbox), (int)words, s) != hipSuccess) return RNN_EHIP;
        if (launch_zero_words(at<int32_t>(workspace, pl.gbox), (int)(z.N * z.H * 2), s) != hipSuccess) return RNN_EHIP;
    }
    return RNN_OK;
}

}  // extern "C"
