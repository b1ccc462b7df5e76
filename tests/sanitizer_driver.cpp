// Driver for tests/test_sanitizers.py: built together with csrc/pd_host.cpp and oracle/layer_oracle.c
// under -fsanitize=address,undefined.  Reads one case file written by the test, runs the host entry
// points of the library and the layer oracle on it, and writes every result to an output file that
// the test compares with what the ordinary builds return.  Test infrastructure only.
//
// Case file: int32 header[16] = {d, Hq, Hkv, hd, F, E, top_k, T, n_seqs, B, max_len, n_req, 0...},
// then float32 arrays in this order: g_attn[d], w_q, w_k, w_v, w_o, g_ffn[d], w_gate, w_up, w_down,
// x[T, d], xdec[B, d], int32 cu[n_seqs + 1], float64 arrival[n_req], service[n_req].
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <vector>

#include "pd.h"

extern "C" {
typedef struct {
    int32_t d_model, n_q_heads, n_kv_heads, head_dim, d_ff, n_experts, top_k, act8;
    double rms_eps, rope_base;
} orc_config;
typedef struct {
    const float *g_attn, *w_q, *w_k, *w_v, *w_o, *g_ffn, *w_gate, *w_up, *w_down, *w_router;
} orc_weights;
int orc_prefill(const orc_config *, const orc_weights *, const float *, int, int, const int32_t *, const float *,
                const int32_t *, int, const int32_t *, float *, float *, int32_t *, int, float *, int32_t *, int,
                double, double);
int orc_decode_step(const orc_config *, const orc_weights *, const float *, int, const int32_t *, float *, float *,
                    int32_t *, int, const float *, float *, int32_t *, int, double, double);
int orc_prefill_chunk(const orc_config *, const orc_weights *, const float *, int, int, const int32_t *,
                      const float *, const int32_t *, float *, float *, int32_t *, int, float *, int32_t *, int,
                      double, double);
void orc_quantise_rows(float *, int, int, float *);
void orc_act_quantise_rows(float *, int, int, float *, uint8_t *);
}

static FILE *g_out;
static void put(const void *p, size_t bytes) { fwrite(p, 1, bytes, g_out); }

template <typename T>
static std::vector<T> take(FILE *f, size_t n)
{
    std::vector<T> v(n);
    if (n && fread(v.data(), sizeof(T), n, f) != n) {
        fprintf(stderr, "short case file\n");
        exit(3);
    }
    return v;
}

int main(int argc, char **argv)
{
    if (argc != 3) return 2;
    FILE *f = fopen(argv[1], "rb");
    g_out = fopen(argv[2], "wb");
    if (!f || !g_out) return 2;
    std::vector<int32_t> h = take<int32_t>(f, 16);
    const int d = h[0], Hq = h[1], Hkv = h[2], hd = h[3], F = h[4], E = h[5], top_k = h[6], T = h[7], n_seqs = h[8],
              B = h[9], max_len = h[10], n_req = h[11];
    const int G = E > 0 ? E : 1;
    auto g_attn = take<float>(f, d);
    auto w_q = take<float>(f, (size_t)Hq * hd * d), w_k = take<float>(f, (size_t)Hkv * hd * d),
         w_v = take<float>(f, (size_t)Hkv * hd * d), w_o = take<float>(f, (size_t)d * Hq * hd);
    auto g_ffn = take<float>(f, d);
    auto w_gate = take<float>(f, (size_t)G * F * d), w_up = take<float>(f, (size_t)G * F * d),
         w_down = take<float>(f, (size_t)G * d * F);
    auto w_router = take<float>(f, (size_t)E * d);
    auto x = take<float>(f, (size_t)T * d), xdec = take<float>(f, (size_t)B * d);
    auto cu = take<int32_t>(f, (size_t)n_seqs + 1);
    auto arrival = take<double>(f, n_req), service = take<double>(f, n_req);
    fclose(f);

    // ---- allocation model and queue formulas ------------------------------------------------------
    {
        // the worked example of the paper's Evaluation section, then the error paths
        int32_t batch[3] = {8, 34, 64};
        double tpot[3] = {0.012, 0.020, 0.031};
        pd_measured_curves cv;
        memset(&cv, 0, sizeof(cv));
        cv.prefill_max_tps = 28300.0; cv.n_decode = 3; cv.decode_batch = batch; cv.decode_tpot_s = tpot;
        cv.t_overhead_s = 0.1; cv.rounding = 0;
        pd_allocation a;
        memset(&a, 0, sizeof(a));
        int32_t st = pd_allocate(5e6 / 60.0, 6144.0, 512.0, 2.0, 0.020, &cv, &a);
        put(&st, 4); put(&a.n_prefill, 4); put(&a.n_decode, 4); put(&a.tp_prefill_eff, 8); put(&a.ratio_pd, 8);
        st = pd_allocate(5e6 / 60.0, 6144.0, 512.0, 0.05, 0.020, &cv, &a); put(&st, 4);     // TTFT infeasible
        st = pd_allocate(5e6 / 60.0, 6144.0, 512.0, 2.0, 0.001, &cv, &a); put(&st, 4);      // TPOT infeasible
        cv.n_decode = 0;
        st = pd_allocate(5e6 / 60.0, 6144.0, 512.0, 2.0, 0.020, &cv, &a); put(&st, 4);      // empty curve
        st = pd_allocate(5e6 / 60.0, 6144.0, 512.0, 2.0, 0.020, nullptr, &a); put(&st, 4);
        const char *msg = pd_last_error();
        put(msg, strlen(msg) > 0 ? 1 : 0);
        double work[3] = {1024.0, 6144.0, 512.0}, tps[3] = {9000.0, 25066.0, 1700.0}, n_real[3];
        int32_t n_inst[3];
        st = pd_allocate_stages(3, 5e6 / 60.0, 6144.0, 512.0, work, tps, 1, n_real, n_inst);
        put(&st, 4); put(n_real, 24); put(n_inst, 12);
        std::vector<double> soj(n_req), soj_b(n_req);
        st = pd_fifo_replay(n_req, arrival.data(), service.data(), soj.data()); put(&st, 4); put(soj.data(), 8 * (size_t)n_req);
        double bsvc[4] = {0.05, 0.08, 0.11, 0.13};
        st = pd_fifo_replay_batched(n_req, arrival.data(), 4, bsvc, soj_b.data()); put(&st, 4); put(soj_b.data(), 8 * (size_t)n_req);
        st = pd_fifo_replay(0, nullptr, nullptr, nullptr); put(&st, 4);
        double t = 0.0;
        st = pd_mm1_sojourn(28300.0, 6144.0, 25066.3 / 6144.0, &t); put(&st, 4); put(&t, 8);
        st = pd_mg1_sojourn(3.0, 0.2, 0.05, &t); put(&st, 4); put(&t, 8);
        st = pd_mg1_sojourn(6.0, 0.2, 0.05, &t); put(&st, 4);
        st = pd_prefill_throughput_dp(28300.0, 6144.0, 2.0, 0.1, 4, &t); put(&st, 4); put(&t, 8);
        st = pd_kv_transfer_overhead(6144.0, 32, 8, 128, 2.0, 50e9, 0.001, &t); put(&st, 4); put(&t, 8);
        for (int s = 0; s <= 9; ++s) {
            const char *name = pd_status_string((pd_status)s);
            put(name, 1);
        }
    }

    // ---- layer oracle ---------------------------------------------------------------------------------
    orc_config c = {d, Hq, Hkv, hd, F, E, top_k, 0, 1e-6, 10000.0};
    orc_weights w = {g_attn.data(), w_q.data(), w_k.data(), w_v.data(), w_o.data(), g_ffn.data(),
                     w_gate.data(), w_up.data(), w_down.data(), E > 0 ? w_router.data() : nullptr};
    const size_t plane = (size_t)Hkv * max_len * hd;
    std::vector<int32_t> slots(n_seqs), eidx((size_t)(T > B ? T : B) * (top_k > 0 ? top_k : 1));
    for (int s = 0; s < n_seqs; ++s) slots[s] = n_seqs - 1 - s;
    for (int pass = 0; pass < 3; ++pass) {
        // pass 0: exact cache; pass 1: 8-bit cache; pass 2: 8-bit activations
        const int fp8 = pass == 1;
        c.act8 = pass == 2;
        std::vector<float> kc((size_t)n_seqs * plane, 0.f), vc((size_t)n_seqs * plane, 0.f);
        std::vector<int32_t> lens(n_seqs, 0);
        std::vector<float> out((size_t)T * d);
        int rc = orc_prefill(&c, &w, x.data(), T, n_seqs, cu.data(), nullptr, nullptr, T, slots.data(), kc.data(),
                             vc.data(), lens.data(), max_len, out.data(), eidx.data(), fp8, 0.5, 0.125);
        put(&rc, 4); put(out.data(), 4 * out.size()); put(lens.data(), 4 * lens.size());
        // sampled rows of the same call
        int32_t rows[3] = {0, T / 2, T - 1};
        std::vector<float> outr((size_t)3 * d);
        rc = orc_prefill(&c, &w, x.data(), T, n_seqs, cu.data(), nullptr, rows, 3, nullptr, nullptr, nullptr, nullptr,
                         0, outr.data(), eidx.data(), 0, 1.0, 1.0);
        put(&rc, 4); put(outr.data(), 4 * outr.size());
        // decode steps on the first B slots until one of them is full
        std::vector<int32_t> dslots(B);
        for (int b = 0; b < B; ++b) dslots[b] = b;
        std::vector<float> outd((size_t)B * d);
        for (int step = 0; step < 3; ++step) {
            rc = orc_decode_step(&c, &w, xdec.data(), B, dslots.data(), kc.data(), vc.data(), lens.data(), max_len,
                                 nullptr, outd.data(), eidx.data(), fp8, 0.5, 0.125);
            put(&rc, 4);
            if (rc == 0) put(outd.data(), 4 * outd.size());
        }
        // a chunk of the prompt rows behind what the slots now hold (capacity error if it does not fit)
        rc = orc_prefill_chunk(&c, &w, x.data(), T, n_seqs, cu.data(), nullptr, slots.data(), kc.data(), vc.data(),
                               lens.data(), max_len, out.data(), eidx.data(), fp8, 0.5, 0.125);
        put(&rc, 4);
        if (rc == 0) put(out.data(), 4 * out.size());
        put(lens.data(), 4 * lens.size());
    }
    {
        std::vector<float> wq = w_q, sc((size_t)Hq * hd);
        orc_quantise_rows(wq.data(), Hq * hd, d, sc.data());
        put(wq.data(), 4 * wq.size()); put(sc.data(), 4 * sc.size());
        std::vector<float> xa = x, sa(T);
        std::vector<uint8_t> codes((size_t)T * d);
        orc_act_quantise_rows(xa.data(), T, d, sa.data(), codes.data());
        put(xa.data(), 4 * xa.size()); put(sa.data(), 4 * sa.size()); put(codes.data(), codes.size());
    }
    fclose(g_out);
    return 0;
}
