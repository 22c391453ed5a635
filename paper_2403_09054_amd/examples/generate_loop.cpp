// Stand-alone use of the Keyformer C ABI (include/keyformer.h) without Python:
// device memory from hipMalloc, a synthetic prompt, prompt scoring + first
// eviction, then a run of generation steps replayed from ONE captured HIP graph
// node set (kf_decode_select_step_at keeps the step number in device memory).
// After every step the program checks what Algorithm 1 guarantees whatever the
// data: the cache holds k tokens, in ascending original position, the w most
// recent ones among them, finite attention outputs, and every unit's scores
// grew by exactly one probability vector.  Exit code 0 = all checks passed.
//
//   hipcc --offload-arch=gfx950 generate_loop.cpp -I../../include -L.. -lkeyformer -o generate_loop
#include <hip/hip_runtime.h>
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <vector>

#include "keyformer.h"

#define HIP_OK(x)                                                                      \
    do {                                                                               \
        hipError_t e_ = (x);                                                           \
        if (e_ != hipSuccess) {                                                        \
            fprintf(stderr, "%s:%d %s: %s\n", __FILE__, __LINE__, #x, hipGetErrorString(e_)); \
            return 2;                                                                  \
        }                                                                              \
    } while (0)
#define KF_OK_(x)                                                                   \
    do {                                                                            \
        kf_status s_ = (x);                                                         \
        if (s_ != KF_OK) {                                                          \
            fprintf(stderr, "%s:%d %s: %d %s\n", __FILE__, __LINE__, #x, (int)s_, kf_last_error()); \
            return 3;                                                               \
        }                                                                           \
    } while (0)

static uint16_t to_bf16(float f) {  // round to nearest even
    uint32_t u;
    memcpy(&u, &f, 4);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

static uint64_t rng_state = 0x2403090541ull;
static float rnd_normal() {  // Box-Muller on a 64-bit LCG: input data only
    rng_state = rng_state * 6364136223846793005ull + 1442695040888963407ull;
    const double u1 = ((rng_state >> 11) + 1.0) / 9007199254740993.0;
    rng_state = rng_state * 6364136223846793005ull + 1442695040888963407ull;
    const double u2 = (rng_state >> 11) / 9007199254740992.0;
    return (float)(sqrt(-2.0 * log(u1)) * cos(6.283185307179586 * u2));
}
static void fill_bf16(std::vector<uint16_t>& v) {
    for (auto& x : v) x = to_bf16(rnd_normal());
}

int main() {
    const int L = 2, B = 2, H = 4, d = 128, n = 384, k = 192, w = 38, T = 24, steps = 30;
    const int U = L * B * H;
    const float scale = 1.0f / sqrtf((float)d);
    const kf_schedule sched = {n, T, 1.0f, 2.0f};

    // ---- prompt cache (cap = n) and generation cache (cap = k+1)
    kf_cache prompt = {}, gen = {};
    prompt.L = gen.L = L;
    prompt.B = gen.B = B;
    prompt.H = gen.H = H;
    prompt.d = gen.d = d;
    prompt.dtype = gen.dtype = KF_BF16;
    prompt.cap = n;
    gen.cap = k + 1;
    for (kf_cache* c : {&prompt, &gen}) {
        const size_t rows = (size_t)U * c->cap;
        HIP_OK(hipMalloc(&c->K, rows * d * 2));
        HIP_OK(hipMalloc(&c->V, rows * d * 2));
        HIP_OK(hipMalloc((void**)&c->score, rows * 4));
        HIP_OK(hipMalloc((void**)&c->pos, rows * 4));
        HIP_OK(hipMalloc((void**)&c->len, (size_t)U * 4));
        HIP_OK(hipMemset(c->len, 0, (size_t)U * 4));
    }
    std::vector<uint16_t> hK((size_t)U * n * d), hV(hK.size()), hQ(hK.size());
    fill_bf16(hK);
    fill_bf16(hV);
    fill_bf16(hQ);
    void* dQ;
    HIP_OK(hipMalloc(&dQ, hQ.size() * 2));
    HIP_OK(hipMemcpy(prompt.K, hK.data(), hK.size() * 2, hipMemcpyHostToDevice));
    HIP_OK(hipMemcpy(prompt.V, hV.data(), hV.size() * 2, hipMemcpyHostToDevice));
    HIP_OK(hipMemcpy(dQ, hQ.data(), hQ.size() * 2, hipMemcpyHostToDevice));

    uint64_t hseeds[B] = {20240309ull, 20240310ull};
    uint64_t* dseeds;
    HIP_OK(hipMalloc((void**)&dseeds, sizeof(hseeds)));
    HIP_OK(hipMemcpy(dseeds, hseeds, sizeof(hseeds), hipMemcpyHostToDevice));

    size_t ws_bytes = kf_workspace_bytes(&prompt, n);
    const size_t ws_gen = kf_workspace_bytes(&gen, 0);
    if (ws_gen > ws_bytes) ws_bytes = ws_gen;
    void* ws;
    HIP_OK(hipMalloc(&ws, ws_bytes));
    HIP_OK(hipMemset(ws, 0, ws_bytes));  // once: the library leaves it reusable

    hipStream_t stream;
    HIP_OK(hipStreamCreate(&stream));
    kf_score_cfg cfg = {};
    cfg.tau = kf_tau(0, T, sched.tau_init, sched.tau_end);
    cfg.scale = scale;
    cfg.noise = KF_NOISE_GUMBEL;
    cfg.seeds = dseeds;

    // ---- prompt phase: score, then keep k of n tokens, gathered into the generation cache
    KF_OK_(kf_prefill_score(&prompt, dQ, n, &cfg, ws, ws_bytes, stream));
    KF_OK_(kf_select_evict_into(&prompt, &gen, 0, k, w, nullptr, ws, ws_bytes, stream));
    HIP_OK(hipStreamSynchronize(stream));

    // ---- generation: one step captured, replayed `steps` times
    void *dq, *dkn, *dvn;
    float* dout;
    int32_t* dstep;
    const size_t vec = (size_t)U * d;
    HIP_OK(hipMalloc(&dq, vec * 2));
    HIP_OK(hipMalloc(&dkn, vec * 2));
    HIP_OK(hipMalloc(&dvn, vec * 2));
    HIP_OK(hipMalloc((void**)&dout, vec * 4));
    HIP_OK(hipMalloc((void**)&dstep, 4));
    const int32_t one = 1;
    HIP_OK(hipMemcpy(dstep, &one, 4, hipMemcpyHostToDevice));

    hipGraph_t graph;
    hipGraphExec_t exec;
    HIP_OK(hipStreamBeginCapture(stream, hipStreamCaptureModeGlobal));
    KF_OK_(kf_decode_select_step_at(&gen, dq, dkn, dvn, &sched, dstep, k + 1, &cfg, dout, k, w, KF_LAYOUT_ORDERED,
                                    nullptr, ws, ws_bytes, stream));
    HIP_OK(hipStreamEndCapture(stream, &graph));
    HIP_OK(hipGraphInstantiate(&exec, graph, nullptr, nullptr, 0));

    std::vector<uint16_t> hq(vec), hkn(vec), hvn(vec);
    std::vector<float> hout(vec), hscore((size_t)U * gen.cap);
    std::vector<int32_t> hpos((size_t)U * gen.cap), hlen(U);
    std::vector<double> mass(U, 0.0);
    auto read_state = [&]() -> int {
        HIP_OK(hipMemcpy(hscore.data(), gen.score, hscore.size() * 4, hipMemcpyDeviceToHost));
        HIP_OK(hipMemcpy(hpos.data(), gen.pos, hpos.size() * 4, hipMemcpyDeviceToHost));
        HIP_OK(hipMemcpy(hlen.data(), gen.len, hlen.size() * 4, hipMemcpyDeviceToHost));
        return 0;
    };
    if (read_state()) return 2;
    for (int u = 0; u < U; ++u) {
        if (hlen[u] != k) { fprintf(stderr, "unit %d: len %d after the prompt phase\n", u, hlen[u]); return 1; }
        for (int j = 0; j < k; ++j) mass[u] += hscore[(size_t)u * gen.cap + j];
    }
    int failures = 0;
    for (int t = 1; t <= steps; ++t) {
        fill_bf16(hq);
        fill_bf16(hkn);
        fill_bf16(hvn);
        HIP_OK(hipMemcpyAsync(dq, hq.data(), vec * 2, hipMemcpyHostToDevice, stream));
        HIP_OK(hipMemcpyAsync(dkn, hkn.data(), vec * 2, hipMemcpyHostToDevice, stream));
        HIP_OK(hipMemcpyAsync(dvn, hvn.data(), vec * 2, hipMemcpyHostToDevice, stream));
        HIP_OK(hipGraphLaunch(exec, stream));
        HIP_OK(hipMemcpyAsync(hout.data(), dout, vec * 4, hipMemcpyDeviceToHost, stream));
        HIP_OK(hipStreamSynchronize(stream));
        if (read_state()) return 2;
        const int q_pos = n + t - 1;
        for (int u = 0; u < U; ++u) {
            const int32_t* p = &hpos[(size_t)u * gen.cap];
            const float* f = &hscore[(size_t)u * gen.cap];
            bool ok = hlen[u] == k;
            for (int j = 1; ok && j < k; ++j) ok = p[j] > p[j - 1];
            for (int j = 0; ok && j < w; ++j) ok = p[k - w + j] == q_pos - w + 1 + j;
            for (int c = 0; ok && c < d; ++c) ok = isfinite(hout[(size_t)u * d + c]);
            // the step added a probability vector to the k+1 scores and removed the evicted token's score:
            // the retained mass can have grown by at most 1 and must not have shrunk by more than that score
            double now = 0.0;
            for (int j = 0; j < k; ++j) now += f[j];
            ok = ok && now <= mass[u] + 1.0 + 1e-3 && now > 0.0;
            mass[u] = now;
            if (!ok) {
                ++failures;
                fprintf(stderr, "step %d unit %d: invariant violated (len %d)\n", t, u, hlen[u]);
            }
        }
    }
    // ---- beam search bookkeeping: sequence 1 is replaced by a continuation of sequence 0
    {
        const int32_t parent[2] = {0, 0};
        int32_t* dparent;
        HIP_OK(hipMalloc((void**)&dparent, sizeof(parent)));
        HIP_OK(hipMemcpy(dparent, parent, sizeof(parent), hipMemcpyHostToDevice));
        KF_OK_(kf_beam_fork(&gen, dparent, ws, ws_bytes, stream));
        HIP_OK(hipStreamSynchronize(stream));
        if (read_state()) return 2;
        for (int l = 0; l < L; ++l) {
            for (int h = 0; h < H; ++h) {
                const size_t u0 = ((size_t)l * B + 0) * H + h, u1 = ((size_t)l * B + 1) * H + h;
                bool ok = hlen[u0] == hlen[u1];
                for (int j = 0; ok && j < hlen[u0]; ++j)
                    ok = hpos[u0 * gen.cap + j] == hpos[u1 * gen.cap + j] && hscore[u0 * gen.cap + j] == hscore[u1 * gen.cap + j];
                if (!ok) {
                    ++failures;
                    fprintf(stderr, "beam fork: layer %d head %d differs from its parent\n", l, h);
                }
            }
        }
        HIP_OK(hipFree(dparent));
    }
    int32_t hstep = 0, herr = 0;
    HIP_OK(hipMemcpy(&hstep, dstep, 4, hipMemcpyDeviceToHost));
    HIP_OK(hipMemcpy(&herr, (int32_t*)ws + KF_WS_ERROR_WORD, 4, hipMemcpyDeviceToHost));
    if (hstep != steps + 1) { fprintf(stderr, "device step counter %d, expected %d\n", hstep, steps + 1); ++failures; }
    if (herr != 0) { fprintf(stderr, "workspace error word %d\n", herr); ++failures; }
    printf("generate_loop: %d units, %d steps replayed from one captured step, tau %.3f -> %.3f, %s\n", U, steps,
           kf_tau(1, T, sched.tau_init, sched.tau_end), kf_tau(T, T, sched.tau_init, sched.tau_end),
           failures ? "FAILED" : "all invariants hold");
    HIP_OK(hipGraphExecDestroy(exec));
    HIP_OK(hipGraphDestroy(graph));
    return failures ? 1 : 0;
}
