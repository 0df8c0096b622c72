// Host-only quantizer behind qtip_quantize: Viterbi on the (L, k, V) bitshift
// trellis (Section 2.3 of arXiv 2406.11235) with the tail-biting approximation of
// Algorithm 4, one T_x x T_y block = one length-256 sequence (Section 4): L = 16 and
// 16 x 16 blocks for the codes of Algorithms 1-3, L = 14 and 32 x 8 blocks for the
// lookup-only code.  It exists to
// produce valid code streams for tests and examples; it is never on a timed path.
//
// The dynamic program is arranged around the trellis' structure: every state y
// with the same top L-kV bits has the same 2^kV predecessors, so the minimum over
// predecessors is taken once per such prefix and shared by its 2^kV children,
// which brings a step down to O(2^L) work.
#include <atomic>
#include <cmath>
#include <cstdint>
#include <cstring>
#include <limits>
#include <thread>
#include <vector>

#include "qtip_internal.h"

namespace qtip {
namespace {

constexpr int T = 256;

float half_bits_to_float(uint16_t h) {
    _Float16 v;
    std::memcpy(&v, &h, 2);
    return (float)v;
}

// The codes on the host (Algorithms 1-3; code 4: a stored table; code 5: Algorithm 3 at
// V = 1), values as float.
void build_codebook(int L, int V, int code_id, const uint16_t *lut, std::vector<float> &C) {
    const int NS = 1 << L;
    C.resize((size_t)NS * V);
    for (uint32_t x = 0; x < (uint32_t)NS; x++) {
        if (code_id == 4) {
            C[x] = half_bits_to_float(lut[x]);
        } else if (code_id == 5) {  // Algorithm 3 with one entry per row, Q = 6
            uint32_t X = x * x + x;
            C[x] = half_bits_to_float((uint16_t)(lut[(X >> 9) & 63u] ^ (X & 0x8000u)));
        } else if (code_id == 0) {
            uint32_t X = x * 34038481u + 76625530u;
            int s = (int)(X & 255u) + (int)((X >> 8) & 255u) + (int)((X >> 16) & 255u) + (int)(X >> 24);
            C[x] = (float)(_Float16)((double)(s - 510) / 147.8);
        } else if (code_id == 1) {
            uint32_t X = x * 89226354u + 64248484u;
            uint32_t Y = (X & 0x8FFF8FFFu) ^ 0x3B603B60u;
            _Float16 sum = (_Float16)(half_bits_to_float((uint16_t)Y) + half_bits_to_float((uint16_t)(Y >> 16)));
            C[x] = (float)sum;
        } else {
            uint32_t X = x * x + x;
            uint32_t idx = (X >> 6) & 511u;
            uint16_t v0 = lut[2 * idx];
            uint16_t v1 = lut[2 * idx + 1];
            if (X & 0x8000u) v1 ^= 0x8000u;
            if (code_id == 3 && (X >> 31)) v0 ^= 0x8000u;  // the two-sign-flip form
            C[2 * (size_t)x] = half_bits_to_float(v0);
            C[2 * (size_t)x + 1] = half_bits_to_float(v1);
        }
    }
}

struct Workspace {
    std::vector<double> val, nxt;
    std::vector<uint8_t> back;  // [G][2^(L-kV)]: which predecessor won for each prefix
    std::vector<uint32_t> states;
};

// One Viterbi pass over `S` (T values).  first_top / last_low < 0 = unconstrained.
double viterbi(const float *S, int L, int k, int V, const float *C, int first_top, int last_low,
               Workspace &ws) {
    const int kV = k * V, ov = L - kV, G = T / V, NS = 1 << L;
    const int NP = 1 << ov, NC = 1 << kV;
    const double INF = std::numeric_limits<double>::infinity();
    ws.val.assign(NS, 0.0);
    ws.nxt.assign(NS, 0.0);
    ws.back.assign((size_t)G * NP, 0);
    ws.states.assign(G, 0);
    auto dist = [&](int y, int t) {
        double d = 0.0;
        for (int j = 0; j < V; j++) {
            double e = (double)C[(size_t)y * V + j] - (double)S[V * t + j];
            d += e * e;
        }
        return d;
    };
    for (int y = 0; y < NS; y++)
        ws.val[y] = (first_top >= 0 && (y >> kV) != first_top) ? INF : dist(y, 0);
    for (int t = 1; t < G; t++) {
        uint8_t *bk = &ws.back[(size_t)t * NP];
        for (int hi = 0; hi < NP; hi++) {
            double best = INF;
            int arg = 0;
            for (int p = 0; p < NC; p++) {
                double v = ws.val[(p << ov) | hi];
                if (v < best) {
                    best = v;
                    arg = p;
                }
            }
            bk[hi] = (uint8_t)arg;
            for (int c = 0; c < NC; c++) {
                int y = (hi << kV) | c;
                ws.nxt[y] = best + dist(y, t);
            }
        }
        ws.val.swap(ws.nxt);
    }
    double best = INF;
    int arg = 0;
    const int ovmask = NP - 1;
    for (int y = 0; y < NS; y++) {
        if (last_low >= 0 && (y & ovmask) != last_low) continue;
        if (ws.val[y] < best) {
            best = ws.val[y];
            arg = y;
        }
    }
    for (int t = G - 1; t >= 0; t--) {
        ws.states[t] = (uint32_t)arg;
        if (t > 0) arg = ((int)ws.back[(size_t)t * NP + (arg >> kV)] << ov) | (arg >> kV);
    }
    return best;
}

// Algorithm 4 on one sequence; writes 8k words, returns the squared error.
double quantize_sequence(const float *S, int L, int k, int V, const float *C, uint32_t *words,
                         Workspace &ws) {
    const int kV = k * V, ov = L - kV, G = T / V;
    float Sr[T];
    for (int i = 0; i < T; i++) Sr[(i + T / 2) % T] = S[i];
    viterbi(Sr, L, k, V, C, -1, -1, ws);
    const int O = (int)(ws.states[(T / 2) / V - 1] & ((1u << ov) - 1u));
    const double d = viterbi(S, L, k, V, C, O, O, ws);
    std::memset(words, 0, sizeof(uint32_t) * 8 * k);
    for (int t = 0; t < G; t++) {
        const uint32_t top = ws.states[t] >> ov;  // the kV new bits of this step
        for (int i = 0; i < kV; i++) {
            const int pos = t * kV + i;
            if ((top >> (kV - 1 - i)) & 1u) words[pos >> 5] |= 1u << (31 - (pos & 31));
        }
    }
    return d;
}

}  // namespace

int quantize_host(const float *W, int m, int n, int L, int k, int V, int code_id, const uint16_t *lut,
                  uint32_t *codes_out, double *mse_out) {
    std::vector<float> C;
    build_codebook(L, V, code_id, lut, C);
    const int tx = code_id == 4 ? 32 : 16, ty = T / tx;  // the block that is one sequence
    const int tm = m / tx, tn = n / ty;
    const long ntiles = (long)tm * tn;
    unsigned nthreads = std::thread::hardware_concurrency();
    if (nthreads == 0) nthreads = 1;
    if ((long)nthreads > ntiles) nthreads = (unsigned)ntiles;
    std::atomic<long> next(0);
    std::vector<double> err(nthreads, 0.0);
    std::atomic<bool> failed(false);
    auto worker = [&](unsigned id) {
        try {
            Workspace ws;
            float S[T];
            for (;;) {
                const long tile = next.fetch_add(1);
                if (tile >= ntiles) break;
                const long I = tile / tn, J = tile % tn;
                for (int s = 0; s < T; s++)
                    S[s] = W[(size_t)(tx * I + s / ty) * n + (ty * J + s % ty)];
                err[id] += quantize_sequence(S, L, k, V, C.data(), codes_out + (size_t)tile * 8 * k, ws);
            }
        } catch (...) {
            failed = true;
        }
    };
    std::vector<std::thread> pool;
    for (unsigned i = 1; i < nthreads; i++) pool.emplace_back(worker, i);
    worker(0);
    for (auto &th : pool) th.join();
    if (failed) return -1;
    if (mse_out) {
        double tot = 0.0;
        for (double e : err) tot += e;
        *mse_out = tot / ((double)m * n);
    }
    return 0;
}

}  // namespace qtip
